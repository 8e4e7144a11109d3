// cascade_accept kernels for gfx950 (Sec. 4.1 cosine similarity of target hidden states; Eq. 1
// interchangeable set; Eq. 2 convergence set; Eq. 3 aggregated mass).
//
// Kernel 1, one workgroup per parent node p: the Gram matrix of the rows [F_p, F_child_1 ..
// F_child_k] gives every cosine the children of p need at once — sibling/sibling (Eq. 1) and
// parent/child (Eq. 2).  For bf16 hidden states it is a dense contraction and runs on
// v_mfma_f32_16x16x32_bf16 (16 x 16 row blocks, operands loaded straight from global memory as
// 16-byte k-contiguous pieces); for f32 it is plain wave-wide dot products.  The workgroup then
// forms I_a for each child a, sums the mass of its distinct tokens under p's distribution, and
// writes q_tok, m_int, n_int, cos_parent and a 64-bit membership mask of I_a (by sibling rank).
// Kernel 2, one wavefront per node a: C_a from cos_parent of a's children, then m_conv over the
// distinct tokens not already counted (a's own token, tokens of I_a), and n_conv.
#include "common.h"

namespace {

constexpr int MAXW = CASCADE_MAX_WIDTH;   // children per node
constexpr int GN = MAXW + 1;              // rows of the Gram matrix: parent + children
constexpr int GP = GN + 1;                // LDS pitch

// probability of vocabulary entry t under a row's filtered softmax
__device__ __forceinline__ float prob_of(const float* logits_row, float thr, float lse, int t) {
  const float gv = logits_row[t];
  return gv >= thr ? __expf(gv - lse) : 0.f;
}

__device__ __forceinline__ float cos_from(float ab, float aa, float bb) {
  return (aa > 0.f && bb > 0.f) ? ab / (sqrtf(aa) * sqrtf(bb)) : 0.f;
}

__device__ __forceinline__ float dot_rows(const float* a, const float* b, int h, int lane) {
  float s = 0.f;
  for (int k = lane; k < h; k += 64) s = fmaf(a[k], b[k], s);
  return wave_sum(s);
}
__device__ __forceinline__ float dot_rows(const uint16_t* a, const uint16_t* b, int h, int lane) {
  float s = 0.f;
  for (int k = lane * 8; k < h; k += 64 * 8) {   // h is a multiple of 8
    const uint4 ua = *(const uint4*)(a + k), ub = *(const uint4*)(b + k);
    const uint32_t wa[4] = {ua.x, ua.y, ua.z, ua.w}, wb[4] = {ub.x, ub.y, ub.z, ub.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s = fmaf(__uint_as_float(wa[i] << 16), __uint_as_float(wb[i] << 16), s);
      s = fmaf(__uint_as_float(wa[i] & 0xffff0000u), __uint_as_float(wb[i] & 0xffff0000u), s);
    }
  }
  return wave_sum(s);
}

union Frag8 {
  bf16x8 v;
  uint4 u;
};

// C[16x16] += A[16 rows][k] * B[16 rows][k]^T over k in [k0, k1), (k1 - k0) a multiple of 32;
// rowa / rowb are this lane's row pointers, g its 8-wide k group
__device__ __forceinline__ f32x4 gram_tile(const uint16_t* rowa, const uint16_t* rowb, bool same, int k0, int k1, int g) {
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  int k = k0;
  for (; k + 128 <= k1; k += 128) {   // 4 MFMA steps per iteration, loads issued together
    Frag8 fa[4], fb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) fa[s].u = *(const uint4*)(rowa + k + 32 * s + 8 * g);
#pragma unroll
    for (int s = 0; s < 4; ++s) fb[s].u = same ? fa[s].u : *(const uint4*)(rowb + k + 32 * s + 8 * g);
#pragma unroll
    for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[s].v, fb[s].v, acc, 0, 0, 0);
  }
  for (; k < k1; k += 32) {
    Frag8 fa, fb;
    fa.u = *(const uint4*)(rowa + k + 8 * g);
    fb.u = same ? fa.u : *(const uint4*)(rowb + k + 8 * g);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa.v, fb.v, acc, 0, 0, 0);
  }
  return acc;
}

template <typename T>
__global__ __launch_bounds__(256) void accept_gram_kernel(accept_args a, unsigned long long* imask, int* dev_status) {
  __shared__ float gfull[GN * GP];        // Gram matrix; for MFMA tiles only blocks (bi <= bj) are filled
  __shared__ float gq[4][256];            // K-quarter partial tiles when there is a single 16 x 16 block
  __shared__ int s_child[MAXW];
  __shared__ int s_tok[MAXW];
  __shared__ int s_k;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.y, p = blockIdx.x;
  const int lo = a.node_off[b], Tn = a.node_off[b + 1] - lo;
  if (p >= Tn) return;
  const int h = a.hidden;
  const T* H = (const T*)a.h_cond;

  if (wave == 0) {   // ordered list of p's children
    int k = 0;
    for (int base = (p + 1) & ~63; base < Tn; base += 64) {
      const int j = base + lane;
      const bool is = j < Tn && j > p && a.parent[lo + j] == p;
      const unsigned long long m = __ballot(is);
      if (is) {
        const int idx = k + __popcll(m & ((1ull << lane) - 1ull));
        if (idx < MAXW) { s_child[idx] = j; s_tok[idx] = a.token[lo + j]; }
      }
      k += __popcll(m);
    }
    if (k > MAXW) {
      if (lane == 0) atomicOr(dev_status, CASCADE_FLAG_WIDTH);
      k = MAXW;
    }
    if (lane == 0) s_k = k;
  }
  __syncthreads();
  const int k = s_k;
  if (k == 0) return;
  const int n = k + 1, nb = (n + 15) >> 4;
  auto row_of = [&](int r) -> const T* { return H + (int64_t)(lo + (r == 0 ? p : s_child[r - 1])) * h; };

  bool mfma_done = false;
  if constexpr (sizeof(T) == 2) {
    if ((h & 127) == 0) {
      mfma_done = true;
      const int l16 = lane & 15, g = lane >> 4;
      if (nb == 1) {
        // one block: the four waves split the hidden dimension, partial tiles summed in a fixed order
        const uint16_t* ra = (const uint16_t*)row_of(min(l16, n - 1));
        const int kq = h / 4;   // a multiple of 32
        const f32x4 acc = gram_tile(ra, ra, true, wave * kq, (wave + 1) * kq, g);
#pragma unroll
        for (int r = 0; r < 4; ++r) gq[wave][(4 * g + r) * 16 + l16] = acc[r];
        __syncthreads();
        const int i = tid >> 4, j = tid & 15;
        if (i < n && j < n) gfull[i * GP + j] = ((gq[0][tid] + gq[1][tid]) + gq[2][tid]) + gq[3][tid];
      } else {
        // several blocks: block pairs (bi <= bj) are shared out over the waves, full hidden dimension each
        const int npairs = nb * (nb + 1) / 2;
        for (int pi = wave; pi < npairs; pi += 4) {
          int bi = 0, rem = pi;
          while (rem >= nb - bi) { rem -= nb - bi; ++bi; }
          const int bj = bi + rem;
          const uint16_t* ra = (const uint16_t*)row_of(min(16 * bi + l16, n - 1));
          const uint16_t* rb = (const uint16_t*)row_of(min(16 * bj + l16, n - 1));
          const f32x4 acc = gram_tile(ra, rb, bi == bj, 0, h, g);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int i = 16 * bi + 4 * g + r, j = 16 * bj + l16;
            if (i < n && j < n) gfull[i * GP + j] = acc[r];
          }
        }
      }
    }
  }
  if (!mfma_done) {
    const int npairs = n * (n + 1) / 2;
    for (int pi = wave; pi < npairs; pi += 4) {
      int i = 0, rem = pi;
      while (rem >= n - i) { rem -= n - i; ++i; }
      const int j = i + rem;
      const float d = dot_rows(row_of(i), row_of(j), h, lane);
      if (lane == 0) { gfull[i * GP + j] = d; gfull[j * GP + i] = d; }
    }
  }
  __syncthreads();
  // entries (i, j) with i in a later 16-row block than j were produced as (j, i)
  auto G = [&](int i, int j) -> float { return ((i >> 4) > (j >> 4)) ? gfull[j * GP + i] : gfull[i * GP + j]; };

  const float* Lp = a.logits + (int64_t)(lo + p) * a.vocab;
  const float thr = a.row_thr[lo + p], lse = a.row_lse[lo + p];
  const float g00 = G(0, 0);
  for (int i = wave; i < k; i += 4) {   // child i is row i + 1
    const int node = s_child[i];
    const int ta = s_tok[i];
    const bool tok_ok = ta >= 0 && ta < a.vocab;
    const float gii = G(i + 1, i + 1);
    bool member = false;
    int tj = -1;
    if (lane < k && lane != i) {
      tj = s_tok[lane];
      member = cos_from(G(i + 1, lane + 1), gii, G(lane + 1, lane + 1)) >= a.tau_pos;
    }
    const unsigned long long mask = __ballot(member);
    float mass = 0.f;
    if (member && tj != ta && tj >= 0 && tj < a.vocab) {
      bool dup = false;
      for (unsigned long long m = mask & ((1ull << lane) - 1ull); m; m &= m - 1) dup |= (s_tok[__ffsll((long long)m) - 1] == tj);
      if (!dup) mass = prob_of(Lp, thr, lse, tj);
    }
    mass = wave_sum(mass);
    if (lane == 0) {
      if (!tok_ok) atomicOr(dev_status, CASCADE_FLAG_TOKEN);
      const int64_t gi = lo + node;
      a.q_tok[gi] = tok_ok ? prob_of(Lp, thr, lse, ta) : 0.f;
      a.m_int[gi] = mass;
      a.n_int[gi] = __popcll(mask);
      a.cos_parent[gi] = cos_from(G(0, i + 1), g00, gii);
      imask[gi] = mask;
    }
  }
}

__global__ __launch_bounds__(256) void accept_conv_kernel(accept_args a, const unsigned long long* imask, int* dev_status) {
  __shared__ int tok_i[4][MAXW];
  __shared__ int tok_c[4][MAXW];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.y;
  const int lo = a.node_off[b], Tn = a.node_off[b + 1] - lo;
  const int node = blockIdx.x * 4 + wave;
  if (node >= Tn) return;
  const int64_t gi = lo + node;
  const int par = a.parent[gi];
  if (node == 0 || par < 0 || par >= node) {
    // roots, and nodes whose parent pointer is unusable (no workgroup of kernel 1 owns them)
    if (lane == 0) {
      if (node > 0 || par != -1) atomicOr(dev_status, CASCADE_FLAG_PARENT);
      a.q_tok[gi] = 0.f; a.m_int[gi] = 0.f; a.cos_parent[gi] = 0.f; a.n_int[gi] = 0;
      a.m_conv[gi] = 0.f; a.n_conv[gi] = 0;
    }
    return;
  }
  const int ta = a.token[gi];
  const unsigned long long im = imask[gi];
  const int n_i = __popcll(im);
  int n_c = 0, rank = 0, myrank = -1;
  for (int base = 0; base < Tn; base += 64) {
    const int j = base + lane;
    const int pj = j < Tn ? a.parent[lo + j] : -2;
    // siblings in rank order (the rank counts every child of par, this node included)
    const bool sib = pj == par && j > par;
    const unsigned long long sm = __ballot(sib);
    if (sib) {
      const int r = rank + __popcll(sm & ((1ull << lane) - 1ull));
      // position inside I_a = number of member ranks below r
      if (r < MAXW && ((im >> r) & 1ull)) tok_i[wave][__popcll(im & ((1ull << r) - 1ull))] = a.token[lo + j];
    }
    if (node >= base && node < base + 64) myrank = rank + __popcll(sm & ((1ull << (node - base)) - 1ull));
    rank += __popcll(sm);
    // children of this node whose features stay close to it (Eq. 2)
    const bool conv = pj == node && j > node && a.cos_parent[lo + j] >= a.tau_seq;
    const unsigned long long cm = __ballot(conv);
    if (conv) {
      const int idx = n_c + __popcll(cm & ((1ull << lane) - 1ull));
      if (idx < MAXW) tok_c[wave][idx] = a.token[lo + j];
    }
    n_c += __popcll(cm);
  }
  if (myrank >= MAXW) {
    // beyond the width limit: kernel 1 did not list this node (already flagged there)
    if (lane == 0) {
      a.q_tok[gi] = 0.f; a.m_int[gi] = 0.f; a.cos_parent[gi] = 0.f; a.n_int[gi] = 0;
      a.m_conv[gi] = 0.f; a.n_conv[gi] = 0;
    }
    return;
  }
  if (n_c > MAXW) {
    if (lane == 0) atomicOr(dev_status, CASCADE_FLAG_WIDTH);
    n_c = MAXW;
  }
  __builtin_amdgcn_wave_barrier();
  __threadfence_block();
  const float* Lp = a.logits + (int64_t)(lo + par) * a.vocab;
  const float thr = a.row_thr[lo + par], lse = a.row_lse[lo + par];
  float mc = 0.f;
  if (lane < n_c) {
    const int t = tok_c[wave][lane];
    bool dup = (t == ta) || t < 0 || t >= a.vocab;
    for (int e = 0; e < n_i; ++e) dup |= (tok_i[wave][e] == t);
    for (int e = 0; e < lane; ++e) dup |= (tok_c[wave][e] == t);
    if (!dup) mc = prob_of(Lp, thr, lse, t);
  }
  mc = wave_sum(mc);
  if (lane == 0) {
    a.m_conv[gi] = mc;
    a.n_conv[gi] = n_c;
  }
}

}  // namespace

hipError_t launch_accept(cascade_ctx* ctx, const accept_args* a) {
  hipStream_t stream = ctx->stream;
  int* dev_status = ctx->dev_status;
  unsigned long long* imask = (unsigned long long*)ctx->imask_ws;
  KernelTimer t(ctx, CASCADE_K_ACCEPT);
  dim3 g1(ctx->lim.max_nodes_per_tree, a->n_prompts);
  if (a->h_dtype == CASCADE_BF16) hipLaunchKernelGGL(accept_gram_kernel<uint16_t>, g1, dim3(256), 0, stream, *a, imask, dev_status);
  else hipLaunchKernelGGL(accept_gram_kernel<float>, g1, dim3(256), 0, stream, *a, imask, dev_status);
  dim3 g2((ctx->lim.max_nodes_per_tree + 3) / 4, a->n_prompts);
  hipLaunchKernelGGL(accept_conv_kernel, g2, dim3(256), 0, stream, *a, imask, dev_status);
  return hipGetLastError();
}
