// cascade_accept kernel for gfx950 (Sec. 4.1 cosine similarity of target hidden states; Eq. 1
// interchangeable set; Eq. 2 convergence set; Eq. 3 aggregated mass).
//
// One workgroup per node a.  Everything a needs is the cosine of its own feature row against its
// parent, its siblings and its children: one row against at most 1 + 63 + 64 others.  The others
// are taken in blocks of 15; with a as the 16th row, one 16 x 16 Gram tile per block gives every
// a . x (row of a) and every |x|^2 (diagonal) at once.  For bf16 hidden states the tile runs on
// v_mfma_f32_16x16x32_bf16 with the four waves splitting the hidden dimension (operands loaded
// straight from global memory as 16-byte k-contiguous pieces); f32 rows (and logit-space
// similarity) use wave-wide dot products.  The probabilities of the siblings' and children's
// tokens under the parent's distribution are gathered while the rows are still in flight; the sets
// I_a and C_a, the distinct-token masses and all outputs then need only ballots and LDS.
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

// The same Gram tile of one row set with itself over NS k-steps, all of the lane's NS 16-byte pieces
// requested before the first multiplication (one round trip instead of NS / 4), side() issued
// behind them (loads return in order, so what side() requests arrives after the rows), four
// independent accumulator chains.
template <int NS, typename F>
__device__ __forceinline__ f32x4 gram_tile_deep(const uint16_t* row, int k0, int g, F&& side) {
  Frag8 f[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) f[s].u = *(const uint4*)(row + k0 + 32 * s + 8 * g);
  side();
  f32x4 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < NS; ++s) acc[s & 3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[s].v, f[s].v, acc[s & 3], 0, 0, 0);
  return (acc[0] + acc[1]) + (acc[2] + acc[3]);
}

// a . x and x . x in one pass (generic rows)
__device__ __forceinline__ void dot2_rows(const float* a, const float* x, int h, int lane, float& ax, float& xx) {
  float s = 0.f, t = 0.f;
  for (int k = lane; k < h; k += 64) {
    const float xv = x[k];
    s = fmaf(a[k], xv, s);
    t = fmaf(xv, xv, t);
  }
  ax = wave_sum(s);
  xx = wave_sum(t);
}
__device__ __forceinline__ void dot2_rows(const uint16_t* a, const uint16_t* x, int h, int lane, float& ax, float& xx) {
  float s = 0.f, t = 0.f;
  for (int k = lane * 8; k < h; k += 64 * 8) {   // h is a multiple of 8
    const uint4 ua = *(const uint4*)(a + k), ux = *(const uint4*)(x + k);
    const uint32_t wa[4] = {ua.x, ua.y, ua.z, ua.w}, wx[4] = {ux.x, ux.y, ux.z, ux.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float x0 = __uint_as_float(wx[i] << 16), x1 = __uint_as_float(wx[i] & 0xffff0000u);
      s = fmaf(__uint_as_float(wa[i] << 16), x0, s);
      s = fmaf(__uint_as_float(wa[i] & 0xffff0000u), x1, s);
      t = fmaf(x0, x0, t);
      t = fmaf(x1, x1, t);
    }
  }
  ax = wave_sum(s);
  xx = wave_sum(t);
}

constexpr int MAXO = 2 * MAXW;   // others of a node: parent + (siblings - 1) + children <= 1 + 63 + 64

template <typename T>
__global__ __launch_bounds__(256) void accept_node_kernel(accept_args a, int* dev_status) {
  __shared__ float gq[4][256];          // K-quarter partial Gram tiles
  __shared__ float s_cos[MAXO];         // cos(a, other)
  __shared__ int s_other[MAXO];         // node index of every other row: parent, siblings (without a), children
  __shared__ int s_stok[MAXW], s_ctok[MAXW];   // tokens of the siblings (by rank, a included) and of the children
  __shared__ int s_sib[MAXW], s_chl[MAXW];     // node indices of the siblings (by rank, a included) and of the children
  __shared__ float s_sq[MAXW], s_cq[MAXW];     // their probabilities under the parent's distribution
  __shared__ int s_ks, s_kc, s_rank;
  __shared__ float s_aa;                       // |a|^2 (generic path)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.y, node = blockIdx.x;
  const int lo = a.node_off[b], Tn = a.node_off[b + 1] - lo;
  if (node == 0 && Tn > (int)gridDim.x) {
    // the launch was sized for smaller trees: the nodes beyond it are flagged and written as zeros
    if (tid == 0) atomicOr(dev_status, CASCADE_FLAG_TREE_SIZE);
    for (int j = (int)gridDim.x + tid; j < Tn && lo + j < a.n_nodes_total; j += 256) {
      a.q_tok[lo + j] = 0.f; a.m_int[lo + j] = 0.f; a.cos_parent[lo + j] = 0.f; a.n_int[lo + j] = 0;
      a.m_conv[lo + j] = 0.f; a.n_conv[lo + j] = 0;
    }
  }
  if (node >= Tn) return;
  const int64_t gi = lo + node;
  // wave 0 scans the tree for siblings and children, SCAN chunks of 64 nodes per round trip; the first
  // SCAN chunks (parents and tokens) are requested here, before anything waits for this node's own parent
  // pointer
  constexpr int SCAN = 4;
  int pj0[SCAN], tk0[SCAN];
  auto request_chunks = [&](int base) {
#pragma unroll
    for (int c = 0; c < SCAN; ++c) {
      const int j = base + 64 * c + lane;
      pj0[c] = j < Tn ? a.parent[lo + j] : -2;
      tk0[c] = j < Tn ? a.token[lo + j] : -1;
    }
  };
  if (wave == 0) request_chunks(0);
  const int par = a.parent[gi];
  auto write_zero = [&]() {
    if (tid == 0) {
      a.q_tok[gi] = 0.f; a.m_int[gi] = 0.f; a.cos_parent[gi] = 0.f; a.n_int[gi] = 0;
      a.m_conv[gi] = 0.f; a.n_conv[gi] = 0;
    }
  };
  if (node == 0 || par < 0 || par >= node) {   // roots, and nodes whose parent pointer is unusable
    if (tid == 0 && (node > 0 || par != -1)) atomicOr(dev_status, CASCADE_FLAG_PARENT);
    write_zero();
    return;
  }
  const int h = a.hidden;
  const T* H = (const T*)a.h_cond;
  const float* Lp = a.logits + (int64_t)(lo + par) * a.vocab;
  const float thr = a.row_thr[lo + par], lse = a.row_lse[lo + par];

  if (wave == 0) {   // siblings (children of par, in index order, a included) and children of a
    int ks = 0, kc = 0, rank = -1;
    for (int base = 0; base < Tn; base += 64 * SCAN) {
      if (base > 0) request_chunks(base);
#pragma unroll
      for (int c = 0; c < SCAN; ++c) {
        if (base + 64 * c >= Tn) break;
        const int j = base + 64 * c + lane;
        const int pj = pj0[c], tk = tk0[c];
        const bool sib = pj == par && j > par;
        const unsigned long long sm = __ballot(sib);
        if (sib) {
          const int r = ks + __popcll(sm & ((1ull << lane) - 1ull));
          if (r < MAXW) {
            s_sib[r] = j;
            s_stok[r] = tk;
            // other index: parent is 0; siblings keep their rank order with a left out
            if (j != node) s_other[1 + r - (j > node ? 1 : 0)] = j;
          }
          if (j == node) rank = r;
        }
        ks += __popcll(sm);
        const bool ch = pj == node && j > node;
        const unsigned long long cm = __ballot(ch);
        if (ch) {
          const int r = kc + __popcll(cm & ((1ull << lane) - 1ull));
          if (r < MAXW) { s_chl[r] = j; s_ctok[r] = tk; }
        }
        kc += __popcll(cm);
      }
    }
    rank = wave_max_i(rank);
    if (ks > MAXW || kc > MAXW) {
      if (lane == 0) atomicOr(dev_status, CASCADE_FLAG_WIDTH);
      ks = min(ks, MAXW);
      kc = min(kc, MAXW);
    }
    if (lane == 0) { s_ks = ks; s_kc = kc; s_rank = rank; s_other[0] = par; }
  }
  __syncthreads();
  const int ks = s_ks, kc = s_kc, rank = s_rank;
  if (rank < 0 || rank >= MAXW) {   // beyond the width limit (flagged above): not verified
    write_zero();
    return;
  }
  const int n_sib = ks - 1;              // siblings without a
  const int n_other = 1 + n_sib + kc;
  if (tid < kc) s_other[1 + n_sib + tid] = s_chl[tid];   // the children come after the siblings
  __syncthreads();

  // tokens of the siblings (threads 0 .. ks-1) and of the children (threads 64 .. 64+kc-1), left in LDS by
  // the scan; their probabilities under the parent's distribution are gathered while the feature rows are in flight
  const bool own_sib = tid < ks, own_ch = tid >= 64 && tid < 64 + kc;
  int my_tok = -1;
  if (own_sib) my_tok = s_stok[tid];
  else if (own_ch) my_tok = s_ctok[tid - 64];
  float my_q = 0.f, my_logit = -INFINITY;
  const bool q_wanted = (own_sib || own_ch) && my_tok >= 0 && my_tok < a.vocab;
  auto request_q = [&]() {   // the load only; its value is turned into a probability later
    if (q_wanted) my_logit = Lp[my_tok];
  };
  auto finish_q = [&]() { my_q = (q_wanted && my_logit >= thr) ? __expf(my_logit - lse) : 0.f; };
  auto gather_q = [&]() { request_q(); finish_q(); };

  const T* row_a = H + (int64_t)gi * h;
  bool mfma_done = false;
  if constexpr (sizeof(T) == 2) {
    if ((h & 127) == 0) {
      mfma_done = true;
      const int l16 = lane & 15, g = lane >> 4;
      const int kq = h / 4;   // a multiple of 32
      for (int blk = 0; blk * 15 < n_other; ++blk) {
        // tile rows: 0 = a, 1..15 = others 15 blk .. 15 blk + 14 (clamped: extra rows repeat the last one)
        const int o = 15 * blk + l16 - 1;
        const uint16_t* ra = l16 == 0 ? (const uint16_t*)row_a
                                      : (const uint16_t*)(H + (int64_t)(lo + s_other[min(o, n_other - 1)]) * h);
        f32x4 acc;
        if (kq == 1024) {   // hidden = 4096: the whole quarter row in flight at once
          acc = gram_tile_deep<32>(ra, wave * kq, g, [&]() { if (blk == 0) request_q(); });
          if (blk == 0) finish_q();
        } else {
          acc = gram_tile(ra, ra, true, wave * kq, (wave + 1) * kq, g);
          if (blk == 0) gather_q();
        }
        if (blk > 0) __syncthreads();   // the previous block's partial tiles have been consumed
#pragma unroll
        for (int r = 0; r < 4; ++r) gq[wave][(4 * g + r) * 16 + l16] = acc[r];
        __syncthreads();
        if (tid >= 1 && tid < 16 && 15 * blk + tid - 1 < n_other) {
          // row 0 of the tile: a . x_j ; diagonal: |x_j|^2 ; entry (0, 0): |a|^2
          const int j = tid;
          const float ax = ((gq[0][j] + gq[1][j]) + gq[2][j]) + gq[3][j];
          const float xx = ((gq[0][17 * j] + gq[1][17 * j]) + gq[2][17 * j]) + gq[3][17 * j];
          const float aa = ((gq[0][0] + gq[1][0]) + gq[2][0]) + gq[3][0];
          s_cos[15 * blk + j - 1] = cos_from(ax, aa, xx);
        }
      }
    }
  }
  if (!mfma_done) {
    gather_q();
    if (wave == 0) {
      float aa, dummy;
      dot2_rows(row_a, row_a, h, lane, dummy, aa);
      if (lane == 0) s_aa = aa;
    }
    __syncthreads();
    for (int oi = wave; oi < n_other; oi += 4) {
      float ax, xx;
      dot2_rows(row_a, H + (int64_t)(lo + s_other[oi]) * h, h, lane, ax, xx);
      if (lane == 0) s_cos[oi] = cos_from(ax, s_aa, xx);
    }
  }
  if (own_sib) { s_stok[tid] = my_tok; s_sq[tid] = my_q; }
  else if (own_ch) { s_ctok[tid - 64] = my_tok; s_cq[tid - 64] = my_q; }
  __syncthreads();

  if (wave == 0) {
    const int ta = s_stok[rank];
    const bool tok_ok = ta >= 0 && ta < a.vocab;
    // I_a among the siblings, by rank (lane = rank)
    bool member = false;
    int tj = -1;
    if (lane < ks && lane != rank) {
      tj = s_stok[lane];
      member = s_cos[1 + lane - (lane > rank ? 1 : 0)] >= a.tau_pos;
    }
    const unsigned long long imask = __ballot(member);
    float mi = 0.f;
    if (member && tj != ta && tj >= 0 && tj < a.vocab) {
      bool dup = false;
      for (unsigned long long m = imask & ((1ull << lane) - 1ull); m; m &= m - 1) dup |= (s_stok[__ffsll((long long)m) - 1] == tj);
      if (!dup) mi = s_sq[lane];
    }
    mi = wave_sum(mi);
    // C_a among the children (lane = child rank)
    bool conv = false;
    int tc = -1;
    if (lane < kc) {
      tc = s_ctok[lane];
      conv = s_cos[1 + n_sib + lane] >= a.tau_seq;
    }
    const unsigned long long cmask = __ballot(conv);
    float mc = 0.f;
    if (conv && tc != ta && tc >= 0 && tc < a.vocab) {
      bool dup = false;
      for (unsigned long long m = imask; m; m &= m - 1) dup |= (s_stok[__ffsll((long long)m) - 1] == tc);
      for (unsigned long long m = cmask & ((1ull << lane) - 1ull); m; m &= m - 1) dup |= (s_ctok[__ffsll((long long)m) - 1] == tc);
      if (!dup) mc = s_cq[lane];
    }
    mc = wave_sum(mc);
    if (lane == 0) {
      if (!tok_ok) atomicOr(dev_status, CASCADE_FLAG_TOKEN);
      a.q_tok[gi] = tok_ok ? s_sq[rank] : 0.f;
      a.m_int[gi] = mi;
      a.n_int[gi] = __popcll(imask);
      a.m_conv[gi] = mc;
      a.n_conv[gi] = __popcll(cmask);
      a.cos_parent[gi] = s_cos[0];
    }
  }
}

}  // namespace

hipError_t launch_accept(cascade_ctx* ctx, const accept_args* a) {
  KernelTimer t(ctx, CASCADE_K_ACCEPT);
  dim3 grid(ctx->lim.max_nodes_per_tree, a->n_prompts);
  if (a->h_dtype == CASCADE_BF16) CASCADE_TIMED_LAUNCH(t, accept_node_kernel<uint16_t>, grid, dim3(256), 0, ctx->stream, *a, ctx->dev_status);
  else CASCADE_TIMED_LAUNCH(t, accept_node_kernel<float>, grid, dim3(256), 0, ctx->stream, *a, ctx->dev_status);
  return hipGetLastError();
}
