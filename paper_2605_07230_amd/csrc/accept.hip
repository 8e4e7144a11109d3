// cascade_accept and select_path kernels for gfx950.
//
// cascade_accept: one wavefront per tree node.  The wave finds the node's siblings and children
// by scanning the parent array with ballots, computes the cosine similarity of the target hidden
// states against each of them (Sec. 4.1), forms the interchangeable set (Eq. 1) and the
// convergent set (Eq. 2), and sums the probability mass their distinct tokens carry under the
// distribution that verifies the node (Eq. 3).
//
// select_path: one workgroup per prompt.  Wave 0 runs the serial walk of Alg. 2 over those
// scalars (budget-gated aggregation, then Alg. 1's test r*p < q); the workgroup then draws the
// correction / bonus token by inverse CDF over the terminal node's distribution with the
// rejected siblings' tokens removed.
#include "common.h"

namespace {

// probability of vocabulary entry t under a row's filtered softmax
__device__ __forceinline__ float prob_of(const float* logits_row, float thr, float lse, int t) {
  const float gv = logits_row[t];
  return gv >= thr ? __expf(gv - lse) : 0.f;
}

template <typename T>
struct DotAcc;

// dot(a,b), |b|^2 over one hidden-state row pair, whole wave cooperating
template <>
struct DotAcc<uint16_t> {
  static __device__ __forceinline__ void run(const uint16_t* a, const uint16_t* b, int h, int lane, float& ab, float& bb) {
    float s_ab = 0.f, s_bb = 0.f;
    for (int k = lane * 8; k < h; k += 64 * 8) {   // h is a multiple of 8
      const uint4 ua = *(const uint4*)(a + k), ub = *(const uint4*)(b + k);
      const uint32_t wa[4] = {ua.x, ua.y, ua.z, ua.w}, wb[4] = {ub.x, ub.y, ub.z, ub.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float a0 = __uint_as_float(wa[i] << 16), a1 = __uint_as_float(wa[i] & 0xffff0000u);
        const float b0 = __uint_as_float(wb[i] << 16), b1 = __uint_as_float(wb[i] & 0xffff0000u);
        s_ab = fmaf(a0, b0, s_ab);
        s_ab = fmaf(a1, b1, s_ab);
        s_bb = fmaf(b0, b0, s_bb);
        s_bb = fmaf(b1, b1, s_bb);
      }
    }
    ab = wave_sum(s_ab);
    bb = wave_sum(s_bb);
  }
};
template <>
struct DotAcc<float> {
  static __device__ __forceinline__ void run(const float* a, const float* b, int h, int lane, float& ab, float& bb) {
    float s_ab = 0.f, s_bb = 0.f;
    for (int k = lane; k < h; k += 64) {
      const float av = a[k], bv = b[k];
      s_ab = fmaf(av, bv, s_ab);
      s_bb = fmaf(bv, bv, s_bb);
    }
    ab = wave_sum(s_ab);
    bb = wave_sum(s_bb);
  }
};

__device__ __forceinline__ float cos_from(float ab, float aa, float bb) {
  return (aa > 0.f && bb > 0.f) ? ab / (sqrtf(aa) * sqrtf(bb)) : 0.f;
}

template <typename T>
__global__ __launch_bounds__(256) void accept_kernel(accept_args a, int* dev_status) {
  __shared__ int tok_i[4][CASCADE_MAX_WIDTH];
  __shared__ int tok_c[4][CASCADE_MAX_WIDTH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.y;
  const int lo = a.node_off[b], Tn = a.node_off[b + 1] - lo;
  const int node = blockIdx.x * 4 + wave;
  if (node >= Tn) return;
  const int64_t gi = lo + node;
  const int h = a.hidden;
  const T* H = (const T*)a.h_cond;
  int par = a.parent[gi];
  if (node == 0 || par < 0 || par >= node) {
    if (lane == 0) {
      if (node > 0 || par != -1) atomicOr(dev_status, CASCADE_FLAG_PARENT);
      a.q_tok[gi] = 0.f; a.m_int[gi] = 0.f; a.m_conv[gi] = 0.f; a.cos_parent[gi] = 0.f;
      a.n_int[gi] = 0; a.n_conv[gi] = 0;
    }
    return;
  }
  const int ta = a.token[gi];
  const bool tok_ok = ta >= 0 && ta < a.vocab;
  if (!tok_ok && lane == 0) atomicOr(dev_status, CASCADE_FLAG_TOKEN);
  const float* Lp = a.logits + (int64_t)(lo + par) * a.vocab;
  const float thr = a.row_thr[lo + par], lse = a.row_lse[lo + par];
  const T* Ha = H + gi * h;
  float aa, dummy;
  DotAcc<T>::run(Ha, Ha, h, lane, dummy, aa);
  float ab, bb;
  DotAcc<T>::run(Ha, H + (int64_t)(lo + par) * h, h, lane, ab, bb);
  const float cpar = cos_from(ab, aa, bb);

  int n_i = 0, n_c = 0;
  bool overflow = false;
  for (int base = 0; base < Tn; base += 64) {
    const int j = base + lane;
    const int pj = j < Tn ? a.parent[lo + j] : -2;
    unsigned long long sib = __ballot(pj == par && j != node);
    unsigned long long chi = __ballot(pj == node);
    while (sib) {
      const int bn = base + __ffsll((long long)sib) - 1;
      sib &= sib - 1;
      DotAcc<T>::run(Ha, H + (int64_t)(lo + bn) * h, h, lane, ab, bb);
      if (cos_from(ab, aa, bb) >= a.tau_pos) {
        if (n_i < CASCADE_MAX_WIDTH) { if (lane == 0) tok_i[wave][n_i] = a.token[lo + bn]; ++n_i; }
        else overflow = true;
      }
    }
    while (chi) {
      const int bn = base + __ffsll((long long)chi) - 1;
      chi &= chi - 1;
      DotAcc<T>::run(Ha, H + (int64_t)(lo + bn) * h, h, lane, ab, bb);
      if (cos_from(ab, aa, bb) >= a.tau_seq) {
        if (n_c < CASCADE_MAX_WIDTH) { if (lane == 0) tok_c[wave][n_c] = a.token[lo + bn]; ++n_c; }
        else overflow = true;
      }
    }
  }
  if (overflow && lane == 0) atomicOr(dev_status, CASCADE_FLAG_WIDTH);
  __builtin_amdgcn_wave_barrier();
  __threadfence_block();
  // masses over distinct token ids; lane idx owns member idx
  float mi = 0.f, mc = 0.f;
  if (lane < n_i) {
    const int t = tok_i[wave][lane];
    bool dup = (t == ta) || t < 0 || t >= a.vocab;
    for (int e = 0; e < lane; ++e) dup |= (tok_i[wave][e] == t);
    if (!dup) mi = prob_of(Lp, thr, lse, t);
  }
  if (lane < n_c) {
    const int t = tok_c[wave][lane];
    bool dup = (t == ta) || t < 0 || t >= a.vocab;
    for (int e = 0; e < n_i; ++e) dup |= (tok_i[wave][e] == t);
    for (int e = 0; e < lane; ++e) dup |= (tok_c[wave][e] == t);
    if (!dup) mc = prob_of(Lp, thr, lse, t);
  }
  mi = wave_sum(mi);
  mc = wave_sum(mc);
  if (lane == 0) {
    a.q_tok[gi] = tok_ok ? prob_of(Lp, thr, lse, ta) : 0.f;
    a.m_int[gi] = mi;
    a.m_conv[gi] = mc;
    a.cos_parent[gi] = cpar;
    a.n_int[gi] = n_i;
    a.n_conv[gi] = n_c;
  }
}

// ------------------------------------------------------------------------------- select_path
struct TryResult {
  bool pass;
  float tvd;
};
__device__ __forceinline__ TryResult try_node(const select_args& a, int64_t gi, float tvd) {
  float q = a.q_tok[gi];
  if (a.n_int[gi] > 0) {
    const float m = a.m_int[gi];
    if (tvd + m <= a.eps_tvd) { q += m; tvd += m; }
  }
  if (a.n_conv[gi] > 0) {
    const float m = a.m_conv[gi];
    if (tvd + m <= a.eps_tvd) { q += m; tvd += m; }
  }
  const float px = a.draft_prob ? a.draft_prob[gi] : 1.f;
  TryResult r;
  r.pass = a.u[gi] * px < q;
  r.tvd = tvd;
  return r;
}

constexpr int SEL_THREADS = 256;

__global__ __launch_bounds__(SEL_THREADS) void select_kernel(select_args a, int* dev_status) {
  __shared__ int s_path[CASCADE_MAX_DEPTH];
  __shared__ int s_best[CASCADE_MAX_DEPTH];
  __shared__ int s_tried[CASCADE_MAX_WIDTH];
  __shared__ unsigned char s_haschild[CASCADE_MAX_TREE];
  __shared__ int s_len, s_cur, s_ntried;
  __shared__ float s_tvd;
  __shared__ float s_seg[SEL_THREADS];
  __shared__ float s_total;
  __shared__ int s_pick;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const int lo = a.node_off[b], Tn = min(a.node_off[b + 1] - lo, CASCADE_MAX_TREE);
  const int maxd = min(a.max_depth, CASCADE_MAX_DEPTH);

  if (a.mode == CASCADE_WALK_LONGEST) {
    for (int i = tid; i < Tn; i += SEL_THREADS) s_haschild[i] = 0;
    __syncthreads();
    for (int i = tid; i < Tn; i += SEL_THREADS) {
      const int pi = a.parent[lo + i];
      if (i > 0 && pi >= 0 && pi < i) s_haschild[pi] = 1;
    }
    __syncthreads();
  }

  if (wave == 0) {
    int cur = 0, len = 0, ntried = 0;
    float tvd = 0.f;
    if (a.mode == CASCADE_WALK_SEQUENTIAL) {
      bool going = true;
      while (going) {
        int accepted = -1;
        ntried = 0;
        bool any_child = false;
        for (int base = 0; base < Tn && accepted < 0; base += 64) {
          const int j = base + lane;
          unsigned long long kids = __ballot(j > cur && j < Tn && a.parent[lo + j] == cur);
          while (kids) {
            const int c = base + __ffsll((long long)kids) - 1;
            kids &= kids - 1;
            any_child = true;
            const TryResult r = try_node(a, lo + c, tvd);
            tvd = r.tvd;
            if (r.pass) { accepted = c; break; }
            if (ntried < CASCADE_MAX_WIDTH) { if (lane == 0) s_tried[ntried] = a.token[lo + c]; ++ntried; }
            else if (lane == 0) atomicOr(dev_status, CASCADE_FLAG_WIDTH);
          }
        }
        (void)any_child;
        if (accepted < 0) break;
        if (len >= maxd) { if (lane == 0) atomicOr(dev_status, CASCADE_FLAG_DEPTH); break; }
        if (lane == 0) s_path[len] = accepted;
        ++len;
        cur = accepted;
      }
    } else {
      int best_len = -1, best_cur = 0, best_ntried = 0, best_tried_tok = -1;
      float best_tvd = 0.f;
      for (int leaf = 0; leaf < Tn; ++leaf) {
        if (s_haschild[leaf]) continue;
        // chain root -> leaf, climbed into s_path backwards (uniform across the wave)
        int depth = 0;
        for (int x = leaf; x > 0 && depth <= CASCADE_MAX_TREE; ) {
          const int px = a.parent[lo + x];
          ++depth;
          if (px < 0 || px >= x) break;
          x = px;
        }
        if (depth > maxd) { if (lane == 0) atomicOr(dev_status, CASCADE_FLAG_DEPTH); continue; }
        if (lane == 0) {
          int x = leaf;
          for (int d = depth - 1; d >= 0; --d) { s_path[d] = x; x = a.parent[lo + x]; }
        }
        __builtin_amdgcn_wave_barrier();
        __threadfence_block();
        float t = 0.f;
        int l = 0, c_cur = 0, nt = 0, tt = -1;
        for (int d = 0; d < depth; ++d) {
          const int c = s_path[d];
          const TryResult r = try_node(a, lo + c, t);
          t = r.tvd;
          if (!r.pass) { nt = 1; tt = a.token[lo + c]; break; }
          ++l;
          c_cur = c;
        }
        if (l > best_len) {
          best_len = l; best_cur = c_cur; best_ntried = nt; best_tried_tok = tt; best_tvd = t;
          if (lane == 0) for (int d = 0; d < l; ++d) s_best[d] = s_path[d];
        }
        __builtin_amdgcn_wave_barrier();
      }
      if (best_len < 0) best_len = 0;
      len = best_len; cur = best_cur; ntried = best_ntried; tvd = best_tvd;
      if (lane == 0) {
        for (int d = 0; d < len; ++d) s_path[d] = s_best[d];
        if (ntried) s_tried[0] = best_tried_tok;
      }
    }
    if (lane == 0) { s_len = len; s_cur = cur; s_ntried = ntried; s_tvd = tvd; }
  }
  __syncthreads();

  // correction / bonus token from the terminal node's distribution
  const int len = s_len, cur = s_cur, ntried = s_ntried;
  const int V = a.vocab;
  const float* Lr = a.logits + (int64_t)(lo + cur) * V;
  const float thr = a.row_thr[lo + cur], lse = a.row_lse[lo + cur];
  const int seg = (V + SEL_THREADS - 1) / SEL_THREADS;
  const int v_lo = tid * seg, v_hi = min(V, v_lo + seg);
  bool use_ban = true;
  for (int attempt = 0; attempt < 2; ++attempt) {
    float ssum = 0.f;
    for (int v = v_lo; v < v_hi; ++v) {
      const float gv = Lr[v];
      if (gv >= thr) {
        bool banned = false;
        if (use_ban) for (int e = 0; e < ntried; ++e) banned |= (s_tried[e] == v);
        if (!banned) ssum += __expf(gv - lse);
      }
    }
    s_seg[tid] = ssum;
    __syncthreads();
    if (tid == 0) {
      float tot = 0.f;
      for (int i = 0; i < SEL_THREADS; ++i) tot += s_seg[i];
      s_total = tot;
      s_pick = -1;
      if (tot > 0.f) {
        const float target = a.u_bonus[b] * tot;
        float run = 0.f;
        int pick = -1;
        for (int i = 0; i < SEL_THREADS; ++i) {
          if (run + s_seg[i] > target) { pick = i; break; }
          run += s_seg[i];
        }
        s_pick = pick;            // -1: never exceeded (rounding) -> last kept entry
        s_seg[0] = run;           // mass before the picked segment (s_seg[0] no longer needed: see below)
      }
    }
    __syncthreads();
    if (s_total > 0.f) break;
    use_ban = false;              // everything was removed: fall back to the unfiltered row
    __syncthreads();
  }
  const float total = s_total;
  const int pick = s_pick;
  // NOTE: s_seg[0] now holds the running mass before segment `pick` (written by thread 0 after
  // every read of s_seg in the scan above).
  if (pick >= 0 && tid == pick) {
    const float target = a.u_bonus[b] * total;
    float run = s_seg[0];
    int x = -1;
    for (int v = v_lo; v < v_hi; ++v) {
      const float gv = Lr[v];
      if (gv >= thr) {
        bool banned = false;
        if (use_ban) for (int e = 0; e < ntried; ++e) banned |= (s_tried[e] == v);
        if (!banned) {
          run += __expf(gv - lse);
          x = v;
          if (run > target) break;
        }
      }
    }
    a.emitted[(int64_t)b * (a.max_depth + 1) + len] = x;
  }
  if (pick < 0) {
    // fall-back: last kept, not banned entry of the row (block-wide max of candidate indices)
    int last = -1;
    for (int v = v_lo; v < v_hi; ++v) {
      const float gv = Lr[v];
      if (gv >= thr) {
        bool banned = false;
        if (use_ban) for (int e = 0; e < ntried; ++e) banned |= (s_tried[e] == v);
        if (!banned) last = v;
      }
    }
    __syncthreads();
    s_seg[tid] = (float)last;
    __syncthreads();
    if (tid == 0) {
      float m = -1.f;
      for (int i = 0; i < SEL_THREADS; ++i) m = fmaxf(m, s_seg[i]);
      a.emitted[(int64_t)b * (a.max_depth + 1) + len] = (int)m;
    }
  }
  // the rest of the outputs
  for (int d = tid; d < a.max_depth; d += SEL_THREADS)
    a.path_nodes[(int64_t)b * a.max_depth + d] = d < len ? s_path[d] : -1;
  for (int d = tid; d <= a.max_depth; d += SEL_THREADS) {
    if (d < len) a.emitted[(int64_t)b * (a.max_depth + 1) + d] = a.token[lo + s_path[d]];
    else if (d > len) a.emitted[(int64_t)b * (a.max_depth + 1) + d] = -1;
  }
  if (tid == 0) {
    a.accept_len[b] = len;
    a.terminal[b] = cur;
    a.tvd_used[b] = s_tvd;
  }
}

}  // namespace

hipError_t launch_accept(cascade_ctx* ctx, const accept_args* a) {
  hipStream_t stream = ctx->stream;
  int* dev_status = ctx->dev_status;
  dim3 grid((ctx->lim.max_nodes_per_tree + 3) / 4, a->n_prompts);
  KernelTimer t(ctx, CASCADE_K_ACCEPT);
  if (a->h_dtype == CASCADE_BF16) hipLaunchKernelGGL(accept_kernel<uint16_t>, grid, dim3(256), 0, stream, *a, dev_status);
  else hipLaunchKernelGGL(accept_kernel<float>, grid, dim3(256), 0, stream, *a, dev_status);
  return hipGetLastError();
}

hipError_t launch_select(cascade_ctx* ctx, const select_args* a) {
  hipStream_t stream = ctx->stream;
  int* dev_status = ctx->dev_status;
  KernelTimer t(ctx, CASCADE_K_SELECT);
  hipLaunchKernelGGL(select_kernel, dim3(a->n_prompts), dim3(SEL_THREADS), 0, stream, *a, dev_status);
  return hipGetLastError();
}
