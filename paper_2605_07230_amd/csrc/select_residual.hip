// select_path with full drafter distributions: the SEQUENTIAL walk of Alg. 2 in which every
// rejection replaces the verifying distribution f by Alg. 1's residual norm([f - p]_+) against the
// rejected node's drafter row, and the last token is drawn from what is left.
//
// One workgroup of 16 waves per prompt.  The verifying distribution lives in registers for the
// whole walk: wave w owns the vocabulary segment [w * SEG, (w + 1) * SEG), SEG = 256 * VQ, as VQ
// four-wide vectors per lane (entry = w * SEG + 256 * i + 4 * lane + c).  A rejection costs one
// coalesced read of the drafter row, a workgroup sum and a rescale; an acceptance one read of the
// new node's logits row.  All decisions are taken by every thread on the same broadcast scalars,
// so control flow stays uniform.  The inverse CDF at the end runs over the same registers.
#include "common.h"

namespace {

constexpr int NW = 16;

struct Try {
  bool pass;
  float tvd;
};
__device__ __forceinline__ Try try_node(float q, float mi, float mc, float up, float tvd, float eps) {
  if (tvd + mi <= eps) { q += mi; tvd += mi; }
  if (tvd + mc <= eps) { q += mc; tvd += mc; }
  Try r;
  r.pass = up < q;
  r.tvd = tvd;
  return r;
}

__device__ __forceinline__ float readlane_f(float v, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

// EXACT: vocab == 16 * SEG, every lane's entries exist (no clamping, plain immediate offsets)
template <int VQ, bool EXACT>
__global__ __launch_bounds__(1024) void select_residual_kernel(select_args a, int* dev_status) {
  constexpr int SEG = 256 * VQ;
  __shared__ int s_child[CASCADE_MAX_WIDTH];
  __shared__ int s_path[CASCADE_MAX_DEPTH];
  __shared__ int s_m, s_x;
  __shared__ float s_q;
  __shared__ float s_wsum[NW];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const int lo = a.node_off[b], Tn = min(a.node_off[b + 1] - lo, CASCADE_MAX_TREE);
  if (tid == 0 && a.node_off[b + 1] - lo > CASCADE_MAX_TREE) atomicOr(dev_status, CASCADE_FLAG_TREE_SIZE);
  const int V = a.vocab;   // a multiple of 4, at most 16 * SEG (checked by the host)
  const int maxd = min(a.max_depth, CASCADE_MAX_DEPTH);
  const float eps = a.eps_tvd;
  const int e_base = wave * SEG + lane * 4;

  f32x4 f[VQ];
  auto load_target = [&](int node) {
    const float* Lr = a.logits + (int64_t)(lo + node) * V;
    const float thr = a.row_thr[lo + node], lse = a.row_lse[lo + node];
#pragma unroll
    for (int i = 0; i < VQ; ++i) {
      const int e = e_base + 256 * i;
      const f32x4 g = *(const f32x4*)((const char*)Lr + 4u * (unsigned)(EXACT ? e : min(e, V - 4)));   // clamped: always in bounds, masked below
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float x = __expf(g[c] - lse);
        f[i][c] = ((EXACT || e < V) && g[c] >= thr) ? x : 0.f;
      }
      if ((i & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // at most four row loads in flight: registers
    }
  };

  int cur = 0, len = 0;
  float tvd = 0.f;
  load_target(0);
  while (true) {
    if (wave == 0) {   // ordered list of cur's children
      int k = 0;
      for (int base = (cur + 1) & ~63; base < Tn; base += 64) {
        const int j = base + lane;
        const bool is = j < Tn && j > cur && a.parent[lo + j] == cur;
        const unsigned long long m = __ballot(is);
        if (is) {
          const int idx = k + __popcll(m & ((1ull << lane) - 1ull));
          if (idx < CASCADE_MAX_WIDTH) s_child[idx] = j;
        }
        k += __popcll(m);
      }
      if (k > CASCADE_MAX_WIDTH) {
        if (lane == 0) atomicOr(dev_status, CASCADE_FLAG_WIDTH);
        k = CASCADE_MAX_WIDTH;
      }
      if (lane == 0) s_m = k;
    }
    __syncthreads();
    const int m = s_m;
    int accepted = -1;
    for (int j = 0; j < m; ++j) {
      const int ch = s_child[j];
      const int ta = a.token[lo + ch];
      const bool tok_ok = ta >= 0 && ta < V;
      const float* prow = a.draft_dist + (int64_t)(lo + ch) * V;
      if (tok_ok) {
        const int w_owner = ta / SEG, r = ta - w_owner * SEG;
        if (wave == w_owner && lane == ((r & 255) >> 2)) {
          float val = 0.f;
#pragma unroll
          for (int i = 0; i < VQ; ++i)
#pragma unroll
            for (int c = 0; c < 4; ++c)
              if ((r >> 8) == i && (r & 3) == c) val = f[i][c];
          s_q = val;
        }
      } else if (tid == 0) {
        atomicOr(dev_status, CASCADE_FLAG_TOKEN);
        s_q = 0.f;
      }
      __syncthreads();
      const float px = tok_ok ? prow[ta] : 1.f;
      const Try t = try_node(s_q, a.m_int[lo + ch], a.m_conv[lo + ch], a.u[lo + ch] * px, tvd, eps);
      tvd = t.tvd;
      if (t.pass) { accepted = ch; break; }
      // rejected: f <- norm([f - p]_+), kept as it is when nothing would be left.  Two passes over the
      // drafter row (the second one hits the cache) instead of a second register copy of f.
      float loc = 0.f;
#pragma unroll
      for (int i = 0; i < VQ; ++i) {
        const int e = e_base + 256 * i;
        f32x4 p4 = *(const f32x4*)((const char*)prow + 4u * (unsigned)(EXACT ? e : min(e, V - 4)));
        if (!EXACT && e >= V) p4 = f32x4{0.f, 0.f, 0.f, 0.f};   // f is 0 there as well
        loc += ((fmaxf(f[i][0] - p4[0], 0.f) + fmaxf(f[i][1] - p4[1], 0.f)) + fmaxf(f[i][2] - p4[2], 0.f)) +
               fmaxf(f[i][3] - p4[3], 0.f);
        if ((i & 3) == 3) __builtin_amdgcn_sched_barrier(0);
      }
      const float ws = wave_sum(loc);
      if (lane == 0) s_wsum[wave] = ws;
      __syncthreads();
      float Z = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) Z += s_wsum[w];
      if (Z > 0.f) {
        const float inv = 1.f / Z;
#pragma unroll
        for (int i = 0; i < VQ; ++i) {
          const int e = e_base + 256 * i;
          const f32x4 p4 = *(const f32x4*)((const char*)prow + 4u * (unsigned)(EXACT ? e : min(e, V - 4)));   // beyond V: f is 0 and stays 0
#pragma unroll
          for (int c = 0; c < 4; ++c) f[i][c] = fmaxf(f[i][c] - p4[c], 0.f) * inv;
          if ((i & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (accepted < 0) break;
    if (len >= maxd) {
      if (tid == 0) atomicOr(dev_status, CASCADE_FLAG_DEPTH);
      break;
    }
    if (tid == 0) s_path[len] = accepted;
    ++len;
    cur = accepted;
    load_target(cur);
  }
  __syncthreads();   // the last reads of s_wsum / s_q are done

  // ---- last token: inverse CDF over f, vocabulary order = (wave, i, lane, c)
  float cs[VQ], wt = 0.f;
#pragma unroll
  for (int i = 0; i < VQ; ++i) {
    cs[i] = wave_sum(((f[i][0] + f[i][1]) + f[i][2]) + f[i][3]);
    wt += cs[i];
  }
  if (lane == 0) s_wsum[wave] = wt;
  if (tid == 0) s_x = -1;
  __syncthreads();
  float total = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) total += s_wsum[w];
  const float target = a.u_bonus[b] * total;
  // the wave whose segment crosses the target; if rounding lets no segment cross, the last one with mass
  int wstar = -1, wlast = -1;
  float base = 0.f, run = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const float x = s_wsum[w];
    if (x > 0.f) wlast = w;
    if (wstar < 0 && x > 0.f && run + x > target) { wstar = w; base = run; }
    run += x;
  }
  const bool forced_last = wstar < 0;
  if (forced_last) wstar = wlast;
  if (total > 0.f && wave == wstar) {
    int x = 0x7fffffff, last = -1;
    float r0 = base;
    bool done = false;
#pragma unroll
    for (int i = 0; i < VQ; ++i) {
      const int e0 = e_base + 256 * i;
#pragma unroll
      for (int c = 0; c < 4; ++c) if (f[i][c] > 0.f) last = e0 + c;
      if (!done && !forced_last && cs[i] > 0.f && r0 + cs[i] > target) {
        const float p0 = f[i][0], p1 = p0 + f[i][1], p2 = p1 + f[i][2], p3 = p2 + f[i][3];
        const float incl = wave_scan_incl_f(p3);
        const float rl = r0 + (incl - p3);
        int cand = 0x7fffffff;
        if (f[i][0] > 0.f && rl + p0 > target) cand = e0;
        else if (f[i][1] > 0.f && rl + p1 > target) cand = e0 + 1;
        else if (f[i][2] > 0.f && rl + p2 > target) cand = e0 + 2;
        else if (f[i][3] > 0.f && rl + p3 > target) cand = e0 + 3;
        x = wave_min_i(cand);
        done = x != 0x7fffffff;   // rounding inside the chunk may leave no crossing: fall through to later chunks
      }
      if (!done) r0 += cs[i];
    }
    if (x == 0x7fffffff) x = wave_max_i(last);
    if (lane == 0) s_x = x;
  }
  __syncthreads();

  for (int d = tid; d < a.max_depth; d += 1024)
    a.path_nodes[(int64_t)b * a.max_depth + d] = d < len ? s_path[d] : -1;
  for (int d = tid; d <= a.max_depth; d += 1024) {
    int v = -1;
    if (d < len) v = a.token[lo + s_path[d]];
    else if (d == len) v = s_x;
    a.emitted[(int64_t)b * (a.max_depth + 1) + d] = v;
  }
  if (tid == 0) {
    a.accept_len[b] = len;
    a.terminal[b] = cur;
    a.tvd_used[b] = tvd;
  }
}

}  // namespace

hipError_t launch_select_residual(cascade_ctx* ctx, const select_args* a) {
  KernelTimer t(ctx, CASCADE_K_SELECT);
  dim3 grid(a->n_prompts);
  const int V = a->vocab;
#define CASCADE_LAUNCH_RESIDUAL(VQ, EX) \
  CASCADE_TIMED_LAUNCH(t, (select_residual_kernel<VQ, EX>), grid, dim3(1024), 0, ctx->stream, *a, ctx->dev_status)
  if (V <= 16 * 256) { if (V == 16 * 256) CASCADE_LAUNCH_RESIDUAL(1, true); else CASCADE_LAUNCH_RESIDUAL(1, false); }
  else if (V <= 16 * 1024) { if (V == 16 * 1024) CASCADE_LAUNCH_RESIDUAL(4, true); else CASCADE_LAUNCH_RESIDUAL(4, false); }
  else { if (V == 16 * 4096) CASCADE_LAUNCH_RESIDUAL(16, true); else CASCADE_LAUNCH_RESIDUAL(16, false); }
#undef CASCADE_LAUNCH_RESIDUAL
  return hipGetLastError();
}
