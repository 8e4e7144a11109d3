// select_path kernel for gfx950: one workgroup per prompt.
//
// SEQUENTIAL (Alg. 2 as printed): wave 0 holds the per-node scalars of the whole tree in registers
// (one node per lane per 64-node chunk).  The children of the current node are found with one
// ballot per chunk, and the serial budget / acceptance arithmetic of the tried children runs on
// values fetched with readlane, so a level costs no memory access at all.
// LONGEST: the same rule along every root-to-leaf path on its own is a top-down recurrence
// (state of a node = f(state of its parent)); it is evaluated level by level in LDS, then the
// best leaf is picked with an integer atomic max.
// Both end with Alg. 1's correction step: inverse CDF over the terminal node's filtered softmax
// with the rejected tokens removed, as per-256-entry chunk sums, a scan over the chunk sums and
// a scan inside the crossing chunk.
#include "common.h"

namespace {

constexpr int MAXCHUNKS = CASCADE_MAX_VOCAB / 256;

__device__ __forceinline__ float readlane_f(float v, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

struct Try {
  bool pass;
  float tvd;
};
// Alg. 2 body for one tried node: budget-gated aggregation (a mass of 0 changes nothing, so the set
// sizes need not be consulted), then Alg. 1's test r * p < q
__device__ __forceinline__ Try try_node(float q, float mi, float mc, float up, float tvd, float eps) {
  if (tvd + mi <= eps) { q += mi; tvd += mi; }
  if (tvd + mc <= eps) { q += mc; tvd += mc; }
  Try r;
  r.pass = up < q;
  r.tvd = tvd;
  return r;
}

// NT = threads; TCH = 64-node chunks of the tree held in registers by the walking wave
// (Tn <= 64 * TCH); CPW = 256-entry vocabulary chunks each wave keeps in registers
// (V <= 256 * (NT / 64) * CPW)
template <int NT, int TCH, int CPW>
__global__ __launch_bounds__(NT) void select_kernel(select_args a, int* dev_status) {
  constexpr int SEL_THREADS = NT, SEL_WAVES = NT / 64;
  __shared__ int s_path[CASCADE_MAX_DEPTH];
  __shared__ int s_tried[CASCADE_MAX_WIDTH];
  __shared__ int s_len, s_cur, s_ntried, s_best;
  __shared__ float s_tvd;
  __shared__ float s_chunk[MAXCHUNKS];
  __shared__ float s_total, s_base;
  __shared__ int s_cstar, s_lastkept;
  // LONGEST only
  __shared__ int s_par[CASCADE_MAX_TREE];
  __shared__ float s_ntvd[CASCADE_MAX_TREE];
  __shared__ unsigned char s_alive[CASCADE_MAX_TREE], s_ready[CASCADE_MAX_TREE], s_depth[CASCADE_MAX_TREE], s_haschild[CASCADE_MAX_TREE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const int lo = a.node_off[b], Tn = min(a.node_off[b + 1] - lo, 64 * TCH);
  // a tree larger than the launch was sized for is walked over its first 64 * TCH nodes only, and flagged
  if (tid == 0 && a.node_off[b + 1] - lo > 64 * TCH) atomicOr(dev_status, CASCADE_FLAG_TREE_SIZE);
  const int maxd = min(a.max_depth, CASCADE_MAX_DEPTH);
  const float eps = a.eps_tvd;

  if (a.mode == CASCADE_WALK_SEQUENTIAL) {
    if (wave == 0) {
      const int nch = (Tn + 63) >> 6;
      int par[TCH], tok[TCH];
      float qv[TCH], mi[TCH], mc[TCH], up[TCH];
#pragma unroll
      for (int c = 0; c < TCH; ++c) {
        const int j = c * 64 + lane;
        par[c] = -2; tok[c] = -1; qv[c] = 0.f; mi[c] = 0.f; mc[c] = 0.f; up[c] = 0.f;
        if (c < nch && j < Tn) {
          par[c] = a.parent[lo + j];
          tok[c] = a.token[lo + j];
          qv[c] = a.q_tok[lo + j];
          mi[c] = a.m_int[lo + j];
          mc[c] = a.m_conv[lo + j];
          up[c] = a.u[lo + j] * (a.draft_prob ? a.draft_prob[lo + j] : 1.f);
        }
      }
      int cur = 0, len = 0, ntried = 0;
      float tvd = 0.f;
      while (true) {
        int accepted = -1;
        ntried = 0;
#pragma unroll
        for (int c = 0; c < TCH; ++c) {
          if (c < nch && accepted < 0) {
            const int j = c * 64 + lane;
            unsigned long long kids = __ballot(par[c] == cur && j > cur);
            while (kids) {
              const int l = __ffsll((long long)kids) - 1;
              kids &= kids - 1;
              const Try r = try_node(readlane_f(qv[c], l), readlane_f(mi[c], l), readlane_f(mc[c], l),
                                     readlane_f(up[c], l), tvd, eps);
              tvd = r.tvd;
              if (r.pass) { accepted = c * 64 + l; break; }
              const int tt = __builtin_amdgcn_readlane(tok[c], l);
              if (ntried < CASCADE_MAX_WIDTH) { if (lane == 0) s_tried[ntried] = tt; ++ntried; }
              else if (lane == 0) atomicOr(dev_status, CASCADE_FLAG_WIDTH);
            }
          }
        }
        if (accepted < 0) break;
        if (len >= maxd) { if (lane == 0) atomicOr(dev_status, CASCADE_FLAG_DEPTH); break; }
        if (lane == 0) s_path[len] = accepted;
        ++len;
        cur = accepted;
      }
      if (lane == 0) { s_len = len; s_cur = cur; s_ntried = ntried; s_tvd = tvd; }
    }
  } else {
    // top-down recurrence over the tree, one level per round
    for (int i = tid; i < Tn; i += SEL_THREADS) {
      int pi = a.parent[lo + i];
      if (i == 0) pi = -1;
      else if (pi < 0 || pi >= i) { atomicOr(dev_status, CASCADE_FLAG_PARENT); pi = -1; }   // orphan: never reached
      s_par[i] = pi;
      s_alive[i] = i == 0;
      s_ready[i] = i == 0;
      s_depth[i] = 0;
      s_ntvd[i] = 0.f;
      s_haschild[i] = 0;
    }
    if (tid == 0) s_best = -1;
    __syncthreads();
    for (int i = tid; i < Tn; i += SEL_THREADS)
      if (s_par[i] >= 0) s_haschild[s_par[i]] = 1;
    for (int round = 0; round < maxd; ++round) {
      bool can[(CASCADE_MAX_TREE + SEL_THREADS - 1) / SEL_THREADS];
#pragma unroll
      for (int k = 0; k < (CASCADE_MAX_TREE + SEL_THREADS - 1) / SEL_THREADS; ++k) {
        const int i = tid + k * SEL_THREADS;
        can[k] = i < Tn && !s_ready[i] && s_par[i] >= 0 && s_ready[s_par[i]];
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < (CASCADE_MAX_TREE + SEL_THREADS - 1) / SEL_THREADS; ++k) {
        const int i = tid + k * SEL_THREADS;
        if (can[k]) {
          const int pi = s_par[i];
          float t = s_ntvd[pi];
          bool alive = false;
          if (s_alive[pi]) {
            const float up = a.u[lo + i] * (a.draft_prob ? a.draft_prob[lo + i] : 1.f);
            const Try r = try_node(a.q_tok[lo + i], a.m_int[lo + i], a.m_conv[lo + i], up, t, eps);
            t = r.tvd;
            alive = r.pass;
          }
          s_ntvd[i] = t;
          s_alive[i] = alive;
          s_depth[i] = s_depth[pi] + 1;
          s_ready[i] = 1;
        }
      }
      __syncthreads();
    }
    // every leaf: deepest accepted node on its chain; best = longest, ties to the smallest leaf index
    for (int i = tid; i < Tn; i += SEL_THREADS) {
      if (!s_ready[i] && s_par[i] >= 0) atomicOr(dev_status, CASCADE_FLAG_DEPTH);
      if (!s_haschild[i]) {
        int x = i;
        while (x >= 0 && !s_alive[x]) x = s_par[x];   // parents have smaller indices: ends at the root, or at -1 under an orphan
        if (x >= 0) atomicMax(&s_best, (int)s_depth[x] * CASCADE_MAX_TREE + (CASCADE_MAX_TREE - 1 - i));
      }
    }
    __syncthreads();
    if (tid == 0) {
      const int best = max(s_best, CASCADE_MAX_TREE - 1);   // no usable leaf (bad parent array): root only
      const int leaf = CASCADE_MAX_TREE - 1 - (best % CASCADE_MAX_TREE);
      int x = leaf, first_dead = -1;
      while (x > 0 && !s_alive[x]) { first_dead = x; x = s_par[x]; }
      if (x < 0) { x = 0; first_dead = -1; }
      const int len = s_depth[x];
      s_len = len;
      s_cur = x;
      s_tvd = first_dead >= 0 ? s_ntvd[first_dead] : s_ntvd[x];
      s_ntried = first_dead >= 0 ? 1 : 0;
      if (first_dead >= 0) s_tried[0] = a.token[lo + first_dead];
      for (int d = len - 1, y = x; d >= 0; --d) { s_path[d] = y; y = s_par[y]; }
    }
  }
  __syncthreads();

  // ---- correction / bonus token: inverse CDF over the terminal node's distribution
  const int len = s_len, cur = s_cur, ntried = s_ntried;
  const int V = a.vocab;
  const float* Lr = a.logits + (int64_t)(lo + cur) * V;
  const float thr = a.row_thr[lo + cur], lse = a.row_lse[lo + cur];
  const int nchunks = (V + 255) >> 8;
  const bool vec = (V & 3) == 0;
  const float ub = a.u_bonus[b];

  // every wave owns the chunks wave, wave + NW, ...; their logits are loaded in batches of 8 chunks
  // (all loads of a batch in flight together).  With a single batch (CPW == 8) the registers are
  // kept, and the crossing chunk is later resolved by its owner without a second trip to memory.
  constexpr int NBATCH = CPW / 8;
  auto load_chunk = [&](int c) -> f32x4 {
    const int e0 = c * 256 + lane * 4;
    f32x4 v = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    if (c < nchunks) {
      if (vec && e0 + 3 < V) {
        v = *(const f32x4*)(Lr + e0);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) if (e0 + i < V) v[i] = Lr[e0 + i];
      }
    }
    return v;
  };
  f32x4 gv[8];
  if (NBATCH == 1) {
#pragma unroll
    for (int ci = 0; ci < 8; ++ci) gv[ci] = load_chunk(wave + SEL_WAVES * ci);
  }
  // masses of the 4 entries a lane owns inside chunk c
  // lane e holds the e-th rejected token; chunk_vals visits them with readlane (no LDS in the loop)
  const int tried_reg = lane < ntried ? s_tried[lane] : -1;
  auto chunk_vals = [&](int c, const f32x4& g4, bool use_ban, float r[4]) {
    const int e0 = c * 256 + lane * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = (g4[i] >= thr && e0 + i < V) ? __expf(g4[i] - lse) : 0.f;
    if (use_ban) {
      for (int e = 0; e < ntried; ++e) {
        const int t = __builtin_amdgcn_readlane(tried_reg, e);
        if ((t >> 8) == c && lane == ((t & 255) >> 2)) {
#pragma unroll
          for (int i = 0; i < 4; ++i) if ((t & 3) == i) r[i] = 0.f;
        }
      }
    }
  };

  bool use_ban = true;
  for (int attempt = 0; attempt < 2; ++attempt) {
    for (int bt = 0; bt < NBATCH; ++bt) {
      if (NBATCH > 1) {
#pragma unroll
        for (int ci = 0; ci < 8; ++ci) gv[ci] = load_chunk(wave + SEL_WAVES * (8 * bt + ci));
      }
#pragma unroll
      for (int ci = 0; ci < 8; ++ci) {
        const int c = wave + SEL_WAVES * (8 * bt + ci);
        if (c < nchunks) {
          float r[4];
          chunk_vals(c, gv[ci], use_ban, r);
          const float cs = wave_sum(((r[0] + r[1]) + r[2]) + r[3]);
          if (lane == 0) s_chunk[c] = cs;
        }
      }
    }
    __syncthreads();
    if (wave == 0) {
      // lane l owns chunks 4l .. 4l+3
      float cs[4], loc = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        cs[i] = 4 * lane + i < nchunks ? s_chunk[4 * lane + i] : 0.f;
        loc += cs[i];
      }
      const float incl = wave_scan_incl_f(loc);
      const float total = readlane_f(incl, 63);
      const float target = ub * total;
      float run = incl - loc;
      int cand = 0x7fffffff;
      float cbase = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (cand == 0x7fffffff && cs[i] > 0.f && run + cs[i] > target) { cand = 4 * lane + i; cbase = run; }
        run += cs[i];
      }
      const int best = wave_min_i(cand);
      if (best == 0x7fffffff) {
        // rounding kept the running sum at or below the target: take the last chunk that holds mass
        int lastc = -1;
#pragma unroll
        for (int i = 0; i < 4; ++i) if (cs[i] > 0.f) lastc = 4 * lane + i;
        lastc = wave_max_i(lastc);
        if (lane == 0) { s_cstar = lastc; s_base = 0.f; s_lastkept = 1; }
      } else if (cand == best) {
        s_cstar = best;
        s_base = cbase;
        s_lastkept = 0;
      }
      if (lane == 0) s_total = total;
    }
    __syncthreads();
    if (s_total > 0.f || attempt == 1) break;
    use_ban = false;   // every kept entry was removed: fall back to the unfiltered row
    __syncthreads();
  }

  {
    const int cstar = s_cstar;
    const bool ok = s_total > 0.f && cstar >= 0;
    if (!ok && tid == 0) a.emitted[(int64_t)b * (a.max_depth + 1) + len] = -1;
#pragma unroll
    for (int ci = 0; ci < 8; ++ci) {
      // the owner of the crossing chunk finishes (kept registers, or one reload when there were several batches)
      if (ok && (NBATCH == 1 ? wave + SEL_WAVES * ci == cstar : (ci == 0 && wave == cstar % SEL_WAVES))) {
        const float target = ub * s_total;
        float r[4];
        const f32x4 g4 = NBATCH == 1 ? gv[ci] : load_chunk(cstar);
        chunk_vals(cstar, g4, use_ban, r);
        const float p0 = r[0], p1 = p0 + r[1], p2 = p1 + r[2], p3 = p2 + r[3];
        const float incl = wave_scan_incl_f(p3);
        const float run = s_base + (incl - p3);
        int cand = 0x7fffffff;
        const int e0 = cstar * 256 + lane * 4;
        if (!s_lastkept) {
          if (r[0] > 0.f && run + p0 > target) cand = e0;
          else if (r[1] > 0.f && run + p1 > target) cand = e0 + 1;
          else if (r[2] > 0.f && run + p2 > target) cand = e0 + 2;
          else if (r[3] > 0.f && run + p3 > target) cand = e0 + 3;
        }
        const int best = wave_min_i(cand);
        int x = best;
        if (best == 0x7fffffff) {
          int last = -1;
#pragma unroll
          for (int i = 0; i < 4; ++i) if (r[i] > 0.f) last = e0 + i;
          x = wave_max_i(last);
        }
        if (lane == 0) a.emitted[(int64_t)b * (a.max_depth + 1) + len] = x;
      }
    }
  }
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

hipError_t launch_select(cascade_ctx* ctx, const select_args* a) {
  KernelTimer t(ctx, CASCADE_K_SELECT);
  const bool small_tree = ctx->lim.max_nodes_per_tree <= 256, small_vocab = a->vocab <= 16384;
  dim3 grid(a->n_prompts);
  if (small_tree && small_vocab) CASCADE_TIMED_LAUNCH(t, (select_kernel<512, 4, 8>), grid, dim3(512), 0, ctx->stream, *a, ctx->dev_status);
  else if (small_tree) CASCADE_TIMED_LAUNCH(t, (select_kernel<1024, 4, 16>), grid, dim3(1024), 0, ctx->stream, *a, ctx->dev_status);
  else if (small_vocab) CASCADE_TIMED_LAUNCH(t, (select_kernel<512, 16, 8>), grid, dim3(512), 0, ctx->stream, *a, ctx->dev_status);
  else CASCADE_TIMED_LAUNCH(t, (select_kernel<1024, 16, 16>), grid, dim3(1024), 0, ctx->stream, *a, ctx->dev_status);
  return hipGetLastError();
}
