// tree_verify_attn kernels for gfx950.
//
// Every node of a row attends the row's prefix KV positions plus its ancestors in the drafted
// tree plus itself (Preliminaries: parallel target pass; tree decoding with a tree mask).
//
// bf16 path: one workgroup = (row, kv head, query super-block, kv split).  K and V tiles (64 keys) are
// both staged row-major ([key][d]) in LDS; the K operand of the score MFMA is read as 16-byte words, the
// V operand of the second MFMA through the transposing LDS read (ds_read_b64_tr_b16), so no tile is ever
// transposed in memory.  Scores are produced TRANSPOSED, S^T = K Q^T, with v_mfma_f32_16x16x32_bf16: a
// lane then owns one query column, so the online-softmax statistics are per-lane scalars and the
// probabilities are already laid out as the B operand of O^T = V^T P^T.  The ancestor mask of the 64
// tree keys of a tile is one 64-bit word per query, built in LDS by climbing parent pointers.  Four
// kernels share this scheme and differ in how work is cut: query rows split over waves (tiny batches),
// key groups inside the workgroup (small trees), 256 query rows per workgroup on a three-deep LDS ring
// filled by LDS-direct loads (large trees), and the double-buffered predecessor of the latter, which
// writes split-KV partials to the workspace for a small merge kernel when the keys must be split across
// workgroups to fill the GPU.
//
// f32 path: a plain one-workgroup-per-(node, head) kernel, used by the small fp32 configuration.
#include <type_traits>

#include "common.h"

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

struct AttnParams {
  const int32_t* node_off;
  const int32_t* parent;
  const int32_t* prefix_len;
  const void* q;
  const void* k_tree;
  const void* v_tree;
  const void* k_cache;
  const void* v_cache;
  int64_t sr, sh, sp;
  void* out;
  float* lse;
  float* ws_o;     // [n_split][N*Hq][D]
  float* ws_ml;    // [n_split][N*Hq][2]
  int* dev_status;
  int n_heads, n_kv_heads, group;
  int n_split, n_sb;
  int n_rows_total;  // N * Hq
  int max_tree;      // the host's bound on any row's node count (the grid was sized for it)
  float scale_log2e;
};

// ------------------------------------------------------------------------------------------ f32
// grid (N, Hq); 256 threads.  Keys are visited in chunks of 256 with a running max / sum.
template <int DMAX>
__global__ __launch_bounds__(256) void attn_f32_kernel(AttnParams p, int n_rows, int D) {
  __shared__ float qs[DMAX];
  __shared__ float sc[256];
  __shared__ int anc[CASCADE_MAX_DEPTH + 2];
  __shared__ float red[8];
  __shared__ int s_row, s_nanc;
  const int node = blockIdx.x, head = blockIdx.y, tid = threadIdx.x;
  const int kvh = head / p.group;
  if (tid == 0) {
    int s = 0;
    while (s + 1 < n_rows && p.node_off[s + 1] <= node) ++s;
    s_row = s;
    int lo = p.node_off[s];
    int i = node - lo, n = 0;
    while (i >= 0 && n < CASCADE_MAX_DEPTH + 1) {
      anc[n++] = i;
      int pi = p.parent[lo + i];
      if (pi >= i) { atomicOr(p.dev_status, CASCADE_FLAG_PARENT); break; }
      i = pi;
    }
    if (i >= 0 && n == CASCADE_MAX_DEPTH + 1) atomicOr(p.dev_status, CASCADE_FLAG_DEPTH);
    s_nanc = n;
  }
  const float* q = (const float*)p.q + ((int64_t)node * p.n_heads + head) * D;
  for (int d = tid; d < D; d += 256) qs[d] = q[d];
  __syncthreads();
  const int s = s_row, lo = p.node_off[s], P = p.prefix_len[s], nanc = s_nanc;
  const int L = P + nanc;
  const float* kc = (const float*)p.k_cache + s * p.sr + kvh * p.sh;
  const float* vc = (const float*)p.v_cache + s * p.sr + kvh * p.sh;
  const float* kt = (const float*)p.k_tree;
  const float* vt = (const float*)p.v_tree;
  float m = -INFINITY, l = 0.f, acc = 0.f;  // acc: output element tid (tid < D)
  for (int base = 0; base < L; base += 256) {
    const int j = base + tid;
    float z = -INFINITY;
    if (j < L) {
      const float* kp = (j < P) ? kc + (int64_t)j * p.sp
                                : kt + ((int64_t)(lo + anc[j - P]) * p.n_kv_heads + kvh) * D;
      float dot = 0.f;
      for (int d = 0; d < D; ++d) dot = fmaf(qs[d], kp[d], dot);
      z = dot * p.scale_log2e;
    }
    float cm = wave_max(z);
    if ((tid & 63) == 0) red[tid >> 6] = cm;
    __syncthreads();
    cm = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float m_new = fmaxf(m, cm);
    const float alpha = exp2f(m - m_new);   // m = -inf on the first chunk gives 0
    const float e = (j < L) ? exp2f(z - m_new) : 0.f;
    sc[tid] = e;
    float cs = wave_sum(e);
    if ((tid & 63) == 0) red[4 + (tid >> 6)] = cs;
    __syncthreads();
    l = l * alpha + (red[4] + red[5] + red[6] + red[7]);
    m = m_new;
    if (tid < D) {
      acc *= alpha;
      const int cnt = min(256, L - base);
      for (int jj = 0; jj < cnt; ++jj) {
        const int j2 = base + jj;
        const float* vp = (j2 < P) ? vc + (int64_t)j2 * p.sp
                                   : vt + ((int64_t)(lo + anc[j2 - P]) * p.n_kv_heads + kvh) * D;
        acc = fmaf(sc[jj], vp[tid], acc);
      }
    }
    __syncthreads();
  }
  if (tid < D) ((float*)p.out)[((int64_t)node * p.n_heads + head) * D + tid] = acc / l;
  if (tid == 0 && p.lse) p.lse[(int64_t)node * p.n_heads + head] = m * LN2 + logf(l);
}

// ----------------------------------------------------------------------------------------- bf16
constexpr int KT = 64;  // keys per tile

// Workgroups are dispatched in index order, and with ragged prefixes the rows differ several-fold in
// work: a heavy row that happens to sit at the end of the batch would start when the rest of the grid
// is almost done and finish alone.  Dispatch position z therefore takes the z-th heaviest row
// (keys = prefix + tree nodes; ties by index), computed redundantly by every wave from the two small
// arrays it reads anyway.  Batches of more than 64 rows keep their order.
// The row's first node, node count and prefix length come back with it: the lanes already hold them, so the
// workgroup does not go to memory a second time for three values that the next loads depend on.
struct RowInfo {
  int s, lo, T, P;
};
__device__ __forceinline__ RowInfo row_by_work_rank(const AttnParams& p, int z, int n_rows, int lane) {
  RowInfo ri;
  if (n_rows > 64 || n_rows <= 1) {
    ri.s = z;
    ri.lo = p.node_off[z];
    ri.T = p.node_off[z + 1] - ri.lo;
    ri.P = p.prefix_len[z];
    return ri;
  }
  int lo_l = 0, t_l = 0, p_l = 0, work = -1;
  if (lane < n_rows) {
    lo_l = p.node_off[lane];
    t_l = p.node_off[lane + 1] - lo_l;
    p_l = p.prefix_len[lane];
    work = p_l + t_l;
  }
  int rank = 0;
  for (int r = 0; r < n_rows; ++r) {
    const int wr = __builtin_amdgcn_readlane(work, r);
    rank += (wr > work || (wr == work && r < lane)) ? 1 : 0;
  }
  const unsigned long long hit = __ballot(lane < n_rows && rank == z);
  ri.s = hit ? __ffsll((long long)hit) - 1 : z;   // (ranks are a permutation: some lane always hits)
  ri.lo = __builtin_amdgcn_readlane(lo_l, ri.s);
  ri.T = __builtin_amdgcn_readlane(t_l, ri.s);
  ri.P = __builtin_amdgcn_readlane(p_l, ri.s);
  return ri;
}

// Workgroups are dealt round-robin to the 8 XCDs (one L2 each) in launch order: hardware id h runs on
// XCD h % 8.  A unit = the nx workgroups of one (row, kv head).  This renumbering keeps a unit's
// workgroups on one XCD (they meet in one L2) while consecutive units still go to different XCDs, so
// rows with long and short prefixes stay spread over the chip.  Needs a unit count divisible by 8;
// otherwise the launch order is kept.
__device__ __forceinline__ unsigned xcd_local_order(unsigned h, unsigned nx, unsigned n_units) {
  if (n_units & 7u) return h;
  const unsigned x = h & 7u, k = h >> 3;          // XCD, slot inside the XCD
  return ((k / nx) * 8u + x) * nx + k % nx;       // unit (k / nx) * 8 + x, workgroup k % nx of it
}


// A row whose tree has more nodes than the host's bound is not computed (the grid and the LDS arrays
// were sized for the bound): the precondition flag is raised and the row's outputs are still defined -
// zeros and lse = -inf, or empty split partials that the merge kernel turns into the same.  Called by
// every workgroup of such a row; the one with query block 0 of each (kv head, split) does the writing.
template <int D, bool SPLIT>
__device__ __forceinline__ void skip_oversize_row(const AttnParams& p, int lo, int T, int kvh, int sb, int split, int tid, int nthreads) {
  if (sb != 0) return;
  if (tid == 0) atomicOr(p.dev_status, CASCADE_FLAG_TREE_SIZE);
  const int G = p.group;
  const int Tc = min(T, p.n_rows_total / p.n_heads - lo);   // never past the packed arrays
  for (int r = tid; r < Tc * G; r += nthreads) {
    const int64_t rowg = (int64_t)(lo + r / G) * p.n_heads + kvh * G + r % G;
    if (SPLIT) {
      float* wm = p.ws_ml + ((int64_t)split * p.n_rows_total + rowg) * 2;
      wm[0] = -INFINITY;
      wm[1] = 0.f;
    } else {
      uint4* o = (uint4*)((uint16_t*)p.out + rowg * D);
#pragma unroll
      for (int c = 0; c < D / 8; ++c) o[c] = make_uint4(0, 0, 0, 0);
      if (p.lse) p.lse[rowg] = -INFINITY;
    }
  }
}

// two floats -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  const bf16x2_t v = __builtin_convertvector(f32x2_t{a, b}, bf16x2_t);
  return *(const uint32_t*)&v;
}
// 2^x for x <= 0 or -inf (v_exp_f32; no range handling needed here)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

union Frag8 {
  bf16x8 v;
  uint4 u;
  uint2 h[2];
};

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

template <int D>
struct TileSmem {
  static constexpr int KP = D + 8;      // K row pitch (elements)
  static constexpr int VP = D + 16;     // V row pitch (elements): 4 consecutive keys fall on distinct bank groups
  uint16_t k[KT * KP];
  uint16_t v[KT * VP];
};

// Large trees.  Workgroup = (row, kv head, 16*NQ*NW query rows, kv split); its NW waves own NQ 16-row
// query blocks each and share every 64-key K/V tile through LDS.  Tiles are double-buffered in LDS
// and prefetched through registers: while tile t is multiplied, tile t+1 is written to the other
// buffer and tile t+2 is in flight from HBM, with one workgroup barrier per tile.  K and V are
// stored row-major; the V^T operand is fetched with the transposing LDS read.
template <int D, int NQ, int NW, bool SPLIT>
__global__ __launch_bounds__(64 * NW, (NQ == 4 || NW == 8) ? 1 : 2) void attn_bf16_kernel(AttnParams p) {
  using TS = TileSmem<D>;
  extern __shared__ __align__(16) char smem_raw[];
  TS* tiles = (TS*)smem_raw;                                                    // [2]
  int* s_parent = (int*)(smem_raw + 2 * sizeof(TS));                            // [CASCADE_MAX_TREE]
  unsigned long long* s_anc = (unsigned long long*)(s_parent + CASCADE_MAX_TREE);   // [2][RW]
  constexpr int NT = 64 * NW;        // threads
  constexpr int RW = 16 * NQ * NW;   // query rows of the workgroup
  constexpr int KS = D / 32;   // 32-wide d steps of the score MFMA
  constexpr int DB = D / 16;   // 16-wide d blocks of the output
  constexpr int DC = D / 8;    // 16-byte chunks per row
  constexpr int NPC = KT * DC / NT;   // 16-byte pieces of K (and of V) per thread per tile
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  // the query blocks and splits of a (row, kv head), which stream the same keys and values, share an L2
  const unsigned nx = gridDim.x, ny = gridDim.y;
  const unsigned lid = xcd_local_order(blockIdx.x + nx * (blockIdx.y + ny * blockIdx.z), nx, ny * gridDim.z);
  const int bx = (int)(lid % nx), kvh = (int)((lid / nx) % ny);
  const RowInfo ri = row_by_work_rank(p, (int)(lid / (nx * ny)), (int)gridDim.z, threadIdx.x & 63);
  const int s = ri.s, lo = ri.lo, T = ri.T, P = ri.P;
  const int split = bx % p.n_split, sb = bx / p.n_split;
  const int G = p.group;
  const int M = T * G;
  const int row0 = sb * RW;
  if (T > p.max_tree) { skip_oversize_row<D, SPLIT>(p, lo, T, kvh, sb, split, tid, NT); return; }
  if (row0 >= M || T > CASCADE_MAX_TREE) return;
  const int n_pt = (P + KT - 1) / KT, n_tt = (T + KT - 1) / KT, nt = n_pt + n_tt;
  const int per = (nt + p.n_split - 1) / p.n_split;
  const int t_begin = split * per, t_end = min(nt, t_begin + per);

  const uint16_t* kc = (const uint16_t*)p.k_cache + s * p.sr + kvh * p.sh;
  const uint16_t* vc = (const uint16_t*)p.v_cache + s * p.sr + kvh * p.sh;
  const uint16_t* ktr = (const uint16_t*)p.k_tree + ((int64_t)lo * p.n_kv_heads + kvh) * D;
  const uint16_t* vtr = (const uint16_t*)p.v_tree + ((int64_t)lo * p.n_kv_heads + kvh) * D;
  const int64_t tree_pitch = (int64_t)p.n_kv_heads * D;

  // tile staging registers: piece c = tid + 256 it -> key c / DC, 8 d at c % DC
  u32x4 kr[NPC], vr[NPC];
  auto request_tile = [&](int t) {
    const bool tree_tile = t >= n_pt;
    const int kbase = tree_tile ? (t - n_pt) * KT : t * KT;
    const int klimit = tree_tile ? T : P;
    const uint16_t* ksrc = tree_tile ? ktr : kc;
    const uint16_t* vsrc = tree_tile ? vtr : vc;
    const int64_t pitch = tree_tile ? tree_pitch : p.sp;
#pragma unroll
    for (int it = 0; it < NPC; ++it) {
      const int c = tid + NT * it, key = c / DC, dc = c % DC;
      kr[it] = u32x4{0u, 0u, 0u, 0u};
      vr[it] = u32x4{0u, 0u, 0u, 0u};
      if (t < t_end && kbase + key < klimit) {
        kr[it] = *(const u32x4*)(ksrc + (int64_t)(kbase + key) * pitch + 8 * dc);
        vr[it] = *(const u32x4*)(vsrc + (int64_t)(kbase + key) * pitch + 8 * dc);
      }
    }
  };
  // registers -> LDS buffer, plus (tree tiles) one ancestor-or-self word per query row of the workgroup
  auto store_tile = [&](int t, int buf) {
#pragma unroll
    for (int it = 0; it < NPC; ++it) {
      const int c = tid + NT * it, key = c / DC, dc = c % DC;
      *(u32x4*)(&tiles[buf].k[key * TS::KP + 8 * dc]) = kr[it];
      *(u32x4*)(&tiles[buf].v[key * TS::VP + 8 * dc]) = vr[it];
    }
    if (t < t_end && t >= n_pt && tid < RW) {
      const int kbase = (t - n_pt) * KT;
      const int r = row0 + tid;
      unsigned long long wbits = 0ull;
      if (r < M) {
        int a = r % T, guard = 0;
        while (a >= 0 && guard++ <= CASCADE_MAX_TREE) {
          const int rel = a - kbase;
          if (rel < 0) break;   // ancestors only get smaller
          if (rel < 64) wbits |= 1ull << rel;
          a = s_parent[a];
        }
      }
      s_anc[buf * RW + tid] = wbits;
    }
  };

  request_tile(t_begin);   // in flight while parents and queries are fetched
  if (t_end > n_pt) {
    for (int i = tid; i < T; i += NT) {
      int pi = p.parent[lo + i];
      if (pi >= i || pi < -1 || (i == 0 && pi != -1) || (i > 0 && pi < 0)) {
        atomicOr(p.dev_status, CASCADE_FLAG_PARENT);
        pi = (i == 0) ? -1 : 0;   // keep the climb finite
      }
      s_parent[i] = pi;
    }
  }

  // query fragments (B operand of S^T): lane = (query l16, d group g)
  Frag8 qf[NQ][KS];
  int64_t out_row[NQ];   // index into [N*Hq] or -1
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    const int r = row0 + 16 * (wave + NW * n) + l16;
    const bool ok = r < M;
    const int i = ok ? r % T : 0, hg = ok ? r / T : 0;
    const int64_t rowg = (int64_t)(lo + i) * p.n_heads + kvh * G + hg;
    out_row[n] = ok ? rowg : -1;
    const uint16_t* qp = (const uint16_t*)p.q + rowg * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ok) qf[n][ks].u = *(const uint4*)(qp + 32 * ks);
      else qf[n][ks].u = make_uint4(0, 0, 0, 0);
    }
  }

  f32x4 ot[NQ][DB];
  float m_run[NQ], l_run[NQ];
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    m_run[n] = -INFINITY;
    l_run[n] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db) ot[n][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  __syncthreads();               // parent array complete
  store_tile(t_begin, 0);
  request_tile(t_begin + 1);
  __syncthreads();

  for (int t = t_begin; t < t_end; ++t) {
    const int buf = (t - t_begin) & 1;
    const TS& tl = tiles[buf];
    const bool tree_tile = t >= n_pt;
    const int kbase = tree_tile ? (t - n_pt) * KT : t * KT;
    const int klimit = tree_tile ? T : P;
    // tile t+1 (requested one iteration ago) goes to the other buffer, tile t+2 is requested
    store_tile(t + 1, buf ^ 1);
    request_tile(t + 2);

    // S^T = K Q^T : st[n][kt] holds keys 16*kt + 4*g + c for query l16
    f32x4 st[NQ][4];
#pragma unroll
    for (int n = 0; n < NQ; ++n)
#pragma unroll
      for (int kt = 0; kt < 4; ++kt) st[n][kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Frag8 kf;
        kf.u = *(const uint4*)(&tl.k[(16 * kt + l16) * TS::KP + 32 * ks + 8 * g]);
#pragma unroll
        for (int n = 0; n < NQ; ++n)
          st[n][kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, qf[n][ks].v, st[n][kt], 0, 0, 0);
      }
    }

    // mask + online softmax; probabilities packed as the B operand of the second MFMA
    Frag8 pf[NQ][2];
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      unsigned long long valid;
      if (tree_tile) {
        valid = s_anc[buf * RW + 16 * (wave + NW * n) + l16];
      } else {
        const int rem = klimit - kbase;
        valid = rem >= 64 ? ~0ull : ((1ull << rem) - 1ull);
      }
      if (out_row[n] < 0) valid = 0ull;
      float mx = -INFINITY;
      if (__ballot(valid != ~0ull) == 0ull) {
        // every key of the tile is visible to every query of the block: no masking
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            st[n][kt][c] *= p.scale_log2e;
            mx = fmaxf(mx, st[n][kt][c]);
          }
      } else {
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
          const uint32_t nib = (uint32_t)(valid >> (16 * kt + 4 * g));   // this lane's 4 keys of sub-tile kt
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const float z = ((nib >> c) & 1u) ? st[n][kt][c] * p.scale_log2e : -INFINITY;
            st[n][kt][c] = z;
            mx = fmaxf(mx, z);
          }
        }
      }
      mx = rows4_max(mx);
      const float m_new = fmaxf(m_run[n], mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      float ls = 0.f;
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float e = fast_exp2(st[n][kt][c] - m_use);
          st[n][kt][c] = e;
          ls += e;
        }
      if (__ballot(m_new != m_run[n]) != 0ull) {
        // the running maximum moved for some query of the block: rescale the accumulators
        const float alpha = fast_exp2(m_run[n] - m_use);   // -inf - finite = -inf -> 0
        l_run[n] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db) ot[n][db] *= alpha;
        m_run[n] = m_new;
      }
      l_run[n] += ls;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        pf[n][j].u.x = pack_bf16x2(st[n][2 * j][0], st[n][2 * j][1]);
        pf[n][j].u.y = pack_bf16x2(st[n][2 * j][2], st[n][2 * j][3]);
        pf[n][j].u.z = pack_bf16x2(st[n][2 * j + 1][0], st[n][2 * j + 1][1]);
        pf[n][j].u.w = pack_bf16x2(st[n][2 * j + 1][2], st[n][2 * j + 1][3]);
      }
    }

    // O^T += V^T P^T.  Operand slots of lane (l16, g): keys 32j + 4g + {0..3} and 32j + 16 + 4g + {0..3}
    // at d = 16 db + l16, fetched by two transposing loads from the row-major V tile.
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const uint16_t* vp = &tl.v[(32 * j + 4 * g + (l16 >> 2)) * TS::VP + 16 * db + 4 * (l16 & 3)];
        union { Frag8 f; s16x4 h[2]; } vf;
        vf.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp));
        vf.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp + 16 * TS::VP));
#pragma unroll
        for (int n = 0; n < NQ; ++n)
          ot[n][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.f.v, pf[n][j].v, ot[n][db], 0, 0, 0);
      }
    }
    __syncthreads();   // tile t consumed by every wave; tile t+1 complete in the other buffer
  }

  // epilogue: lane (query l16, g) owns d = 16*db + 4*g + c
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    float l = l_run[n];
    l = rows4_sum(l);
    if (out_row[n] < 0) continue;
    if (SPLIT) {
      float* wo = p.ws_o + ((int64_t)split * p.n_rows_total + out_row[n]) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db) *(f32x4*)(wo + 16 * db + 4 * g) = ot[n][db];
      if (g == 0) {
        float* wm = p.ws_ml + ((int64_t)split * p.n_rows_total + out_row[n]) * 2;
        wm[0] = m_run[n];
        wm[1] = l;
      }
    } else {
      const float inv = 1.f / l;
      uint16_t* o = (uint16_t*)p.out + out_row[n] * D;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        uint2 w;
        w.x = pack_bf16x2(ot[n][db][0] * inv, ot[n][db][1] * inv);
        w.y = pack_bf16x2(ot[n][db][2] * inv, ot[n][db][3] * inv);
        *(uint2*)(o + 16 * db + 4 * g) = w;
      }
      if (g == 0 && p.lse) p.lse[out_row[n]] = m_run[n] * LN2 + logf(l);
    }
  }
}

// A wave's own LDS-direct loads have landed when at most the N youngest are outstanding; its LDS writes and
// reads are complete at lgkmcnt(0); then the workgroup barrier, bare (a fenced barrier would wait for every
// outstanding load, i.e. for the whole prefetch ring).
template <int N>
__device__ __forceinline__ void wait_and_sync() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// ---------------------------------------------------------------------- bf16, large trees
// Workgroup = (row, kv head, 256 query rows, kv split): eight waves x two 16-row query blocks share every
// 64-key K / V tile.  Tiles never pass through registers on their way in: 16-byte LDS-direct loads
// (global_load_lds_dwordx4, M0 = LDS address of the wave's 1 KiB chunk) write them into two rings of NS
// tiles each, NS - 1 tiles ahead of their use; a wave waits only for its own chunks of the tile that is
// needed next (vmcnt), then one bare s_barrier per tile makes everybody's chunks visible and the oldest
// tile's buffer free.  An LDS-direct load puts lane l's 16 bytes at 16 l behind M0, so a tile cannot be
// padded; bank conflicts are avoided by choosing WHICH 16-byte piece of a key row each lane fetches: LDS
// slot q of row r holds piece q ^ swz(r) (K: the 16 keys a score MFMA reads together land in 16 different
// slots; V: the 8 keys x 32 bytes of half a transposing read likewise).
// The loop is software-pipelined inside a wave: the score MFMAs of tile t+1 are issued between the
// exponentials of tile t (matrix cores and vector ALU run side by side), then the PV MFMAs of tile t.
// The running maximum that the exponentials refer to is only moved when a row's maximum has grown by
// more than 2^8 (the result does not depend on the reference, p <= 256 is exact enough in bf16 and far
// from overflow in the float accumulators), so the accumulator rescale is a rarely taken branch.
template <int D>
struct RingGeom {
  static constexpr int RB = 2 * D;        // bytes per key row
  static constexpr int PPR = RB / 16;     // 16-byte pieces per row
  static constexpr int RPC = 1024 / RB;   // rows per 1 KiB chunk (one wave-wide LDS-direct load)
  static constexpr int CPT = KT / RPC;    // chunks per tile
  static constexpr int TILE = KT * RB;    // bytes per K (or V) tile
  // slot swizzles (see above); both depend on the key index modulo 16 only
  __device__ static constexpr int kswz(int key) { return D == 128 ? (key & 15) : ((key >> 1) & 7); }
  __device__ static constexpr int vswz(int key) { return D == 128 ? 2 * (key & 7) : 2 * ((key >> 1) & 3); }
};

constexpr float RESCALE_STEP = 8.f;   // log2 units

// Maxima of MFMA results (or -inf).  The IEEE-754-2019 maximum maps to v_maximum3_f32 without the input-quieting
// copies that fmaxf costs in IEEE mode.  It must stay a compiler-visible operation: a vector ALU instruction that
// reads a register too soon after the matrix core was told to write it gets the register's OLD contents, the
// hardware does not interlock that case, and the compiler pads only the instructions it can see - the same
// maximum written as inline assembly read stale registers whenever the scheduler put it right behind its MFMA.
__device__ __forceinline__ float vmax3(float a, float b, float c) {
  return __builtin_elementwise_maximum(__builtin_elementwise_maximum(a, b), c);
}
__device__ __forceinline__ float vmax2(float a, float b) { return __builtin_elementwise_maximum(a, b); }
__device__ __forceinline__ float rows4_max_raw(float v) {
  cascade_u32x2 a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = vmax2(__uint_as_float(a.x), __uint_as_float(a.y));
  cascade_u32x2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return vmax2(__uint_as_float(b.x), __uint_as_float(b.y));
}

template <int D, int NS>
__global__ __launch_bounds__(512, 1) void attn_bf16_ring_kernel(AttnParams p) {
  using GM = RingGeom<D>;
  constexpr int NW = 8, NQ = 2, NT = 64 * NW, RW = 16 * NQ * NW;
  constexpr int KS = D / 32, DB = D / 16;
  constexpr int CPW = GM::CPT / NW;     // chunks of K (and of V) a wave loads per tile: 2 (D = 128) or 1 (D = 64)
  constexpr int LPI = 2 * CPW;          // LDS-direct loads a wave issues per iteration
  static_assert(GM::CPT % NW == 0 && NS == 3, "ring geometry: the loop below is unrolled three times");
  extern __shared__ __align__(1024) char ring_smem[];
  char* const smem_raw = ring_smem;
  // [K ring: NS tiles][V ring: NS tiles][parent: CASCADE_MAX_TREE ints][ancestor words: 2 x RW]
  int* s_parent = (int*)(smem_raw + 2 * NS * GM::TILE);
  unsigned long long* s_anc = (unsigned long long*)(s_parent + CASCADE_MAX_TREE);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g = lane >> 4;
  const unsigned nx = gridDim.x, ny = gridDim.y;
  const unsigned lid = xcd_local_order(blockIdx.x + nx * (blockIdx.y + ny * blockIdx.z), nx, ny * gridDim.z);
  const int bx = (int)(lid % nx), kvh = (int)((lid / nx) % ny);
  const RowInfo ri = row_by_work_rank(p, (int)(lid / (nx * ny)), (int)gridDim.z, lane);
  const int s = ri.s, lo = ri.lo, T = ri.T, P = ri.P;
  const int sb = bx;   // the keys of a row are never split across workgroups here (n_split == 1)
  const int G = p.group;
  const int M = T * G;
  const int row0 = sb * RW;
  if (T > p.max_tree) { skip_oversize_row<D, false>(p, lo, T, kvh, sb, 0, tid, NT); return; }
  if (row0 >= M || T > CASCADE_MAX_TREE) return;
  const int n_pt = (P + KT - 1) / KT, n_tt = (T + KT - 1) / KT, nt = n_pt + n_tt;
  const int t_begin = 0, t_end = nt;   // nt >= 1: a tree has at least its root

  const char* kc = (const char*)((const uint16_t*)p.k_cache + s * p.sr + kvh * p.sh);
  const char* vc = (const char*)((const uint16_t*)p.v_cache + s * p.sr + kvh * p.sh);
  const char* ktr = (const char*)((const uint16_t*)p.k_tree + ((int64_t)lo * p.n_kv_heads + kvh) * D);
  const char* vtr = (const char*)((const uint16_t*)p.v_tree + ((int64_t)lo * p.n_kv_heads + kvh) * D);
  const unsigned tree_pitch_b = (unsigned)(p.n_kv_heads * D * 2), cache_pitch_b = (unsigned)(p.sp * 2);
  const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(size_t)smem_raw);

  // ---- loader: chunk c = CPW wave + i of a tile; lane -> row c RPC + lane / PPR, LDS slot lane % PPR.
  // Ring stages are numbered by the workgroup's own tile count (tile t lives in stage (t - t_begin) % NS), so
  // that inside the loop, which is unrolled NS times, every LDS address is a per-lane register + a constant.
  int ld_row[CPW];
  unsigned ld_kpiece[CPW], ld_vpiece[CPW], ld_kfull[CPW], ld_vfull[CPW];
#pragma unroll
  for (int i = 0; i < CPW; ++i) {
    const int r = (CPW * wave + i) * GM::RPC + lane / GM::PPR, q = lane % GM::PPR;
    ld_row[i] = r;
    ld_kpiece[i] = 16u * (unsigned)(q ^ GM::kswz(r));
    ld_vpiece[i] = 16u * (unsigned)(q ^ GM::vswz(r));
    ld_kfull[i] = (unsigned)r * cache_pitch_b + ld_kpiece[i];   // offsets inside a whole prefix tile
    ld_vfull[i] = (unsigned)r * cache_pitch_b + ld_vpiece[i];
  }
  // One matrix (K or V) of tile tk into ring stage `stage`.  tk is clamped to the workgroup's last tile (the
  // extra requests keep the per-iteration load count fixed; their data lands in a free stage and is never
  // used); rows past the end of the tile's source are read from its last row (always in bounds; their scores
  // are masked, so the finite clamped values contribute exactly nothing).
  auto request = [&](int tk, int stage, bool is_v) {
    const int tc = min(tk, t_end - 1);
    const unsigned ldst = lds0 + (is_v ? NS * GM::TILE : 0) + stage * GM::TILE + CPW * wave * 1024;
    if (tc < n_pt && (tc + 1) * KT <= P) {
      // a whole tile of the prefix: nothing to clamp, the per-lane offsets are constants
      const char* src = (is_v ? vc : kc) + (int64_t)tc * KT * cache_pitch_b;
#pragma unroll
      for (int i = 0; i < CPW; ++i) {
        const unsigned l = ldst + i * 1024;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(l), "v"(is_v ? ld_vfull[i] : ld_kfull[i]), "s"(src) : "memory");
      }
    } else {
      const bool tree_tile = tc >= n_pt;
      const int kb = tree_tile ? (tc - n_pt) * KT : tc * KT;
      const int lim = (tree_tile ? T : P) - 1 - kb;                 // last valid row of the tile, >= 0
      const unsigned pitch_b = tree_tile ? tree_pitch_b : cache_pitch_b;
      const char* src = (is_v ? (tree_tile ? vtr : vc) : (tree_tile ? ktr : kc)) + (int64_t)kb * pitch_b;
#pragma unroll
      for (int i = 0; i < CPW; ++i) {
        const unsigned voff = (unsigned)min(ld_row[i], lim) * pitch_b + (is_v ? ld_vpiece[i] : ld_kpiece[i]);
        const unsigned l = ldst + i * 1024;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(l), "v"(voff), "s"(src) : "memory");
      }
    }
  };

  // ancestor-or-self words of tree tile tt (tile index in the workgroup's numbering) for the 256 query rows
  auto build_mask = [&](int tt) {
    if (tid < RW) {
      const int kbase = (tt - n_pt) * KT;
      const int r = row0 + tid;
      unsigned long long wbits = 0ull;
      if (r < M) {
        int a = r % T, guard = 0;
        while (a >= 0 && guard++ <= CASCADE_MAX_TREE) {
          const int rel = a - kbase;
          if (rel < 0) break;   // ancestors only get smaller
          if (rel < 64) wbits |= 1ull << rel;
          a = s_parent[a];
        }
      }
      s_anc[(tt & 1) * RW + tid] = wbits;
    }
  };

  // ---- prologue: K(t_begin) first, then the steady-state order K(t + NS), V(t + NS - 1) of iterations -NS+1 .. -1
  request(t_begin, 0, false);
#pragma unroll
  for (int i = 1 - NS; i < 0; ++i) {
    request(t_begin + i + NS, (i + NS) % NS, false);
    request(t_begin + i + NS - 1, (i + NS - 1) % NS, true);
  }
  if (t_end > n_pt) {
    for (int i = tid; i < T; i += NT) {
      int pi = p.parent[lo + i];
      if (pi >= i || pi < -1 || (i == 0 && pi != -1) || (i > 0 && pi < 0)) {
        atomicOr(p.dev_status, CASCADE_FLAG_PARENT);
        pi = (i == 0) ? -1 : 0;   // keep the climb finite
      }
      s_parent[i] = pi;
    }
  }
  // query fragments (B operand of S^T): lane = (query l16, d group g)
  Frag8 qf[NQ][KS];
  int64_t out_row[NQ];   // index into [N*Hq] or -1
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    const int r = row0 + 16 * (wave + NW * n) + l16;
    const bool ok = r < M;
    const int i = ok ? r % T : 0, hg = ok ? r / T : 0;
    const int64_t rowg = (int64_t)(lo + i) * p.n_heads + kvh * G + hg;
    out_row[n] = ok ? rowg : -1;
    const uint16_t* qp = (const uint16_t*)p.q + rowg * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ok) qf[n][ks].u = *(const uint4*)(qp + 32 * ks);
      else qf[n][ks].u = make_uint4(0, 0, 0, 0);
    }
  }
  f32x4 ot[NQ][DB];
  f32x4 lsum[NQ];        // row sums of the (bf16) probabilities, produced by the matrix cores: every entry holds the sum
  float m_ref[NQ];
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    m_ref[n] = -INFINITY;
    lsum[n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int db = 0; db < DB; ++db) ot[n][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  Frag8 ones;            // a V^T fragment of bf16 ones: ones x P^T = the probabilities' row sums
  ones.u = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);

  // ---- LDS read addresses.  K fragment (kt, ks): key 16 kt + l16, pieces of d 32 ks + 8 g: slot (4 ks + g) ^ swz;
  // V operand (db, j): keys 32 j + 4 g + (l16 >> 2) (+ 16), 4 consecutive d at 16 db + 4 (l16 & 3): slot
  // (2 db + ((l16 & 3) >> 1)) ^ swz.  ks and db enter by XOR into a per-lane constant (one register each), the
  // stage, kt and j are compile-time byte offsets.
  const unsigned k_lane = (unsigned)(l16 * GM::RB) + 16u * (unsigned)(g ^ GM::kswz(l16));
  const int vkey = 4 * g + (l16 >> 2);
  const unsigned v_lane = (unsigned)(vkey * GM::RB) + ((16u * (unsigned)((l16 & 3) >> 1)) ^ (16u * (unsigned)GM::vswz(vkey))) + 8u * (unsigned)(l16 & 1);
  static_assert(GM::kswz(0) == GM::kswz(16) && GM::vswz(3) == GM::vswz(19) && GM::vswz(3) == GM::vswz(35), "swizzles have period 16");
  const char* k_addr[KS];
  const char* v_addr[DB];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) k_addr[ks] = smem_raw + (k_lane ^ (unsigned)(64 * ks));
#pragma unroll
  for (int db = 0; db < DB; ++db) v_addr[db] = smem_raw + NS * GM::TILE + (v_lane ^ (unsigned)(32 * db));

  f32x4 st[NQ][4];   // scores: st[n][kt] holds keys 16 kt + 4 g + c for query l16
  // K fragments of one 16-key sub-tile kt of the tile in K stage `stage` (A operand of S^T = K Q^T)
  auto load_kfrags = [&](Frag8 (&kf)[KS], int stage, int kt) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kf[ks].u = *(const uint4*)(k_addr[ks] + stage * GM::TILE + 16 * kt * GM::RB);
  };
  auto score_kt = [&](const Frag8 (&kf)[KS], int kt) {
#pragma unroll
    for (int n = 0; n < NQ; ++n) st[n][kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int n = 0; n < NQ; ++n) st[n][kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks].v, qf[n][ks].v, st[n][kt], 0, 0, 0);
  };
  // V operand of step i = (db, j) = (i / 2, i % 2) of the tile in V stage `stage`: keys 32 j + 4 g + {0..3} and
  // 32 j + 16 + 4 g + {0..3} at d = 16 db + l16, fetched by two transposing loads from the row-major tile
  union VFrag { Frag8 f; s16x4 h[2]; };
  auto load_vfrag = [&](VFrag& vf, int stage, int i) {
    const char* vp = v_addr[i >> 1] + stage * GM::TILE + 32 * (i & 1) * GM::RB;
    vf.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp));
    vf.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp + 16 * GM::RB));
  };
  // largest of a lane's 16 scores of query block n (raw, before the scale)
  auto lane_max = [&](int n) {
    float a = vmax3(st[n][0][0], st[n][0][1], st[n][0][2]);
    a = vmax3(a, st[n][0][3], st[n][1][0]);
    a = vmax3(a, st[n][1][1], st[n][1][2]);
    a = vmax3(a, st[n][1][3], st[n][2][0]);
    a = vmax3(a, st[n][2][1], st[n][2][2]);
    a = vmax3(a, st[n][2][3], st[n][3][0]);
    a = vmax3(a, st[n][3][1], st[n][3][2]);
    return vmax2(a, st[n][3][3]);
  };

  __syncthreads();                    // parent array complete (the compiler's own waits cover its loads)
  if (t_begin >= n_pt) build_mask(t_begin);
  wait_and_sync<LPI * (NS - 1)>();    // K(t_begin) everywhere (and the first mask)
  float lmax[NQ];                     // lane_max of the scores in st (valid for tiles that need no mask)
  {
    Frag8 kf[2][KS];
    load_kfrags(kf[0], 0, 0);
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
      if (kt < 3) load_kfrags(kf[(kt + 1) & 1], 0, kt + 1);
      score_kt(kf[kt & 1], kt);
    }
#pragma unroll
    for (int n = 0; n < NQ; ++n) lmax[n] = lane_max(n);
  }

  // One tile.  ST = ring stage of tile t (compile time: the loop below is unrolled NS times).
  auto tile_step = [&](int t, auto st_const) {
    constexpr int ST = decltype(st_const)::value;
    constexpr int ST_K = (ST + 1) % NS;             // stage of K(t+1)
    constexpr int ST_VNEW = (ST + NS - 1) % NS;     // stage V(t + NS - 1) goes to (V(t-1) has been consumed)
    const bool tree_tile = t >= n_pt;
    const int kbase = tree_tile ? (t - n_pt) * KT : t * KT;
    const int rem = (tree_tile ? T : P) - kbase;
    wait_and_sync<LPI * (NS - 2)>();   // K(t+1), V(t) landed everywhere; K(t), V(t-1) free
    request(t + NS, ST, false);
    request(t + NS - 1, ST_VNEW, true);
    Frag8 kf[2][KS];
    load_kfrags(kf[0], ST_K, 0);       // in flight during the reference check
    if (t + 1 < t_end && t + 1 >= n_pt) build_mask(t + 1);   // read after the next barrier

    // ---- masks (tree tiles and the ragged last prefix tile) and the reference of the exponentials
    if (tree_tile || rem < KT) {
#pragma unroll
      for (int n = 0; n < NQ; ++n) {
        unsigned long long valid = tree_tile ? s_anc[(t & 1) * RW + 16 * (wave + NW * n) + l16]
                                             : (rem >= 64 ? ~0ull : ((1ull << rem) - 1ull));
        if (out_row[n] < 0) valid = 0ull;
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
          const uint32_t nib = (uint32_t)(valid >> (16 * kt + 4 * g));   // this lane's 4 keys of sub-tile kt
#pragma unroll
          for (int c = 0; c < 4; ++c) st[n][kt][c] = ((nib >> c) & 1u) ? st[n][kt][c] : -INFINITY;
        }
        lmax[n] = lane_max(n);
      }
    }
    // a lane sees 16 of its row's 64 scores; if none of a wave's lanes exceeds its row's reference by more than
    // the step, no row does, and the reference stays (scale > 0: the maximum commutes with it)
    bool moved = false;
#pragma unroll
    for (int n = 0; n < NQ; ++n) moved |= lmax[n] * p.scale_log2e > m_ref[n] + RESCALE_STEP;   // -inf + 8 = -inf: a first finite score always moves it
    if (__ballot(moved) != 0ull) {
#pragma unroll
      for (int n = 0; n < NQ; ++n) {
        const float mx = rows4_max_raw(lmax[n]) * p.scale_log2e;
        const float m_new = (mx > m_ref[n] + RESCALE_STEP) ? mx : m_ref[n];
        const float use_new = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = fast_exp2(m_ref[n] - use_new);   // -inf - finite = -inf -> 0 ; equal -> 1
        lsum[n] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db) ot[n][db] *= alpha;
        m_ref[n] = m_new;
      }
    }
    float m_neg[NQ];
#pragma unroll
    for (int n = 0; n < NQ; ++n) m_neg[n] = (m_ref[n] == -INFINITY) ? 0.f : -m_ref[n];

    // ---- probabilities of tile t and scores of tile t+1.  Sub-tile kt's scores are consumed by the exponentials
    // (and packed as the B operand of the second MFMA) before the MFMAs of tile t+1 overwrite the same registers,
    // so the matrix cores work on sub-tile kt while the vector ALU is busy with sub-tile kt + 1.
    Frag8 pf[NQ][2];
    auto probs_kt = [&](int kt) {
#pragma unroll
      for (int n = 0; n < NQ; ++n) {
        float e[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) e[c] = fast_exp2(fmaf(st[n][kt][c], p.scale_log2e, m_neg[n]));   // -inf stays -inf -> 0
        const uint32_t lo2 = pack_bf16x2(e[0], e[1]), hi2 = pack_bf16x2(e[2], e[3]);
        if (kt & 1) { pf[n][kt >> 1].u.z = lo2; pf[n][kt >> 1].u.w = hi2; }
        else { pf[n][kt >> 1].u.x = lo2; pf[n][kt >> 1].u.y = hi2; }
      }
    };
    constexpr int NVS = 2 * DB, VW = 4;   // V steps per tile, steps whose fragments are requested ahead
    VFrag vf[VW];
    probs_kt(0);
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
      if (kt < 3) load_kfrags(kf[(kt + 1) & 1], ST_K, kt + 1);
      else {
#pragma unroll
        for (int i = 0; i < VW; ++i) load_vfrag(vf[i], ST, i);
        // left to itself the scheduler sinks every V read to just in front of its MFMA (fewer live registers) and
        // the second half of the step then waits out one LDS round trip per pair of MFMAs
        __builtin_amdgcn_sched_barrier(0);
      }
      score_kt(kf[kt & 1], kt);
      if (kt < 3) probs_kt(kt + 1);
    }

    // ---- O^T += V^T P^T, row sums += ones P^T; the vector ALU meanwhile looks at the next tile's scores
#pragma unroll
    for (int n = 0; n < NQ; ++n)
#pragma unroll
      for (int j = 0; j < 2; ++j) lsum[n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones.v, pf[n][j].v, lsum[n], 0, 0, 0);
#pragma unroll
    for (int n = 0; n < NQ; ++n) lmax[n] = lane_max(n);
#pragma unroll
    for (int i = 0; i < NVS; ++i) {
#pragma unroll
      for (int n = 0; n < NQ; ++n) ot[n][i >> 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[i % VW].f.v, pf[n][i & 1].v, ot[n][i >> 1], 0, 0, 0);
      if (i + VW < NVS) load_vfrag(vf[i % VW], ST, i + VW);
      __builtin_amdgcn_sched_barrier(0);   // keeps the read of step i + VW here, VW steps ahead of its use
    }
  };

  for (int t = t_begin; t < t_end; t += NS) {
    tile_step(t, std::integral_constant<int, 0>{});
    if (t + 1 >= t_end) break;
    tile_step(t + 1, std::integral_constant<int, 1>{});
    if (t + 2 >= t_end) break;
    tile_step(t + 2, std::integral_constant<int, 2>{});
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the clamped extra requests must not outlive the workgroup's LDS

  // epilogue: lane (query l16, g) owns d = 16*db + 4*g + c
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    const float l = lsum[n][0];
    if (out_row[n] < 0) continue;
    const float inv = 1.f / l;   // l >= 1: the node's own key is never masked
    uint16_t* o = (uint16_t*)p.out + out_row[n] * D;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      uint2 w;
      w.x = pack_bf16x2(ot[n][db][0] * inv, ot[n][db][1] * inv);
      w.y = pack_bf16x2(ot[n][db][2] * inv, ot[n][db][3] * inv);
      *(uint2*)(o + 16 * db + 4 * g) = w;
    }
    if (g == 0 && p.lse) p.lse[out_row[n]] = m_ref[n] * LN2 + logf(l);
  }
}

// ---------------------------------------------------------------------- bf16, small trees
// Workgroup = (row, kv head, 64 query rows, kv split), NKG key groups x 4 query blocks of waves.
// In every round the key groups take NKG consecutive 64-key tiles; the four waves of a
// group copy their tile into the group's LDS buffer (each a quarter of it), then each wave runs
// its own 16 query rows against it.  The next round's tile is requested from memory before the
// current one is consumed.  K and V are both stored row-major with plain 16-byte stores; the V^T
// operand of the second MFMA is read with the transposing LDS load (ds_read_b64_tr_b16): inside
// each group of 16 lanes, lane i passes the address of 4 consecutive d of key (i / 4), and lane L
// receives the 4 keys at d + L.  The key groups' (m, l, O) are merged through LDS at the
// end, so a drafted tree against a short prefix needs neither workspace traffic nor a second kernel.

template <int D>
struct KsplitGroupSmem {
  static constexpr int KP = D + 8;      // K row pitch (elements)
  static constexpr int VP = D + 16;     // V row pitch (elements): 4 consecutive keys fall on distinct bank groups
  uint16_t k[KT * KP];
  uint16_t v[KT * VP];
};

// NKG = key groups (the workgroup has NKG * 4 waves)
template <int D, int NKG, bool SPLIT>
// (four waves per workgroup: at most 168 registers, so that three workgroups share a CU)
__global__ __launch_bounds__(NKG * 256, (NKG == 1 ? 3 : 1)) void attn_bf16_ksplit_kernel(AttnParams p) {
  constexpr int NT = NKG * 256;
  using GS = KsplitGroupSmem<D>;
  extern __shared__ __align__(16) char smem_raw[];
  constexpr int KS = D / 32, DB = D / 16, DC = D / 8;
  constexpr int OP = D + 4;            // merge buffer row pitch (floats)
  constexpr int NPC = KT * DC / 256;   // 16-byte pieces of K (and of V) each lane copies per tile
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kg = wave >> 2, qb = wave & 3;     // key group, query block
  const int gl = tid & 255;                    // lane index inside the key group
  const int l16 = lane & 15, g = lane >> 4;
  GS* gs = (GS*)smem_raw + kg;
  int* s_parent = (int*)(smem_raw + NKG * sizeof(GS));                                         // [CASCADE_MAX_TREE]
  unsigned long long* s_anc = (unsigned long long*)(s_parent + CASCADE_MAX_TREE) + 64 * kg;   // [NKG][64]
  // the query blocks and splits of a (row, kv head) share an L2
  const unsigned nx = gridDim.x, ny = gridDim.y;
  const unsigned lid = xcd_local_order(blockIdx.x + nx * (blockIdx.y + ny * blockIdx.z), nx, ny * gridDim.z);
  const int bx = (int)(lid % nx), kvh = (int)((lid / nx) % ny);
  const RowInfo ri = row_by_work_rank(p, (int)(lid / (nx * ny)), (int)gridDim.z, threadIdx.x & 63);
  const int s = ri.s, lo = ri.lo, T = ri.T, P = ri.P;
  const int split = bx % p.n_split, sb = bx / p.n_split;
  const int G = p.group;
  const int M = T * G;
  const int row0 = sb * 64;
  if (T > p.max_tree) { skip_oversize_row<D, SPLIT>(p, lo, T, kvh, sb, split, tid, NT); return; }
  if (row0 >= M || T > CASCADE_MAX_TREE) return;
  const int n_pt = (P + KT - 1) / KT, n_tt = (T + KT - 1) / KT, nt = n_pt + n_tt;
  const int per = (nt + p.n_split - 1) / p.n_split;
  const int t_begin = split * per, t_end = min(nt, t_begin + per);
  const int n_rounds = (max(t_end - t_begin, 0) + NKG - 1) / NKG;

  const uint16_t* kc = (const uint16_t*)p.k_cache + s * p.sr + kvh * p.sh;
  const uint16_t* vc = (const uint16_t*)p.v_cache + s * p.sr + kvh * p.sh;
  const uint16_t* ktr = (const uint16_t*)p.k_tree + ((int64_t)lo * p.n_kv_heads + kvh) * D;
  const uint16_t* vtr = (const uint16_t*)p.v_tree + ((int64_t)lo * p.n_kv_heads + kvh) * D;
  const int64_t tree_pitch = (int64_t)p.n_kv_heads * D;

  // a quarter of the group's tile per wave: pieces gl, gl + 256, ... (piece c = key c / DC, 8 d at c % DC),
  // requested one round ahead (two rounds ahead, with a second register set, changed nothing).  Keys
  // past the end of the tile's source are read from its last row (clamped: always in bounds) and not
  // zeroed: their scores are masked to -inf, so their probabilities are exactly 0 and the clamped
  // (finite) rows contribute nothing; a select or a branch on the loaded value would make the compiler
  // wait for every load on the spot.
  uint4 kr[NPC], vr[NPC];
#pragma unroll
  for (int it = 0; it < NPC; ++it) kr[it] = vr[it] = make_uint4(0, 0, 0, 0);
  auto request_tile = [&](int t) {
    if (t >= t_end) return;   // uniform per wave
    const bool tree_tile = t >= n_pt;
    const int kbase = tree_tile ? (t - n_pt) * KT : t * KT;
    const int last = (tree_tile ? T : P) - 1;   // >= 0: a tile exists only if its source has keys
    const uint16_t* ksrc = tree_tile ? ktr : kc;
    const uint16_t* vsrc = tree_tile ? vtr : vc;
    const int64_t pitch = tree_tile ? tree_pitch : p.sp;
#pragma unroll
    for (int it = 0; it < NPC; ++it) {
      const int c = gl + 256 * it, key = c / DC, dc = c % DC;
      const int64_t o = (int64_t)min(kbase + key, last) * pitch + 8 * dc;
      kr[it] = *(const uint4*)(ksrc + o);
      vr[it] = *(const uint4*)(vsrc + o);
    }
  };
  request_tile(t_begin + kg);   // first round's tile: in flight while queries and parents are fetched

  if (t_end > n_pt) {
    for (int i = tid; i < T; i += NT) {
      int pi = p.parent[lo + i];
      if (pi >= i || pi < -1 || (i == 0 && pi != -1) || (i > 0 && pi < 0)) {
        atomicOr(p.dev_status, CASCADE_FLAG_PARENT);
        pi = (i == 0) ? -1 : 0;
      }
      s_parent[i] = pi;
    }
  }

  // this wave's 16 query rows (B operand of S^T): lane = (query l16, d group g)
  Frag8 qf[KS];
  const int qr = row0 + 16 * qb + l16;
  const bool q_ok = qr < M;
  {
    const int i = q_ok ? qr % T : 0, hg = q_ok ? qr / T : 0;
    const uint16_t* qp = (const uint16_t*)p.q + ((int64_t)(lo + i) * p.n_heads + kvh * G + hg) * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (q_ok) qf[ks].u = *(const uint4*)(qp + 32 * ks);
      else qf[ks].u = make_uint4(0, 0, 0, 0);
    }
  }
  f32x4 ot[DB];
  float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int db = 0; db < DB; ++db) ot[db] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int r = 0; r < n_rounds; ++r) {
    const int t = t_begin + NKG * r + kg;
    const bool active = t < t_end;
    const bool tree_tile = t >= n_pt;
    const int kbase = tree_tile ? (t - n_pt) * KT : t * KT;
    const int klimit = tree_tile ? T : P;
    __syncthreads();   // the previous pass's tiles are consumed (and, before the first pass, the parent array is complete)
#pragma unroll
    for (int it = 0; it < NPC; ++it) {
      const int c = gl + 256 * it, key = c / DC, dc = c % DC;
      *(uint4*)(&gs->k[key * GS::KP + 8 * dc]) = kr[it];
      *(uint4*)(&gs->v[key * GS::VP + 8 * dc]) = vr[it];
    }
    if (active && tree_tile && qb == 0) {
      // ancestor-or-self bits of this tile's 64 tree keys for query row (row0 + lane)
      const int rr = row0 + lane;
      unsigned long long wbits = 0ull;
      if (rr < M) {
        int a = rr % T, guard = 0;
        while (a >= 0 && guard++ <= CASCADE_MAX_TREE) {
          const int rel = a - kbase;
          if (rel < 0) break;
          if (rel < 64) wbits |= 1ull << rel;
          a = s_parent[a];
        }
      }
      s_anc[lane] = wbits;
    }
    request_tile(t + NKG);   // next round streams in while this one is consumed
    __syncthreads();
    if (!active) continue;

    // S^T = K Q^T : st[kt] holds keys 16*kt + 4*g + c for query l16
    f32x4 st[4];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
      st[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Frag8 kf;
        kf.u = *(const uint4*)(&gs->k[(16 * kt + l16) * GS::KP + 32 * ks + 8 * g]);
        st[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, qf[ks].v, st[kt], 0, 0, 0);
      }
    }
    unsigned long long valid;
    if (tree_tile) {
      valid = s_anc[16 * qb + l16];
    } else {
      const int rem = klimit - kbase;
      valid = rem >= 64 ? ~0ull : ((1ull << rem) - 1ull);
    }
    if (!q_ok) valid = 0ull;
    float mx = -INFINITY;
    if (__ballot(valid != ~0ull) == 0ull) {
      // every key of the tile is visible to every query of the block: no masking
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          st[kt][c] *= p.scale_log2e;
          mx = fmaxf(mx, st[kt][c]);
        }
    } else {
#pragma unroll
      for (int kt = 0; kt < 4; ++kt) {
        const uint32_t nib = (uint32_t)(valid >> (16 * kt + 4 * g));   // this lane's 4 keys of sub-tile kt
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float z = ((nib >> c) & 1u) ? st[kt][c] * p.scale_log2e : -INFINITY;
          st[kt][c] = z;
          mx = fmaxf(mx, z);
        }
      }
    }
    mx = rows4_max(mx);
    const float m_new = fmaxf(m_run, mx);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(m_run - m_use);
    float ls = 0.f;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float e = fast_exp2(st[kt][c] - m_use);
        st[kt][c] = e;
        ls += e;
      }
    l_run = l_run * alpha + ls;
    m_run = m_new;
#pragma unroll
    for (int db = 0; db < DB; ++db) ot[db] *= alpha;
    Frag8 pf[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      pf[j].u.x = pack_bf16x2(st[2 * j][0], st[2 * j][1]);
      pf[j].u.y = pack_bf16x2(st[2 * j][2], st[2 * j][3]);
      pf[j].u.z = pack_bf16x2(st[2 * j + 1][0], st[2 * j + 1][1]);
      pf[j].u.w = pack_bf16x2(st[2 * j + 1][2], st[2 * j + 1][3]);
    }
    // O^T += V^T P^T.  Operand slots of lane (l16, g): keys 32j + 4g + {0..3} and 32j + 16 + 4g + {0..3}
    // at d = 16 db + l16, fetched by two transposing loads from the row-major V tile.
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const uint16_t* vp = &gs->v[(32 * j + 4 * g + (l16 >> 2)) * GS::VP + 16 * db + 4 * (l16 & 3)];
        union { Frag8 f; s16x4 h[2]; } vf;
        vf.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp));
        vf.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp + 16 * GS::VP));
        ot[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.f.v, pf[j].v, ot[db], 0, 0, 0);
      }
    }
  }

  l_run = rows4_sum(l_run);
  if (NKG == 1) {
    // one key group: nothing to merge - every wave writes its 16 rows from its registers (lane (l16, g) owns
    // d = 16 db + 4 g + c of query l16), no LDS round trip and no barrier
    if (q_ok) {
      const int i = qr % T, hg = qr / T;
      const int64_t rowg = (int64_t)(lo + i) * p.n_heads + kvh * G + hg;
      if (SPLIT) {
        float* wo = p.ws_o + ((int64_t)split * p.n_rows_total + rowg) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db) *(f32x4*)(wo + 16 * db + 4 * g) = ot[db];
        if (g == 0) {
          float* wm = p.ws_ml + ((int64_t)split * p.n_rows_total + rowg) * 2;
          wm[0] = m_run;
          wm[1] = l_run;
        }
      } else {
        const float inv = 1.f / l_run;
        uint16_t* op = (uint16_t*)p.out + rowg * D;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          uint2 w2;
          w2.x = pack_bf16x2(ot[db][0] * inv, ot[db][1] * inv);
          w2.y = pack_bf16x2(ot[db][2] * inv, ot[db][3] * inv);
          *(uint2*)(op + 16 * db + 4 * g) = w2;
        }
        if (g == 0 && p.lse) p.lse[rowg] = m_run * LN2 + logf(l_run);
      }
    }
    return;
  }
  // merge the key groups through LDS (the tile buffers are reused)
  __syncthreads();
  float* mo = (float*)smem_raw;                 // [NKG][64 rows][OP]
  float* mml = mo + NKG * 64 * OP;              // [NKG][64 rows][2]
  {
    float* orow = mo + ((kg * 64) + 16 * qb + l16) * OP;
#pragma unroll
    for (int db = 0; db < DB; ++db) *(f32x4*)(orow + 16 * db + 4 * g) = ot[db];
    if (g == 0) {
      mml[((kg * 64) + 16 * qb + l16) * 2] = m_run;
      mml[((kg * 64) + 16 * qb + l16) * 2 + 1] = l_run;
    }
  }
  __syncthreads();
  {
    constexpr int TPR = NT / 64;                 // threads per output row
    constexpr int DQ = D / TPR;                  // d range of one thread
    const int row = tid / TPR, dq = tid % TPR;
    const int rr = row0 + row;
    if (rr < M) {
      float mw[NKG], m = -INFINITY;
#pragma unroll
      for (int w = 0; w < NKG; ++w) { mw[w] = mml[(w * 64 + row) * 2]; m = fmaxf(m, mw[w]); }
      float l = 0.f, o[DQ];
#pragma unroll
      for (int d = 0; d < DQ; ++d) o[d] = 0.f;
#pragma unroll
      for (int w = 0; w < NKG; ++w) {
        if (mw[w] == -INFINITY) continue;
        const float sc = fast_exp2(mw[w] - m);
        l += sc * mml[(w * 64 + row) * 2 + 1];
        const float* orow = mo + (w * 64 + row) * OP + DQ * dq;
#pragma unroll
        for (int d = 0; d < DQ; d += 4) {
          const f32x4 v4 = *(const f32x4*)(orow + d);
          o[d] += sc * v4[0]; o[d + 1] += sc * v4[1]; o[d + 2] += sc * v4[2]; o[d + 3] += sc * v4[3];
        }
      }
      const int i = rr % T, hg = rr / T;
      const int64_t rowg = (int64_t)(lo + i) * p.n_heads + kvh * G + hg;
      if (SPLIT) {
        float* wo = p.ws_o + ((int64_t)split * p.n_rows_total + rowg) * D + DQ * dq;
#pragma unroll
        for (int d = 0; d < DQ; d += 4) *(f32x4*)(wo + d) = f32x4{o[d], o[d + 1], o[d + 2], o[d + 3]};
        if (dq == 0) {
          float* wm = p.ws_ml + ((int64_t)split * p.n_rows_total + rowg) * 2;
          wm[0] = m;
          wm[1] = l;
        }
      } else {
        const float inv = 1.f / l;
        uint16_t* op = (uint16_t*)p.out + rowg * D + DQ * dq;
#pragma unroll
        for (int d = 0; d < DQ; d += 4) {
          uint2 w2;
          w2.x = pack_bf16x2(o[d] * inv, o[d + 1] * inv);
          w2.y = pack_bf16x2(o[d + 2] * inv, o[d + 3] * inv);
          *(uint2*)(op + d) = w2;
        }
        if (dq == 0 && p.lse) p.lse[rowg] = m * LN2 + logf(l);
      }
    }
  }
}

// ---------------------------------------------------------------------- bf16, few query rows
// When a step has so few (row, kv head, 64-query block) units that they cannot fill the GPU, the
// query rows are split instead of the keys: workgroup = (row, kv head, 16 query rows), eight
// waves, wave w owning the 64-key tiles w, w + 8, ... of the whole key range.  A wave keeps its
// tile to itself: K is loaded from global memory directly in MFMA operand order (16-byte pieces of
// one key row per lane), V goes through a wave-private LDS region only to be read back transposed.
// No workgroup barrier inside the tile loop; the eight (m, l, O) partials are merged through LDS at
// the end.  Keys and values are read by every query block of a (row, kv head) - from L2.
template <int D>
__global__ __launch_bounds__(512) void attn_bf16_qsplit_kernel(AttnParams p) {
  constexpr int NWV = 8, NT = 512;
  constexpr int KS = D / 32, DB = D / 16, DC = D / 8;
  constexpr int VP = D + 16;           // V row pitch (elements), as in the other kernels
  constexpr int OP = D + 4;            // merge buffer row pitch (floats)
  constexpr int NVC = KT * DC / 64;    // 16-byte pieces of V per lane per tile
  extern __shared__ __align__(16) char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  uint16_t* vt = (uint16_t*)smem_raw + (size_t)wave * KT * VP;                         // this wave's V tile
  int* s_parent = (int*)(smem_raw + (size_t)NWV * KT * VP * sizeof(uint16_t));         // [128]
  unsigned long long* s_anc = (unsigned long long*)(s_parent + 128);                   // [2 tree tiles][16 rows]

  // the query blocks of a (row, kv head) share an L2
  const unsigned nx = gridDim.x, ny = gridDim.y;
  const unsigned lid = xcd_local_order(blockIdx.x + nx * (blockIdx.y + ny * blockIdx.z), nx, ny * gridDim.z);
  const int sb = (int)(lid % nx), kvh = (int)((lid / nx) % ny), s = (int)(lid / (nx * ny));
  const int lo = p.node_off[s];
  const int T = p.node_off[s + 1] - lo;
  const int P = p.prefix_len[s];
  const int G = p.group;
  const int M = T * G;
  const int row0 = sb * 16;
  if (T > p.max_tree) { skip_oversize_row<D, false>(p, lo, T, kvh, sb, 0, tid, NT); return; }
  if (row0 >= M || T > 128) return;
  const int n_pt = (P + KT - 1) / KT, n_tt = (T + KT - 1) / KT, nt = n_pt + n_tt;

  const uint16_t* kc = (const uint16_t*)p.k_cache + s * p.sr + kvh * p.sh;
  const uint16_t* vc = (const uint16_t*)p.v_cache + s * p.sr + kvh * p.sh;
  const uint16_t* ktr = (const uint16_t*)p.k_tree + ((int64_t)lo * p.n_kv_heads + kvh) * D;
  const uint16_t* vtr = (const uint16_t*)p.v_tree + ((int64_t)lo * p.n_kv_heads + kvh) * D;
  const int64_t tree_pitch = (int64_t)p.n_kv_heads * D;

  // tile registers: K fragments kf[kt][ks] = key 16 kt + l16, d 32 ks + 8 g .. + 7 ; V pieces c = lane + 64 it
  u32x4 kf[4][KS], vr[NVC];
  auto request_tile = [&](int t) {
    const bool tree_tile = t >= n_pt;
    const int kbase = tree_tile ? (t - n_pt) * KT : t * KT;
    const int klimit = tree_tile ? T : P;
    const uint16_t* ksrc = tree_tile ? ktr : kc;
    const uint16_t* vsrc = tree_tile ? vtr : vc;
    const int64_t pitch = tree_tile ? tree_pitch : p.sp;
    // Keys past the end of the tile's source are read from its last row (clamped: always in bounds)
    // and are NOT zeroed here: their scores are masked to -inf below, so their probabilities are
    // exactly 0 and the clamped (finite) K and V rows contribute nothing.  A select on the loaded
    // value would make the compiler wait for every load right here, before the next one is issued.
    const int last = max(klimit - 1, 0);
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
      const int key = kbase + 16 * kt + l16;
      const uint16_t* kp = ksrc + (int64_t)min(key, last) * pitch + 8 * g;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[kt][ks] = *(const u32x4*)(kp + 32 * ks);
    }
#pragma unroll
    for (int it = 0; it < NVC; ++it) {
      const int c = lane + 64 * it, key = kbase + c / DC, dc = c % DC;
      vr[it] = *(const u32x4*)(vsrc + (int64_t)min(key, last) * pitch + 8 * dc);
    }
  };
  for (int i = tid; i < T; i += NT) {
    int pi = p.parent[lo + i];
    if (pi >= i || pi < -1 || (i == 0 && pi != -1) || (i > 0 && pi < 0)) {
      atomicOr(p.dev_status, CASCADE_FLAG_PARENT);
      pi = (i == 0) ? -1 : 0;
    }
    s_parent[i] = pi;
  }

  // the workgroup's 16 query rows (B operand of S^T): lane = (query l16, d group g)
  Frag8 qf[KS];
  const int qr = row0 + l16;
  const bool q_ok = qr < M;
  const int qi = q_ok ? qr % T : 0, qh = q_ok ? qr / T : 0;
  const int64_t rowg = (int64_t)(lo + qi) * p.n_heads + kvh * G + qh;
  {
    const uint16_t* qp = (const uint16_t*)p.q + rowg * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (q_ok) qf[ks].u = *(const uint4*)(qp + 32 * ks);
      else qf[ks].u = make_uint4(0, 0, 0, 0);
    }
  }
  // The first tile is requested AFTER the parent and query loads: loads return in order, so the wait
  // for the parent entry below then leaves the 32 tile loads in flight instead of draining them.
  const bool has_keys = P > 0 || T > 0;   // T >= 1 for a row that reaches this point
  if (wave < nt && has_keys) request_tile(wave);
  __syncthreads();   // parent array complete
  if (tid < 32) {
    // ancestor-or-self bits of the (at most two) tree tiles for the 16 query rows
    const int tt = tid >> 4, rr = row0 + (tid & 15), kbase = tt * KT;
    unsigned long long wbits = 0ull;
    if (rr < M && tt < n_tt) {
      int a = rr % T, guard = 0;
      while (a >= 0 && guard++ <= 128) {
        const int rel = a - kbase;
        if (rel < 0) break;
        if (rel < 64) wbits |= 1ull << rel;
        a = s_parent[a];
      }
    }
    s_anc[tid] = wbits;
  }
  __syncthreads();

  f32x4 ot[DB];
  float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int db = 0; db < DB; ++db) ot[db] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int t = wave; t < nt; t += NWV) {
    const bool tree_tile = t >= n_pt;
    const int kbase = tree_tile ? (t - n_pt) * KT : t * KT;
    const int klimit = tree_tile ? T : P;
    // S^T = K Q^T from the register fragments (K was requested before V and arrives first)
    f32x4 st[4];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
      st[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Frag8 a8;
        a8.u = make_uint4(kf[kt][ks][0], kf[kt][ks][1], kf[kt][ks][2], kf[kt][ks][3]);
        st[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8.v, qf[ks].v, st[kt], 0, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    // V: registers -> this wave's LDS tile (row-major); the previous tile's reads are complete (same wave, in order)
#pragma unroll
    for (int it = 0; it < NVC; ++it) {
      const int c = lane + 64 * it;
      *(u32x4*)(&vt[(c / DC) * VP + 8 * (c % DC)]) = vr[it];
    }
    __builtin_amdgcn_wave_barrier();   // keep the tile's stores ahead of its transposing reads in program order
    if (t + NWV < nt) request_tile(t + NWV);   // next tile of this wave streams in during the softmax

    unsigned long long valid;
    if (tree_tile) {
      valid = s_anc[16 * (t - n_pt) + l16];
    } else {
      const int rem = klimit - kbase;
      valid = rem >= 64 ? ~0ull : ((1ull << rem) - 1ull);
    }
    if (!q_ok) valid = 0ull;
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
      const uint32_t nib = (uint32_t)(valid >> (16 * kt + 4 * g));   // this lane's 4 keys of sub-tile kt
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float z = ((nib >> c) & 1u) ? st[kt][c] * p.scale_log2e : -INFINITY;
        st[kt][c] = z;
        mx = fmaxf(mx, z);
      }
    }
    mx = rows4_max(mx);
    const float m_new = fmaxf(m_run, mx);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(m_run - m_use);
    float ls = 0.f;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float e = fast_exp2(st[kt][c] - m_use);
        st[kt][c] = e;
        ls += e;
      }
    l_run = l_run * alpha + ls;
    m_run = m_new;
#pragma unroll
    for (int db = 0; db < DB; ++db) ot[db] *= alpha;
    Frag8 pf[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      pf[j].u.x = pack_bf16x2(st[2 * j][0], st[2 * j][1]);
      pf[j].u.y = pack_bf16x2(st[2 * j][2], st[2 * j][3]);
      pf[j].u.z = pack_bf16x2(st[2 * j + 1][0], st[2 * j + 1][1]);
      pf[j].u.w = pack_bf16x2(st[2 * j + 1][2], st[2 * j + 1][3]);
    }
    // O^T += V^T P^T with transposing reads of the wave's V tile (LDS operations of one wave complete in order)
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const uint16_t* vp = &vt[(32 * j + 4 * g + (l16 >> 2)) * VP + 16 * db + 4 * (l16 & 3)];
        union { Frag8 f; s16x4 h[2]; } vf;
        vf.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp));
        vf.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp + 16 * VP));
        ot[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.f.v, pf[j].v, ot[db], 0, 0, 0);
      }
    }
    __builtin_amdgcn_wave_barrier();   // and the reads ahead of the next tile's stores
  }

  // merge the eight waves' partials through LDS (the V tiles are reused)
  l_run = rows4_sum(l_run);
  __syncthreads();
  float* mo = (float*)smem_raw;                 // [NWV][16 rows][OP]
  float* mml = mo + NWV * 16 * OP;              // [NWV][16 rows][2]
  {
    float* orow = mo + (wave * 16 + l16) * OP;
#pragma unroll
    for (int db = 0; db < DB; ++db) *(f32x4*)(orow + 16 * db + 4 * g) = ot[db];
    if (g == 0) {
      mml[(wave * 16 + l16) * 2] = m_run;
      mml[(wave * 16 + l16) * 2 + 1] = l_run;
    }
  }
  __syncthreads();
  {
    constexpr int TPR = NT / 16;                 // threads per output row
    constexpr int DQ = D / TPR;                  // d range of one thread (4 for D = 128, 2 for D = 64)
    const int row = tid / TPR, dq = tid % TPR;
    const int rr = row0 + row;
    if (rr < M) {
      float mw[NWV], m = -INFINITY;
#pragma unroll
      for (int w = 0; w < NWV; ++w) { mw[w] = mml[(w * 16 + row) * 2]; m = fmaxf(m, mw[w]); }
      float l = 0.f, o[DQ];
#pragma unroll
      for (int d = 0; d < DQ; ++d) o[d] = 0.f;
#pragma unroll
      for (int w = 0; w < NWV; ++w) {
        if (mw[w] == -INFINITY) continue;
        const float sc = fast_exp2(mw[w] - m);
        l += sc * mml[(w * 16 + row) * 2 + 1];
        const float* orow = mo + (w * 16 + row) * OP + DQ * dq;
#pragma unroll
        for (int d = 0; d < DQ; ++d) o[d] += sc * orow[d];
      }
      const int i = rr % T, hg = rr / T;
      const int64_t rg = (int64_t)(lo + i) * p.n_heads + kvh * G + hg;
      const float inv = 1.f / l;
      uint16_t* op = (uint16_t*)p.out + rg * D + DQ * dq;
#pragma unroll
      for (int d = 0; d < DQ; d += 2) *(uint32_t*)(op + d) = pack_bf16x2(o[d] * inv, o[d + 1] * inv);
      if (dq == 0 && p.lse) p.lse[rg] = m * LN2 + logf(l);
    }
  }
}

// log-sum-exp merge of the split partials: D/4 lanes per output row (a float4 each), 256 threads
template <int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnParams p) {
  constexpr int LPR = D / 4;             // lanes per row
  constexpr int RPB = 256 / LPR;         // rows per block
  const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / LPR;
  const int d4 = threadIdx.x % LPR;
  if (row >= p.n_rows_total) return;
  float m = -INFINITY;
  for (int c = 0; c < p.n_split; ++c) m = fmaxf(m, p.ws_ml[((int64_t)c * p.n_rows_total + row) * 2]);
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
  for (int c = 0; c < p.n_split; ++c) {
    const float* ml = p.ws_ml + ((int64_t)c * p.n_rows_total + row) * 2;
    const float mc = ml[0];
    if (mc == -INFINITY) continue;
    const float w = exp2f(mc - m);
    l += w * ml[1];
    o += w * *(const f32x4*)(p.ws_o + ((int64_t)c * p.n_rows_total + row) * D + 4 * d4);
  }
  const float inv = l > 0.f ? 1.f / l : 0.f;   // a skipped row (every partial empty) comes out as zeros, lse = -inf
  uint2 packed;
  packed.x = pack_bf16x2(o[0] * inv, o[1] * inv);
  packed.y = pack_bf16x2(o[2] * inv, o[3] * inv);
  *(uint2*)((uint16_t*)p.out + row * D + 4 * d4) = packed;
  if (d4 == 0 && p.lse) p.lse[row] = m * LN2 + logf(l);
}

AttnParams make_params(cascade_ctx* ctx, const tree_attn_args* a) {
  AttnParams p;
  p.node_off = a->node_off;
  p.parent = a->parent;
  p.prefix_len = a->prefix_len;
  p.q = a->q;
  p.k_tree = a->k_tree;
  p.v_tree = a->v_tree;
  p.k_cache = a->k_cache;
  p.v_cache = a->v_cache;
  p.sr = a->cache_stride_row;
  p.sh = a->cache_stride_head;
  p.sp = a->cache_stride_pos;
  p.out = a->out;
  p.lse = a->lse;
  p.ws_o = nullptr;
  p.ws_ml = nullptr;
  p.dev_status = ctx->dev_status;
  p.n_heads = a->n_heads;
  p.n_kv_heads = a->n_kv_heads;
  p.group = a->n_heads / a->n_kv_heads;
  p.n_split = 1;
  p.n_sb = 1;
  p.n_rows_total = a->n_nodes_total * a->n_heads;
  p.max_tree = a->max_nodes_per_tree;
  const float scale = a->scale != 0.f ? a->scale : 1.f / sqrtf((float)a->head_dim);
  p.scale_log2e = scale * LOG2E;
  return p;
}

// whole rows of keys per workgroup (n_split == 1): the ring kernel
template <int D>
hipError_t launch_ring_t(cascade_ctx* ctx, AttnParams& p, dim3 grid) {
  constexpr int NS = 3;
  const size_t smem = 2 * NS * RingGeom<D>::TILE + CASCADE_MAX_TREE * sizeof(int) + 2 * 256 * sizeof(unsigned long long);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_bf16_ring_kernel<D, NS>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  KernelTimer t(ctx, CASCADE_K_ATTN);
  CASCADE_TIMED_LAUNCH(t, (attn_bf16_ring_kernel<D, NS>), grid, dim3(512), smem, ctx->stream, p);
  return hipGetLastError();
}

// keys split across workgroups (n_split > 1): partials, then the merge kernel
template <int D, int NQ, int NW>
hipError_t launch_split_t(cascade_ctx* ctx, AttnParams& p, dim3 grid) {
  hipStream_t st = ctx->stream;
  const size_t smem = 2 * sizeof(TileSmem<D>) + CASCADE_MAX_TREE * sizeof(int) + 2 * 256 * sizeof(unsigned long long);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_bf16_kernel<D, NQ, NW, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  {
    KernelTimer t(ctx, CASCADE_K_ATTN);
    CASCADE_TIMED_LAUNCH(t, (attn_bf16_kernel<D, NQ, NW, true>), grid, dim3(64 * NW), smem, st, p);
  }
  KernelTimer t(ctx, CASCADE_K_ATTN_MERGE);
  CASCADE_TIMED_LAUNCH(t, (attn_merge_kernel<D>), dim3((p.n_rows_total + (1024 / D) - 1) / (1024 / D)), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_tree_attn_f32(cascade_ctx* ctx, const tree_attn_args* a) {
  AttnParams p = make_params(ctx, a);
  dim3 grid(a->n_nodes_total, a->n_heads);
  KernelTimer t(ctx, CASCADE_K_ATTN);
  CASCADE_TIMED_LAUNCH(t, (attn_f32_kernel<256>), grid, dim3(256), 0, ctx->stream, p, a->n_rows, a->head_dim);
  return hipGetLastError();
}

// CAN_SPLIT: the dispatcher may split the keys across workgroups for this instantiation (it never does when
// there are two or more workgroups per compute unit anyway, so those partial-writing variants are not built)
template <int D, int NKG, bool CAN_SPLIT>
hipError_t launch_ksplit_t(cascade_ctx* ctx, AttnParams& p, dim3 grid) {
  hipStream_t st = ctx->stream;
  const size_t smem = NKG * sizeof(KsplitGroupSmem<D>) + CASCADE_MAX_TREE * sizeof(int) + NKG * 64 * sizeof(unsigned long long);
  static_assert(NKG * 64 * (D + 4) * 4 + NKG * 64 * 2 * 4 <= NKG * sizeof(KsplitGroupSmem<D>), "merge buffers fit in the tile buffers");
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_bf16_ksplit_kernel<D, NKG, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if constexpr (CAN_SPLIT) {
      if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_bf16_ksplit_kernel<D, NKG, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    }
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  if (p.n_split > 1) {
    if constexpr (CAN_SPLIT) {
      {
        KernelTimer t(ctx, CASCADE_K_ATTN);
        CASCADE_TIMED_LAUNCH(t, (attn_bf16_ksplit_kernel<D, NKG, true>), grid, dim3(NKG * 256), smem, st, p);
      }
      KernelTimer t(ctx, CASCADE_K_ATTN_MERGE);
      CASCADE_TIMED_LAUNCH(t, (attn_merge_kernel<D>), dim3((p.n_rows_total + (1024 / D) - 1) / (1024 / D)), dim3(256), 0, st, p);
    } else {
      return hipErrorInvalidValue;   // the dispatcher never asks for it
    }
  } else {
    KernelTimer t(ctx, CASCADE_K_ATTN);
    CASCADE_TIMED_LAUNCH(t, (attn_bf16_ksplit_kernel<D, NKG, false>), grid, dim3(NKG * 256), smem, st, p);
  }
  return hipGetLastError();
}

template <int D>
hipError_t launch_qsplit_t(cascade_ctx* ctx, AttnParams& p, dim3 grid) {
  constexpr int VP = D + 16;
  const size_t smem = (size_t)8 * KT * VP * sizeof(uint16_t) + 128 * sizeof(int) + 32 * sizeof(unsigned long long);
  static_assert(8 * 16 * (D + 4) * 4 + 8 * 16 * 2 * 4 <= 8 * KT * (D + 16) * 2, "merge buffers fit in the V tiles");
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_bf16_qsplit_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  KernelTimer t(ctx, CASCADE_K_ATTN);
  CASCADE_TIMED_LAUNCH(t, (attn_bf16_qsplit_kernel<D>), grid, dim3(512), smem, ctx->stream, p);
  return hipGetLastError();
}

hipError_t launch_tree_attn_bf16(cascade_ctx* ctx, const tree_attn_args* a) {
  AttnParams p = make_params(ctx, a);
  const int M = a->max_nodes_per_tree * p.group;   // query rows per (row, kv head)
  const int n_tiles = (a->max_prefix_len + KT - 1) / KT + (a->max_nodes_per_tree + KT - 1) / KT;
  const size_t per_split = (size_t)p.n_rows_total * (a->head_dim + 2) * sizeof(float);
  if (M <= 128 && (long)a->n_rows * a->n_kv_heads * ((M + 63) / 64) <= 128 && a->max_nodes_per_tree <= 128) {
    // too few 64-row units to fill the GPU: split the query rows, not the keys (no partials, no merge kernel)
    p.n_sb = (M + 15) / 16;
    dim3 grid(p.n_sb, a->n_kv_heads, a->n_rows);
    return a->head_dim == 128 ? launch_qsplit_t<128>(ctx, p, grid) : launch_qsplit_t<64>(ctx, p, grid);
  }
  if (M <= 128) {
    // small trees: key groups split the tiles inside the workgroup; split across workgroups only when a
    // workgroup would otherwise walk more than 16 tiles (4 rounds) and the GPU is not yet full
    p.n_sb = (M + 63) / 64;
    const long base_wgs = (long)a->n_rows * a->n_kv_heads * p.n_sb;
    int n_split = (n_tiles + 15) / 16;
    const int fill = (int)((512 + base_wgs - 1) / base_wgs);
    if (n_split > fill) n_split = fill;
    if (n_split > 16) n_split = 16;
    if (n_split > 1 && per_split * n_split > ctx->attn_ws_bytes) n_split = (int)(ctx->attn_ws_bytes / per_split);
    if (n_split < 1) n_split = 1;
    p.n_split = n_split;
    if (n_split > 1) {
      p.ws_o = (float*)ctx->attn_ws;
      p.ws_ml = (float*)(ctx->attn_ws + (size_t)n_split * p.n_rows_total * a->head_dim * sizeof(float));
    }
    dim3 grid(n_split * p.n_sb, a->n_kv_heads, a->n_rows);
    // key groups per workgroup: two (head_dim 128: 8 waves, 2 workgroups per CU) or four (head_dim 64) when
    // workgroups are scarce; half as many when there are at least two per CU anyway - smaller workgroups,
    // four resident per CU, hide each other's tile latencies better (54 -> 46 us at 16 rows x 32 heads)
    const bool many = base_wgs >= 512;
    // (many => fill == 1 => n_split == 1 above)
    if (a->head_dim == 128) return many ? launch_ksplit_t<128, 1, false>(ctx, p, grid) : launch_ksplit_t<128, 2, true>(ctx, p, grid);
    return many ? launch_ksplit_t<64, 2, false>(ctx, p, grid) : launch_ksplit_t<64, 4, true>(ctx, p, grid);
  }
  // large trees: NW waves x 2 query blocks each share every K/V tile through LDS
  // (measured at 8 rows x 32 heads x 256 nodes, 4200-key prefix: 283 us with 4 waves x 4 blocks and
  // one workgroup per CU, 217 us with 4 waves x 2 blocks and two workgroups per CU, 196 us with 8 waves
  // x 2 blocks sharing one copy of every tile)
  constexpr int NW = 8;
  const int RW = 32 * NW;
  p.n_sb = (M + RW - 1) / RW;
  const long base_wgs = (long)a->n_rows * a->n_kv_heads * p.n_sb;
  // two workgroups of four waves (or one of eight) are resident per CU: split only to fill those slots
  const long slots = NW == 8 ? 256 : 512;
  int n_split = (int)(slots / base_wgs);
  if (n_split > n_tiles) n_split = n_tiles;
  if (n_split > 16) n_split = 16;
  if (n_split > 1 && per_split * n_split > ctx->attn_ws_bytes) n_split = (int)(ctx->attn_ws_bytes / per_split);
  if (n_split < 1) n_split = 1;
  p.n_split = n_split;
  if (n_split > 1) {
    p.ws_o = (float*)ctx->attn_ws;
    p.ws_ml = (float*)(ctx->attn_ws + (size_t)n_split * p.n_rows_total * a->head_dim * sizeof(float));
  }
  dim3 grid(n_split * p.n_sb, a->n_kv_heads, a->n_rows);
  // Both kernels cover 256 query rows per workgroup.  With whole rows of keys per workgroup the ring kernel runs
  // (tiles straight into LDS, three deep); when the keys are split to fill an otherwise idle GPU, the older
  // double-buffered kernel writes the partials (the ring kernel's register budget has no room for that epilogue).
  if (n_split > 1) return a->head_dim == 128 ? launch_split_t<128, 2, NW>(ctx, p, grid) : launch_split_t<64, 2, NW>(ctx, p, grid);
  return a->head_dim == 128 ? launch_ring_t<128>(ctx, p, grid) : launch_ring_t<64>(ctx, p, grid);
}
