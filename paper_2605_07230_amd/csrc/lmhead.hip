// lmhead_softmax_cfg kernels for gfx950: final projection with the guidance mix in the epilogue
// (Sec. 4.2: the O(hV) projection dominates; App. "Configuration Details": guidance scale,
// temperature, top-k), then one kernel for the per-row softmax statistics.
//
// bf16 projection: a workgroup owns 64 vocabulary columns x 64 nodes (conditional and
// unconditional rows of the same nodes, so the mix happens in registers).  Its four waves split
// the hidden dimension; every wave streams its own slices of W and H straight from global memory
// into v_mfma_f32_32x32x16_bf16 operand registers (both operands are k-contiguous, so a lane's
// 8 operand values are one 16-byte load) and the four partial tiles are summed through LDS once
// at the end.  Nothing is shared between waves inside the main loop, so it has no barriers.
#include "common.h"

namespace {

struct LmParams {
  const void* h_cond;
  const void* h_uncond;
  const void* w;
  float* logits;
  float* row_max;
  float* row_thr;
  float* row_lse;
  const uint4* hp_cond;     // packed hidden states (MFMA operand order), when the packed path runs
  const uint4* hp_uncond;
  int n_nodes, hidden, vocab;
  int n_mchunks;
  float cfg_scale, temperature;
  int top_k;
};

// ------------------------------------------------------------------------------------------ f32
// grid (ceil(V/256), N); the two hidden-state rows sit in LDS, a thread owns one vocabulary entry.
__global__ __launch_bounds__(256) void lmhead_f32_kernel(LmParams p) {
  extern __shared__ float hs[];
  const int node = blockIdx.y, v = blockIdx.x * 256 + threadIdx.x;
  const int K = p.hidden;
  const bool cfg = p.h_uncond != nullptr;
  const float* hc = (const float*)p.h_cond + (int64_t)node * K;
  const float* hu = cfg ? (const float*)p.h_uncond + (int64_t)node * K : nullptr;
  for (int k = threadIdx.x; k < K; k += 256) {
    hs[k] = hc[k];
    if (cfg) hs[K + k] = hu[k];
  }
  __syncthreads();
  if (v >= p.vocab) return;
  const float* wr = (const float*)p.w + (int64_t)v * K;
  float lc = 0.f, lu = 0.f;
  for (int k = 0; k < K; ++k) {
    const float wv = wr[k];
    lc = fmaf(hs[k], wv, lc);
    if (cfg) lu = fmaf(hs[K + k], wv, lu);
  }
  float gmix = cfg ? lu + p.cfg_scale * (lc - lu) : lc;
  p.logits[(int64_t)node * p.vocab + v] = gmix / p.temperature;
}

// ----------------------------------------------------------------------------------------- bf16
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
union Frag8 {
  bf16x8 v;
  uint4 u;
  u32x4 n;
};

template <bool CFG>
struct Group {   // operands of 4 consecutive k16 steps
  static constexpr int NA = CFG ? 4 : 2;
  Frag8 a[4][NA];
  Frag8 b[4][2];
};

template <bool CFG>
__global__ __launch_bounds__(256) void lmhead_bf16_kernel(LmParams p) {
  constexpr int NA = CFG ? 4 : 2;   // 32-row operand blocks: cond0, cond1, (uncond0, uncond1)
  extern __shared__ float red[];    // [4 waves][NA*2 acc][16 regs][64 lanes]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r32 = lane & 31, half = lane >> 5;
  const int K = p.hidden;

  // XCD-aware order: the 8 XCDs take workgroups round-robin; give each XCD a contiguous range of
  // logical ids so that the m-chunks sharing one W tile meet in the same L2.
  int logical = blockIdx.x;
  const int nwg = gridDim.x;
  if ((nwg & 7) == 0) logical = (blockIdx.x & 7) * (nwg >> 3) + (blockIdx.x >> 3);
  const int ntile = logical / p.n_mchunks, mc = logical % p.n_mchunks;
  const int v0 = ntile * 64, node0 = mc * 64;

  const uint16_t* ap[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int node = min(node0 + 32 * (i & 1) + r32, p.n_nodes - 1);   // rows past the end are clamped, never stored
    const uint16_t* base = (i < 2) ? (const uint16_t*)p.h_cond : (const uint16_t*)p.h_uncond;
    ap[i] = base + (int64_t)node * K + 8 * half;
  }
  const uint16_t* bp[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) bp[j] = (const uint16_t*)p.w + (int64_t)(v0 + 32 * j + r32) * K + 8 * half;

  f32x16 acc[NA][2];
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // this wave's k groups (64 wide): 128-wide slices wave, wave+4, ... of the hidden dimension
  const int n_slices = (K / 128 - wave + 3) / 4;   // K is a multiple of 128
  const int n_groups = 2 * n_slices;
  auto k_of = [&](int gi) { return (wave + 4 * (gi >> 1)) * 128 + 64 * (gi & 1); };
  auto load_group = [&](Group<CFG>& G, int k) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
#pragma unroll
      for (int i = 0; i < NA; ++i) G.a[s][i].u = *(const uint4*)(ap[i] + k + 16 * s);
#pragma unroll
      for (int j = 0; j < 2; ++j) G.b[s][j].u = *(const uint4*)(bp[j] + k + 16 * s);
    }
  };
  auto compute_group = [&](const Group<CFG>& G) {
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(G.a[s][i].v, G.b[s][j].v, acc[i][j], 0, 0, 0);
  };

  Group<CFG> g0, g1;
  if (n_groups > 0) load_group(g0, k_of(0));
  for (int gi = 0; gi < n_groups; gi += 2) {   // n_groups is even
    load_group(g1, k_of(gi + 1));
    compute_group(g0);
    if (gi + 2 < n_groups) load_group(g0, k_of(gi + 2));
    compute_group(g1);
  }

  // cross-wave reduction and epilogue
  constexpr int NACC = NA * 2;
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) red[((wave * NACC + i * 2 + j) * 16 + r) * 64 + lane] = acc[i][j][r];
  __syncthreads();
  const int nbk = wave >> 1, nb = wave & 1;
  const float inv_t = 1.f / p.temperature;
  (void)inv_t;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float c = 0.f, u = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      c += red[((w * NACC + nbk * 2 + nb) * 16 + r) * 64 + lane];
      if (CFG) u += red[((w * NACC + (2 + nbk) * 2 + nb) * 16 + r) * 64 + lane];
    }
    const float gmix = CFG ? u + p.cfg_scale * (c - u) : c;
    const int node = node0 + 32 * nbk + 8 * (r >> 2) + 4 * half + (r & 3);
    if (node < p.n_nodes) p.logits[(int64_t)node * p.vocab + v0 + 32 * nb + r32] = gmix / p.temperature;
  }
}

// ------------------------------------------------------------------------- bf16, packed operands
// Operand order: for a block of 32 rows rb and a 16-wide k step ks, 64 x 16 bytes where entry
// l = (r32, half) holds src[32*rb + r32][16*ks + 8*half .. +7]; the ks blocks of one rb follow
// each other.  One wave-wide 16-byte load per MFMA operand, 1 KiB contiguous.
__global__ __launch_bounds__(256) void pack32_kernel(const uint16_t* __restrict__ src0, uint4* __restrict__ dst0,
                                                      const uint16_t* __restrict__ src1, uint4* __restrict__ dst1, int rows, int K) {
  const uint16_t* src = blockIdx.z ? src1 : src0;
  uint4* dst = blockIdx.z ? dst1 : dst0;
  const int lane = threadIdx.x & 63, r32 = lane & 31, half = lane >> 5;
  const int ks = blockIdx.x * 4 + (threadIdx.x >> 6), rb = blockIdx.y;
  if (ks >= K / 16) return;
  const int row = 32 * rb + r32;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (row < rows) v = *(const uint4*)(src + (int64_t)row * K + 16 * ks + 8 * half);
  dst[((int64_t)rb * (K / 16) + ks) * 64 + lane] = v;
}

// The same operand order for the guidance-mixed rows u + s (c - u) (float32, rounded once to bf16): the
// projection is linear, so one product over these rows gives the mixed logits.
__global__ __launch_bounds__(256) void pack32_mix_kernel(const uint16_t* __restrict__ src_c, const uint16_t* __restrict__ src_u,
                                                          uint4* __restrict__ dst, int rows, int K, float s) {
  const int lane = threadIdx.x & 63, r32 = lane & 31, half = lane >> 5;
  const int ks = blockIdx.x * 4 + (threadIdx.x >> 6), rb = blockIdx.y;
  if (ks >= K / 16) return;
  const int row = 32 * rb + r32;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (row < rows) {
    const int64_t o = (int64_t)row * K + 16 * ks + 8 * half;
    const uint4 c = *(const uint4*)(src_c + o), u = *(const uint4*)(src_u + o);
    const uint32_t cw[4] = {c.x, c.y, c.z, c.w}, uw[4] = {u.x, u.y, u.z, u.w};
    uint32_t m[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float c0 = __uint_as_float(cw[i] << 16), c1 = __uint_as_float(cw[i] & 0xffff0000u);
      const float u0 = __uint_as_float(uw[i] << 16), u1 = __uint_as_float(uw[i] & 0xffff0000u);
      typedef __bf16 b2 __attribute__((ext_vector_type(2)));
      typedef float f2 __attribute__((ext_vector_type(2)));
      const b2 r = __builtin_convertvector(f2{u0 + s * (c0 - u0), u1 + s * (c1 - u1)}, b2);   // round to nearest even
      m[i] = *(const uint32_t*)&r;
    }
    v = make_uint4(m[0], m[1], m[2], m[3]);
  }
  dst[((int64_t)rb * (K / 16) + ks) * 64 + lane] = v;
}

// NSTEPS > 0: k16 steps per wave known at compile time (K = 64 * NSTEPS), deep fully unrolled pipeline.
template <bool CFG, int NSTEPS>
__global__ __launch_bounds__(256) void lmhead_bf16_packed_kernel(LmParams p) {
  constexpr bool DEEP = NSTEPS > 0;
  constexpr int NA = CFG ? 4 : 2;
  extern __shared__ float red[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r32 = lane & 31, half = lane >> 5;
  const int K = p.hidden, KS = K / 16;

  int logical = blockIdx.x;
  const int nwg = gridDim.x;
  if ((nwg & 7) == 0) logical = (blockIdx.x & 7) * (nwg >> 3) + (blockIdx.x >> 3);
  const int ntile = logical / p.n_mchunks, mc = logical % p.n_mchunks;
  const int v0 = ntile * 64, node0 = mc * 64;

  const uint4* ap[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const uint4* base = (i < 2) ? p.hp_cond : p.hp_uncond;
    ap[i] = base + ((int64_t)(mc * 2 + (i & 1)) * KS) * 64 + lane;
  }
  const uint4* bp[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) bp[j] = (const uint4*)p.w + ((int64_t)(ntile * 2 + j) * KS) * 64 + lane;

  f32x16 acc[NA][2];
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int n_slices = (K / 128 - wave + 3) / 4;   // 128-wide slices wave, wave+4, ... of the hidden dimension
  if constexpr (DEEP) {
    // Deep software pipeline, one k16 step at a time.
    // W streams from HBM: requested WD = 16 steps ahead (32 KiB in flight per wave).  H comes from
    // L2: requested HD = 8 steps ahead.  Registers: 32 + 32 operand fragments and 8 accumulators.
    // After a step's MFMAs its own ring slots are refilled, H first, so that waiting for the H
    // fragment of a later step never waits for younger W requests.
    constexpr int HD = 8, WD = 16;
    static_assert(!DEEP || (NSTEPS % 8 == 0 && NSTEPS >= WD), "whole 128-wide slices per wave");
    // Workgroups that run side by side start at different slices of the hidden dimension (rot), so
    // that at any moment they read different parts of H (spread over the L2 channels instead of all
    // hitting the same lines) and their W streams differ in the low address bits as well.
    constexpr int NSL = NSTEPS / 8;                               // slices per wave (a power of two is not required)
    const int rot = __builtin_amdgcn_readfirstlane(((blockIdx.x >> 3) + (blockIdx.x & 7)) % NSL);
    auto ks_of_step = [&](int t) { return (wave + 4 * (((t >> 3) + rot) % NSL)) * 8 + (t & 7); };
    Frag8 hr[HD][NA];
    Frag8 wr[WD][2];
    auto load_h = [&](int slot, int t) {
      const int64_t o = (int64_t)ks_of_step(t) * 64;
#pragma unroll
      for (int i = 0; i < NA; ++i) hr[slot][i].u = ap[i][o];
    };
    auto load_w = [&](int slot, int t) {
      const int64_t o = (int64_t)ks_of_step(t) * 64;
#pragma unroll
      for (int j = 0; j < 2; ++j) wr[slot][j].u = bp[j][o];
    };
    // prologue in the same request order as the steady state (..., H(t+8), W(t+16), ...)
#pragma unroll
    for (int t = 0; t < WD - HD; ++t) load_w(t, t);
#pragma unroll
    for (int t = 0; t < HD; ++t) {
      load_h(t, t);
      load_w(WD - HD + t, WD - HD + t);
    }
    // fully unrolled: the whole schedule is straight-line code with exact outstanding-load counts
#pragma unroll
    for (int t = 0; t < NSTEPS; ++t) {
#pragma unroll
      for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
          acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hr[t % HD][i].v, wr[t % WD][jj].v, acc[i][jj], 0, 0, 0);
      if (t + HD < NSTEPS) load_h(t % HD, t + HD);
      if (t + WD < NSTEPS) load_w(t % WD, t + WD);
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
    const int n_groups = 2 * n_slices;
    auto ks_of = [&](int gi) { return (wave + 4 * (gi >> 1)) * 8 + 4 * (gi & 1); };   // first k16 step of the group
    auto load_group = [&](Group<CFG>& G, int ks) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int i = 0; i < NA; ++i) G.a[s][i].u = ap[i][(int64_t)(ks + s) * 64];
#pragma unroll
        for (int j = 0; j < 2; ++j) G.b[s][j].u = bp[j][(int64_t)(ks + s) * 64];
      }
    };
    auto compute_group = [&](const Group<CFG>& G) {
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < NA; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(G.a[s][i].v, G.b[s][j].v, acc[i][j], 0, 0, 0);
    };
    Group<CFG> g0, g1;
    if (n_groups > 0) load_group(g0, ks_of(0));
    for (int gi = 0; gi < n_groups; gi += 2) {
      load_group(g1, ks_of(gi + 1));
      compute_group(g0);
      if (gi + 2 < n_groups) load_group(g0, ks_of(gi + 2));
      compute_group(g1);
    }
  }

  constexpr int NACC = NA * 2;
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) red[((wave * NACC + i * 2 + j) * 16 + r) * 64 + lane] = acc[i][j][r];
  __syncthreads();
  const int nbk = wave >> 1, nb = wave & 1;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float c = 0.f, u = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      c += red[((w * NACC + nbk * 2 + nb) * 16 + r) * 64 + lane];
      if (CFG) u += red[((w * NACC + (2 + nbk) * 2 + nb) * 16 + r) * 64 + lane];
    }
    const float gmix = CFG ? u + p.cfg_scale * (c - u) : c;
    const int node = node0 + 32 * nbk + 8 * (r >> 2) + 4 * half + (r & 3);
    if (node < p.n_nodes) p.logits[(int64_t)node * p.vocab + v0 + 32 * nb + r32] = gmix / p.temperature;
  }
}


// ------------------------------------------------------------------- bf16, packed, many rows
// LDS-tiled projection for steps with several hundred rows (batched prompts), where the kernel is
// bound by the matrix cores instead of by streaming W.  Workgroup tile = 256 rows x 256 vocabulary
// columns: with guidance 128 nodes (4 conditional + 4 unconditional 32-row blocks), without 256
// nodes.  The eight waves form a 2 x 4 grid; a wave owns 4 row blocks (two node blocks, conditional
// and unconditional, so the mix stays in registers) x 2 column blocks = 8 accumulators, two waves
// share a SIMD and one wave's waits are covered by the other's MFMAs (four waves with 16
// accumulators each were 10 % slower).
//
// Both operands are packed in MFMA operand order and never pass through registers on their way in:
// gfx950's 16-byte LDS-direct loads write each wave-wide 1 KiB block straight into a ring of four
// half-stages (2 k16 steps = 32 KiB each), so there are no staging registers, no LDS store
// instructions and no register pressure in the loop (a register-staged version of this kernel ran
// at the 256-register limit; a single spilled address in its loop was reloaded behind a wait for
// all outstanding loads and cost 8 %).  Per half-stage h:
//   - step 0 is multiplied; between the multiplications (each occupies the matrix core for 32
//     cycles, so the other instructions are free) step 1's fragments are read and the loads of
//     half-stage h + 3 are issued into the buffer that h - 1 was read from;
//   - the wave waits for its own loads of h + 1 and for its LDS reads, then the workgroup barrier
//     (bare: a fenced barrier would wait for every outstanding load);
//   - step 1 is multiplied while the first fragments of h + 1 are read.
// The barrier sits before the last step's multiplications, which cover it.
// HALF (no guidance only): 128-row tiles for steps whose 256-row tiles would leave compute units idle - a wave owns
// 2 x 2 accumulators; the tile has four H blocks per k16 step, eight per half-stage: wave w requests block w % 4 of
// step w / 4, so every wave issues three loads per half-stage (one H, two W) and the wait counts stay uniform.
template <bool CFG, bool HALF>
__global__ __launch_bounds__(512) void lmhead_bf16_tiled_kernel(LmParams p, int n_mtiles) {
  static_assert(!(CFG && HALF), "half tiles exist for the plain projection only");
  constexpr int NI = HALF ? 2 : 4;   // row blocks per wave
  extern __shared__ u32x4 lds[];     // [4 half-stages][2 k16 steps][16 blocks: 8 H then 8 W][64 lanes]
  constexpr int NBUF = 4, HS = 2, HBYTES = HS * 16 * 1024;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: everything derived from it stays scalar
  const int r32 = lane & 31, half = lane >> 5;
  const int KS = p.hidden / 16, n_half = KS / HS;
  const unsigned lane_off = 16u * lane;                        // byte offset of this lane's 16-byte piece in a block

  int logical = blockIdx.x;
  const int nwg = gridDim.x;
  if ((nwg & 7) == 0) logical = (blockIdx.x & 7) * (nwg >> 3) + (blockIdx.x >> 3);
  const int nt = logical / n_mtiles, mt = logical % n_mtiles;

  // loader: per k16 step a wave copies block wave (H) and block wave + 8 (W); both base pointers are scalars
  const char* src[2];
#pragma unroll
  for (int b4 = 0; b4 < 2; ++b4) {
    const char* base;
    int64_t rb;   // 32-row block index in the source matrix
    if (b4 == 0) {
      if (CFG) { base = (const char*)(wave < 4 ? p.hp_cond : p.hp_uncond); rb = (int64_t)mt * 4 + (wave & 3); }
      else if (HALF) { base = (const char*)p.hp_cond; rb = (int64_t)mt * 4 + (wave & 3); }
      else { base = (const char*)p.hp_cond; rb = (int64_t)mt * 8 + wave; }
    } else {
      base = (const char*)p.w;
      rb = (int64_t)nt * 8 + wave;
    }
    src[b4] = base + rb * KS * 1024;
  }
  const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(size_t)lds);
  const int last = n_half - 1;
  // request i of a half-stage: k16 step i / 2, H (i even) or W (i odd).  h may run past the end:
  // clamped, that data is never multiplied.  M0 carries the LDS address of the wave's 1 KiB block;
  // each lane's 16 bytes land at 16 * lane behind it.
  auto request = [&](int h, int buf, int i) {
    if (HALF && i == 2) return;                                   // (i is a constant after unrolling)
    const int ks = (HALF && i == 0) ? (wave >> 2) : (i >> 1);     // half tiles: the wave's one H block belongs to step wave / 4
    const char* g = src[i & 1] + ((int64_t)min(h, last) * HS + ks) * 1024;
    const int slot = (i & 1) ? 8 + wave : (HALF ? (wave & 3) : wave);
    const unsigned l = lds0 + buf * HBYTES + (ks * 16 + slot) * 1024;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(l), "v"(lane_off), "s"(g) : "memory");
  };
  // A wave's own loads of the next half-stage have landed when at most the 2 x 4 later ones are
  // outstanding; its LDS reads are complete at lgkmcnt(0).
  auto land_and_sync = [&]() {
    if (HALF) asm volatile("s_waitcnt vmcnt(6) lgkmcnt(0)\n\ts_barrier" ::: "memory");   // 2 x 3 later loads
    else asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  };

  // LDS read addresses: one base register per 64 KiB and role, the rest is an immediate.  The bases
  // are made opaque so that the compiler neither re-derives them nor keeps further sums alive.
  char* const lds_b = (char*)lds;
  auto opaque = [](unsigned x) { asm volatile("" : "+v"(x)); return x; };
  const int wm = wave >> 2, wn = wave & 3;
  // row blocks of wave row wm: with guidance 2 wm, 2 wm + 1 (conditional) and the same two of the
  // unconditional half (+4); without, 4 wm .. 4 wm + 3
  const unsigned a_base = 1024u * ((CFG || HALF) ? 2 * wm : 4 * wm) + lane_off, b_base = 1024u * (8 + 2 * wn) + lane_off;
  const unsigned a_off[2] = {opaque(a_base), opaque(a_base + 65536u)};
  const unsigned b_off[2] = {opaque(b_base), opaque(b_base + 65536u)};

  f32x16 acc[NI][2];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  Frag8 fa[2][NI], fb[2][2];   // operand fragments, double-buffered by k16 step
  auto read_one = [&](int slot, int buf, int ks, int idx) {   // idx 0 .. NI-1: H fragment, NI, NI+1: W fragment
    const int byte0 = buf * HBYTES + ks * 16 * 1024;          // compile-time after unrolling
    if (idx < NI) {
      const int rel = CFG ? (idx & 1) + 4 * (idx >> 1) : idx;
      fa[slot][idx].n = *(const u32x4*)(lds_b + a_off[byte0 >> 16] + ((byte0 & 65535) + rel * 1024));
    } else {
      fb[slot][idx - NI].n = *(const u32x4*)(lds_b + b_off[byte0 >> 16] + ((byte0 & 65535) + (idx - NI) * 1024));
    }
  };
  // 2 NI multiplications; after the k-th one, side(k) issues its piece of the other work
  auto multiply_with = [&](int slot, auto&& side) {
#pragma unroll
    for (int k = 0; k < 2 * NI; ++k) {
      __builtin_amdgcn_sched_barrier(0);
      acc[k >> 1][k & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][k >> 1].v, fb[slot][k & 1].v, acc[k >> 1][k & 1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      side(k);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  constexpr int NFR = NI + 2;                          // fragments per k16 step
  constexpr int FRAG_ORDER[6] = {0, NI, NI + 1, 1, 2, 3};   // the order in which the multiplications first need them

#pragma unroll
  for (int h = 0; h < NBUF - 1; ++h)
#pragma unroll
    for (int i = 0; i < 4; ++i) request(h, h, i);
  land_and_sync();
#pragma unroll
  for (int k = 0; k < NFR; ++k) read_one(0, 0, 0, FRAG_ORDER[k]);
  for (int h0 = 0; h0 < n_half; h0 += NBUF) {   // hidden is a multiple of 128: four half-stages always divide it
#pragma unroll
    for (int b = 0; b < NBUF; ++b) {
      const int hn = h0 + b + NBUF - 1, bn = (b + NBUF - 1) % NBUF;
      multiply_with(0, [&](int k) {
        if (HALF) { read_one(1, b, 1, FRAG_ORDER[k]); request(hn, bn, k); }   // four multiplications: a read and a request behind each
        else if (k < 6) read_one(1, b, 1, FRAG_ORDER[k]);
        else { request(hn, bn, 2 * (k - 6)); request(hn, bn, 2 * (k - 6) + 1); }
      });
      land_and_sync();
      multiply_with(1, [&](int k) { if (k < NFR) read_one(0, (b + 1) % NBUF, 0, FRAG_ORDER[k]); });
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the clamped extra requests must not outlive the workgroup's LDS

  // epilogue: accumulator (i, j), register r of lane (r32, half) is row 8 (r / 4) + 4 half + r % 4, column r32
  const int v0 = nt * 256 + 64 * wn;
#pragma unroll
  for (int i = 0; i < (CFG ? 2 : NI); ++i) {
    const int node0 = (CFG || HALF) ? mt * 128 + 32 * (2 * wm + i) : mt * 256 + 32 * (4 * wm + i);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float c = acc[i][j][r];
        const float gmix = CFG ? acc[i + 2][j][r] + p.cfg_scale * (c - acc[i + 2][j][r]) : c;
        const int node = node0 + 8 * (r >> 2) + 4 * half + (r & 3);
        if (node < p.n_nodes) p.logits[(int64_t)node * p.vocab + v0 + 32 * j + r32] = gmix / p.temperature;
        if (r == 15) __builtin_amdgcn_sched_barrier(0);
      }
  }
}

// ------------------------------------------------------------------------------------ row stats
// One workgroup of 1024 threads per row; the row lives in registers (VPT values per thread).
// row_max, exact k-th largest (radix select on order-preserving integer keys), and log-sum-exp
// over the kept entries.
__device__ __forceinline__ uint32_t f32_key(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_f32(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Exact k-th largest by three rounds of radix selection over the order-preserving keys held in
// registers: a 4096-bin LDS histogram (integer atomics) of key bits 31..20, then 1024 bins of bits
// 19..10 among the keys of the chosen bin, then 1024 bins of bits 9..0.  After each round a scan
// from the top bin finds the bin that holds the k-th largest and how many keys lie above it.
// (A row whose entries all share one bin, e.g. all equal, serialises on one LDS address: slow, exact.)
template <int BPT>   // bins per thread; the workgroup's 1024 threads cover 1024 * BPT bins, highest first
__device__ __forceinline__ void find_bin_from_top(const int* hist, int k, int tid, int lane, int wave, int* s_wsum, int* s_bin,
                                                  int* s_above, int pad_bin, int pad) {   // pad entries of bin pad_bin are not part of the row
  constexpr int NB = 1024 * BPT;
  int hb[BPT], loc = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) {
    const int b = NB - 1 - (BPT * tid + i);
    hb[i] = hist[b] - (b == pad_bin ? pad : 0);
    loc += hb[i];
  }
  const int incl = wave_scan_incl_i(loc);
  if (lane == 63) s_wsum[wave] = incl;
  __syncthreads();
  int before = incl - loc;
  for (int w = 0; w < wave; ++w) before += s_wsum[w];
#pragma unroll
  for (int i = 0; i < BPT; ++i) {
    if (before < k && before + hb[i] >= k) { *s_bin = NB - 1 - (BPT * tid + i); *s_above = before; }
    before += hb[i];
  }
  __syncthreads();
}

// Row statistics.  One workgroup of 1024 threads per row; the row lives in registers (VPT values per thread,
// loaded 16 bytes at a time when the row allows it).
//
// Fast path (top-k active): the order-preserving radix rounds above put sign, exponent and three mantissa bits
// into the first digit, so a row of logits lands in a few dozen of its 4096 bins and the 65536 LDS atomics of
// a long row serialise on them.  Instead the first round bins LINEARLY, bin(x) = clamp(int(x s + c), 0, 4095),
// over the range of a 4096-entry sample of the row (each thread's first load), while the rest of the row is
// still arriving.  Any non-decreasing bin function keeps the selection exact: with `above` entries in the bins
// over bin B and above < k <= above + hist[B], the k-th largest is the (k - above)-th largest of bin B.  A
// second sweep over the registers re-evaluates the same fused multiply-add and files every entry of bin B or
// higher (some k + a few dozen of them) into a small per-thread list in LDS; the candidates of bin B are then
// ranked exactly by their integer keys, and only the listed entries see an exponential.
// Rows the fast path does not fit (degenerate or non-finite sample range, k-th largest in the lowest bin, more
// than RS_CAND candidates, a thread with more than RS_CAP listed entries) take the radix rounds: slow, exact.
constexpr int RS_CAP = 12;      // listed entries per thread
constexpr int RS_CAND = 1024;   // candidates ranked by counting
constexpr int RS_PRE_OFFSET = 80 * 1024;   // 80 KiB prefetch buffer behind the structure below (1 KiB aligned)
struct RowStatsSmem {
  int hist1[4096], hist2[1024], hist3[1024];
  float priv[RS_CAP * 1024];    // entry j of thread t at [j * 1024 + t]
  float cand[RS_CAND];
  float f_rng[32], f_max[16], f_sum[16];
  int s_wsum[16];
  int s_bin, s_above, n_cand, flag;
  float s_thr;
};

// Workgroups are persistent: workgroup b takes rows b, b + gridDim.x, ...; the loads of its next row are issued
// as soon as the registers of the current one are no longer needed, so that they overlap the row's tail (list
// processing, candidate ranking, reductions).
template <int VPT, bool VEC>   // VEC: rows start on 16-byte boundaries and V is a multiple of 4
__global__ __launch_bounds__(1024) void row_stats_kernel(LmParams p) {
  extern __shared__ __align__(1024) char rs_smem_raw[];
  RowStatsSmem& sm = *(RowStatsSmem*)rs_smem_raw;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int V = p.vocab;
  const bool topk = p.top_k > 0 && p.top_k < V;
  constexpr int NCH = VPT / 4;
  // Long rows: the last NPRE 16 KiB chunks of the NEXT row are fetched into LDS (LDS-direct loads, no registers
  // needed) while the current row's registers are still in use - HBM would otherwise idle between the end of a
  // row's loads and the moment its registers are free.  A thread reads back exactly the 16 bytes its own lane
  // fetched, so no barrier is involved.
  constexpr int NPRE = (VEC && VPT == 64) ? 5 : 0;
  constexpr int NREG = NCH - NPRE;   // chunks loaded into registers
  float* const pre = (float*)(rs_smem_raw + RS_PRE_OFFSET);
  const unsigned pre_lds = __builtin_amdgcn_readfirstlane((unsigned)(size_t)pre) + 1024u * (unsigned)__builtin_amdgcn_readfirstlane(wave);
  // Chunk jj of this thread, element c, is vocabulary entry 4 (tid + 1024 jj) + c: chunks 0 .. NREG-1 are loaded
  // into registers (and swept in the order they arrive; chunk 0, always inside the row, is the sample), chunks
  // NREG .. NCH-1 come from LDS and are swept last.  Entries past V are masked to -inf before use.  Every load
  // is unconditional (addresses clamped into the row): all of them are in flight at once.
  auto mch = [](int jj) { return jj; };
  float x[VPT];
  // (The thread index is passed through an empty asm so that the per-chunk offsets and masks below are recomputed
  // where they are used instead of being kept in registers across the whole row loop.)
  auto load_row = [&](int row) {
    const char* g = (const char*)(p.logits + (int64_t)row * V);   // uniform base + 32-bit byte offsets
    int t = tid;
    asm volatile("" : "+v"(t));
    if (VEC) {
#pragma unroll
      for (int jj = 0; jj < NREG; ++jj) {
        const float4 q = *(const float4*)(g + 4u * (unsigned)min(4 * (t + 1024 * mch(jj)), V - 4));
        x[4 * jj] = q.x; x[4 * jj + 1] = q.y; x[4 * jj + 2] = q.z; x[4 * jj + 3] = q.w;
      }
    } else {
#pragma unroll
      for (int i = 0; i < VPT; ++i) x[i] = *(const float*)(g + 4u * (unsigned)min(4 * (t + 1024 * (i >> 2)) + (i & 3), V - 1));
    }
  };
  auto prefetch_row = [&](int row) {   // chunks NREG .. NCH-1 -> LDS, lane l's 16 bytes at 16 l behind M0
    const char* g = (const char*)(p.logits + (int64_t)row * V);
    int t = tid;
    asm volatile("" : "+v"(t));
#pragma unroll
    for (int m = 0; m < NPRE; ++m) {
      const unsigned voff = 4u * (unsigned)min(4 * (t + 1024 * (NREG + m)), V - 4);
      const unsigned l = pre_lds + 16384u * m;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(l), "v"(voff), "s"(g) : "memory");
    }
  };
  auto mask_chunks = [&](int jj0, int jj1) {
    if (V != VPT * 1024) {   // workgroup-uniform: a full row needs no masking
      int t = tid;
      asm volatile("" : "+v"(t));
#pragma unroll
      for (int jj = jj0; jj < jj1; ++jj)
#pragma unroll
        for (int c = 0; c < 4; ++c) x[4 * jj + c] = 4 * (t + 1024 * mch(jj)) + c < V ? x[4 * jj + c] : -INFINITY;
    }
  };
  int row = blockIdx.x;
  if (row < p.n_nodes) {
    prefetch_row(row);   // (the first row has nothing to hide behind: same loads, issued first)
    load_row(row);
  }
  for (; row < p.n_nodes; row += gridDim.x) {
    const int next = row + gridDim.x;
    mask_chunks(0, NREG);
#pragma unroll
    for (int i = 0; i < 4; ++i) sm.hist1[tid + 1024 * i] = 0;
    if (tid == 0) { sm.n_cand = 0; sm.flag = 0; }

    // ---- range of the sample (first chunk of every thread)
    float smax = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
    float smin = INFINITY;
#pragma unroll
    for (int c = 0; c < 4; ++c) smin = fminf(smin, x[c] == -INFINITY ? INFINITY : x[c]);   // padding (and -inf logits) aside
    smax = wave_max(smax);
    smin = -wave_max(-smin);
    if (lane == 0) { sm.f_rng[wave] = smax; sm.f_rng[16 + wave] = smin; }
    __syncthreads();
    smax = sm.f_rng[0]; smin = sm.f_rng[16];
#pragma unroll
    for (int w = 1; w < 16; ++w) { smax = fmaxf(smax, sm.f_rng[w]); smin = fminf(smin, sm.f_rng[16 + w]); }
    const float bs = 4096.f / (smax - smin), bc = -smin * bs;
    // usable: finite positive scale and offset (rules out equal, infinite or NaN sample bounds)
    const bool fast = topk && bs > 0.f && bs < INFINITY && fabsf(bc) < INFINITY;

    float mx = -INFINITY;
    auto sweep = [&](int jj0, int jj1) {   // row maximum and first-round histogram of x-chunks jj0 .. jj1-1
      if (fast) {
#pragma unroll
        for (int i = 4 * jj0; i < 4 * jj1; ++i) {
          mx = fmaxf(mx, x[i]);
          const float t = __builtin_amdgcn_fmed3f(fmaf(x[i], bs, bc), 0.f, 4095.f);
          atomicAdd(&sm.hist1[(int)t], 1);
          if ((i & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // keep the unrolled sweep from piling up temporaries
        }
      } else {
#pragma unroll
        for (int i = 4 * jj0; i < 4 * jj1; ++i) mx = fmaxf(mx, x[i]);
      }
    };
    sweep(0, NREG);
    if (NPRE > 0) {
      // every load of this row that went to registers has been waited for; the LDS-direct ones were issued before
      // them and complete in order - waited for explicitly all the same
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      int t = tid;
      asm volatile("" : "+v"(t));
#pragma unroll
      for (int m = 0; m < NPRE; ++m) {
        const float4 q = *(const float4*)(pre + 4096 * m + 4 * t);
        x[4 * (NREG + m)] = q.x; x[4 * (NREG + m) + 1] = q.y; x[4 * (NREG + m) + 2] = q.z; x[4 * (NREG + m) + 3] = q.w;
      }
      mask_chunks(NREG, NCH);
      sweep(NREG, NCH);
      // the values are in registers (the sweep consumed them): the buffer can take the next row's chunks
      if (next < p.n_nodes) prefetch_row(next);
    }
    mx = wave_max(mx);
    if (lane == 0) sm.f_max[wave] = mx;
    __syncthreads();                       // maxima and every atomic of the sweep
    mx = sm.f_max[0];
#pragma unroll
    for (int w = 1; w < 16; ++w) mx = fmaxf(mx, sm.f_max[w]);

    float thr = -INFINITY, se = 0.f;
    bool done = false;
    int cnt = 0, B = 0, n_c = 0, k = p.top_k;
    if (fast) {
      // the -inf padding past V went to bin 0 with everything else at or below the sample's minimum
      find_bin_from_top<4>(sm.hist1, k, tid, lane, wave, sm.s_wsum, &sm.s_bin, &sm.s_above, 0, VPT * 1024 - V);
      B = sm.s_bin;
      n_c = sm.hist1[B];
      k -= sm.s_above;                     // rank of the k-th largest inside bin B, 1 = largest
      if (B > 0 && n_c <= RS_CAND) {       // workgroup-uniform
        const float Bf = (float)B;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
          if (fmaf(x[i], bs, bc) >= Bf) {  // bin(x) >= B (B >= 1: the clamp at 0 plays no part; the one at 4095 cannot matter)
            if (cnt < RS_CAP) sm.priv[cnt * 1024 + tid] = x[i];
            ++cnt;
          }
          if ((i & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
        if (cnt > RS_CAP) sm.flag = 1;
        __syncthreads();
        done = sm.flag == 0;
      }
    }
    // The registers are free (the rounds below re-read the row): the next row arrives during this row's tail.
    if (next < p.n_nodes) load_row(next);
    if (done) {
      // listed entries: above bin B -> kept; in bin B -> candidate
      const float B1f = (float)(B + 1);
      for (int j = 0; j < cnt; ++j) {
        const float xv = sm.priv[j * 1024 + tid];
        if (B < 4095 && fmaf(xv, bs, bc) >= B1f) se += __expf(xv - mx);
        else sm.cand[atomicAdd(&sm.n_cand, 1)] = xv;
      }
      __syncthreads();
      // exact k-th largest of the n_c candidates by counting (ties: lower list index first); wave w ranks
      // candidates w, w + 16, ..., its lanes share the comparisons
      for (int i = wave; i < n_c; i += 16) {
        const uint32_t ki = f32_key(sm.cand[i]);
        int rank = 0;
        for (int j = lane; j < n_c; j += 64) {
          const uint32_t kj = f32_key(sm.cand[j]);
          rank += (kj > ki || (kj == ki && j < i)) ? 1 : 0;
        }
        rank = wave_sum_i(rank);
        if (lane == 0 && rank == k - 1) sm.s_thr = key_f32(ki);
      }
      __syncthreads();
      thr = sm.s_thr;
      const uint32_t tk = f32_key(thr);
      for (int i = tid; i < n_c; i += 1024) {
        const float xi = sm.cand[i];
        if (f32_key(xi) >= tk) se += __expf(xi - mx);
      }
    } else {
      // Radix rounds on the order-preserving keys (also: no top-k -> every entry kept).  Slow and exact: the row
      // is read again from memory (mostly the caches) in every round, a few registers at a time.
      const float* g = p.logits + (int64_t)row * V;
      uint32_t thr_key = 0;
      se = 0.f;
      if (topk) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) sm.hist1[tid + 1024 * i] = 0;
        sm.hist2[tid] = 0;
        sm.hist3[tid] = 0;
        __syncthreads();
        k = p.top_k;
        for (int v = tid; v < V; v += 1024) atomicAdd(&sm.hist1[f32_key(g[v]) >> 20], 1);
        __syncthreads();
        find_bin_from_top<4>(sm.hist1, k, tid, lane, wave, sm.s_wsum, &sm.s_bin, &sm.s_above, 0, 0);
        const uint32_t b1 = (uint32_t)sm.s_bin;
        k -= sm.s_above;
        __syncthreads();   // s_bin / s_above are rewritten by the next round
        for (int v = tid; v < V; v += 1024) {
          const uint32_t key = f32_key(g[v]);
          if ((key >> 20) == b1) atomicAdd(&sm.hist2[(key >> 10) & 1023u], 1);
        }
        __syncthreads();
        find_bin_from_top<1>(sm.hist2, k, tid, lane, wave, sm.s_wsum, &sm.s_bin, &sm.s_above, 0, 0);
        const uint32_t b12 = (b1 << 10) | (uint32_t)sm.s_bin;
        k -= sm.s_above;
        __syncthreads();
        for (int v = tid; v < V; v += 1024) {
          const uint32_t key = f32_key(g[v]);
          if ((key >> 10) == b12) atomicAdd(&sm.hist3[key & 1023u], 1);
        }
        __syncthreads();
        find_bin_from_top<1>(sm.hist3, k, tid, lane, wave, sm.s_wsum, &sm.s_bin, &sm.s_above, 0, 0);
        thr_key = (b12 << 10) | (uint32_t)sm.s_bin;
        thr = key_f32(thr_key);
      }
      for (int v = tid; v < V; v += 1024) {
        const float xv = g[v];
        se += f32_key(xv) >= thr_key ? __expf(xv - mx) : 0.f;
      }
    }
    se = wave_sum(se);
    if (lane == 0) sm.f_sum[wave] = se;
    __syncthreads();
    if (tid == 0) {
      float tot = 0.f;
      for (int w = 0; w < 16; ++w) tot += sm.f_sum[w];
      p.row_max[row] = mx;
      p.row_thr[row] = thr;
      p.row_lse[row] = mx + logf(tot);
    }
  }
}

LmParams make_params(const lmhead_args* a) {
  LmParams p;
  p.h_cond = a->h_cond;
  p.h_uncond = a->h_uncond;
  p.w = a->w;
  p.logits = a->logits;
  p.row_max = a->row_max;
  p.row_thr = a->row_thr;
  p.row_lse = a->row_lse;
  p.hp_cond = nullptr;
  p.hp_uncond = nullptr;
  p.n_nodes = a->n_nodes;
  p.hidden = a->hidden;
  p.vocab = a->vocab;
  p.n_mchunks = (a->n_nodes + 63) / 64;
  p.cfg_scale = a->cfg_scale;
  p.temperature = a->temperature;
  p.top_k = a->top_k;
  return p;
}

}  // namespace

hipError_t launch_lmhead_f32(cascade_ctx* ctx, const lmhead_args* a) {
  hipStream_t stream = ctx->stream;
  KernelTimer t(ctx, CASCADE_K_LMHEAD);
  LmParams p = make_params(a);
  dim3 grid((a->vocab + 255) / 256, a->n_nodes);
  const size_t smem = (size_t)a->hidden * sizeof(float) * (a->h_uncond ? 2 : 1);
  CASCADE_TIMED_LAUNCH(t, lmhead_f32_kernel, grid, dim3(256), smem, stream, p);
  return hipGetLastError();
}

template <bool CFG, int KIND>   // KIND 0: row-major W, 1: packed, 2: packed + deep pipeline
hipError_t launch_bf16_gemm(cascade_ctx* ctx, const LmParams& p, int grid) {
  const size_t smem = (size_t)4 * (CFG ? 8 : 4) * 16 * 64 * sizeof(float);
  auto kern = KIND == 2 ? lmhead_bf16_packed_kernel<CFG, 64> : (KIND == 1 ? lmhead_bf16_packed_kernel<CFG, 0> : lmhead_bf16_kernel<CFG>);
  static bool attr_done = false;   // one flag per template instance
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  KernelTimer t(ctx, CASCADE_K_LMHEAD);
  CASCADE_TIMED_LAUNCH(t, kern, dim3(grid), dim3(256), smem, ctx->stream, p);
  return hipGetLastError();
}

hipError_t launch_lmhead_bf16(cascade_ctx* ctx, const lmhead_args* a) {
  LmParams p = make_params(a);
  const int grid = (a->vocab / 64) * p.n_mchunks;
  // guidance mixed into the hidden rows while they are packed: from here on a plain projection of n_nodes rows
  const bool premix = a->h_uncond != nullptr && a->cfg_mix == CASCADE_CFG_MIX_HIDDEN && a->w_layout == CASCADE_W_PACKED32;
  const bool cfg = a->h_uncond != nullptr && !premix;
  if (a->w_layout == CASCADE_W_PACKED32) {
    // many rows and a vocabulary made of whole 256-column tiles: LDS-tiled kernel, 256-row tiles
    const int rows = a->n_nodes * (cfg ? 2 : 1);
    const bool tiled = rows >= (cfg ? 512 : 257) && (a->vocab % 256) == 0;
    // plain projection: 128-row tiles when the 256-row tiling would leave compute units without a workgroup
    const bool half = !cfg && (long)((a->n_nodes + 255) / 256) * (a->vocab / 256) < ctx->n_cu;
    const int nodes_per_tile = (cfg || half) ? 128 : 256;
    const int n_mtiles = (a->n_nodes + nodes_per_tile - 1) / nodes_per_tile;
    // repack this step's hidden states into operand order (zero rows up to a whole tile / chunk)
    const int rblocks = tiled ? n_mtiles * (nodes_per_tile / 32) : p.n_mchunks * 2;
    const size_t per = (size_t)rblocks * 32 * a->hidden * 2;
    if (per * 2 > ctx->hpack_ws_bytes) return hipErrorInvalidValue;
    uint4* hc = (uint4*)ctx->hpack_ws;
    uint4* hu = (uint4*)(ctx->hpack_ws + per);
    dim3 pgrid((a->hidden / 16 + 3) / 4, rblocks, cfg ? 2 : 1);
    {
      KernelTimer t(ctx, CASCADE_K_PACK);
      if (premix) {
        CASCADE_TIMED_LAUNCH(t, pack32_mix_kernel, pgrid, dim3(256), 0, ctx->stream, (const uint16_t*)a->h_cond,
                             (const uint16_t*)a->h_uncond, hc, a->n_nodes, a->hidden, a->cfg_scale);
      } else {
        CASCADE_TIMED_LAUNCH(t, pack32_kernel, pgrid, dim3(256), 0, ctx->stream, (const uint16_t*)a->h_cond, hc,
                             (const uint16_t*)a->h_uncond, hu, a->n_nodes, a->hidden);
      }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    p.hp_cond = hc;
    p.hp_uncond = hu;
    if (tiled) {
      const size_t smem = (size_t)4 * 32 * 1024;   // ring of four 32 KiB half-stages
      static bool attr_done[3] = {false, false, false};
      auto kern = cfg ? lmhead_bf16_tiled_kernel<true, false> : (half ? lmhead_bf16_tiled_kernel<false, true> : lmhead_bf16_tiled_kernel<false, false>);
      const int which = cfg ? 0 : (half ? 1 : 2);
      if (!attr_done[which]) {
        e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_done[which] = true;
      }
      KernelTimer t(ctx, CASCADE_K_LMHEAD);
      CASCADE_TIMED_LAUNCH(t, kern, dim3((a->vocab / 256) * n_mtiles), dim3(512), smem, ctx->stream, p, n_mtiles);
      return hipGetLastError();
    }
    if (a->hidden == 4096) return cfg ? launch_bf16_gemm<true, 2>(ctx, p, grid) : launch_bf16_gemm<false, 2>(ctx, p, grid);
    return cfg ? launch_bf16_gemm<true, 1>(ctx, p, grid) : launch_bf16_gemm<false, 1>(ctx, p, grid);
  }
  return cfg ? launch_bf16_gemm<true, 0>(ctx, p, grid) : launch_bf16_gemm<false, 0>(ctx, p, grid);
}

hipError_t launch_pack_w(cascade_ctx* ctx, const void* w, int vocab, int hidden, void* w_packed) {
  dim3 grid((hidden / 16 + 3) / 4, vocab / 32);
  hipLaunchKernelGGL(pack32_kernel, grid, dim3(256), 0, ctx->stream, (const uint16_t*)w, (uint4*)w_packed,
                     (const uint16_t*)nullptr, (uint4*)nullptr, vocab, hidden);
  return hipGetLastError();
}

template <int VPT, bool VEC>
hipError_t launch_row_stats_t(cascade_ctx* ctx, const LmParams& p) {
  static_assert(sizeof(RowStatsSmem) <= RS_PRE_OFFSET, "the prefetch buffer starts behind the structure");
  const size_t smem = (VEC && VPT == 64) ? RS_PRE_OFFSET + 80 * 1024 : sizeof(RowStatsSmem);
  static bool attr_done = false;   // one flag per template instance
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)row_stats_kernel<VPT, VEC>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  KernelTimer t(ctx, CASCADE_K_ROW_STATS);
  // one workgroup per compute unit at most (its 1024 threads hold a row in registers), each walking its share of the rows
  const int grid = p.n_nodes < ctx->n_cu ? p.n_nodes : ctx->n_cu;
  CASCADE_TIMED_LAUNCH(t, (row_stats_kernel<VPT, VEC>), dim3(grid), dim3(1024), smem, ctx->stream, p);
  return hipGetLastError();
}

hipError_t launch_row_stats(cascade_ctx* ctx, const lmhead_args* a) {
  LmParams p = make_params(a);
  const int V = a->vocab;
  // 16-byte loads need every row to start on a 16-byte boundary
  const bool vec = V % 4 == 0 && ((uintptr_t)a->logits & 15u) == 0;
  if (V <= 4096) return vec ? launch_row_stats_t<4, true>(ctx, p) : launch_row_stats_t<4, false>(ctx, p);
  if (V <= 16384) return vec ? launch_row_stats_t<16, true>(ctx, p) : launch_row_stats_t<16, false>(ctx, p);
  return vec ? launch_row_stats_t<64, true>(ctx, p) : launch_row_stats_t<64, false>(ctx, p);
}
