// convergence_weights: the Eq. 4 weight mask of the drafter-training loss.  For every pair of
// consecutive positions (k, k+1) of a target-generated sequence: cos(F_k, F_{k+1}) >= tau_seq (the
// convergence set of Eq. 2 between neighbours) gives weight c, otherwise 1.
//
// Bandwidth-bound: every feature row should cross HBM once.  One wavefront walks a run of
// consecutive pairs with the previous row held in registers (16-byte vectors, lane-interleaved so
// that every load instruction covers 1 KiB of contiguous memory), the next row already requested
// while the current one is reduced; only the first row of a run is read by two wavefronts.
#include "common.h"

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

template <typename T> struct Acc;
template <> struct Acc<float> {
  static __device__ __forceinline__ void dot(const u32x4& a, const u32x4& b, float& ab, float& bb) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float x = __uint_as_float(a[i]), y = __uint_as_float(b[i]);
      ab = fmaf(x, y, ab);
      bb = fmaf(y, y, bb);
    }
  }
};
template <> struct Acc<uint16_t> {   // bf16 pairs packed in 32-bit words
  static __device__ __forceinline__ void dot(const u32x4& a, const u32x4& b, float& ab, float& bb) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float x0 = __uint_as_float(a[i] << 16), x1 = __uint_as_float(a[i] & 0xffff0000u);
      const float y0 = __uint_as_float(b[i] << 16), y1 = __uint_as_float(b[i] & 0xffff0000u);
      ab = fmaf(x0, y0, ab);
      ab = fmaf(x1, y1, ab);
      bb = fmaf(y0, y0, bb);
      bb = fmaf(y1, y1, bb);
    }
  }
};

// NV = 16-byte vectors per lane (row bytes <= NV * 1024)
template <typename T, int NV>
__global__ __launch_bounds__(256) void conv_weight_kernel(conv_weight_args a, int runs_per_seq, int RUN) {
  const int lane = threadIdx.x & 63;
  const long long wave_id = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int seq = (int)(wave_id / runs_per_seq), run = (int)(wave_id % runs_per_seq);
  if (seq >= a.n_seqs) return;
  const int K = a.seq_len;
  const int nvec = a.hidden * (int)sizeof(T) / 16;   // 16-byte vectors per row
  const u32x4* base = (const u32x4*)a.features + (long long)seq * K * nvec;
  float* wout = a.weights + (long long)seq * K;
  float* cout = a.cos_next ? a.cos_next + (long long)seq * K : nullptr;
  const int k0 = run * RUN, k1 = min(k0 + RUN, K - 1);   // pairs (k, k+1) for k in [k0, k1)

  auto load_row = [&](int k, u32x4 (&dst)[NV]) {
    const u32x4* row = base + (long long)k * nvec;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int idx = v * 64 + lane;
      const u32x4 x = row[min(idx, nvec - 1)];   // clamped, zeroed below
      dst[v] = idx < nvec ? x : u32x4{0u, 0u, 0u, 0u};
    }
  };

  if (k0 < k1) {
    u32x4 prev[NV], cur[NV], nxt[NV];
    load_row(k0, prev);
    load_row(k0 + 1, cur);
    float pp = 0.f, dummy = 0.f;
#pragma unroll
    for (int v = 0; v < NV; ++v) Acc<T>::dot(prev[v], prev[v], dummy, pp);
    pp = wave_sum(pp);
    for (int k = k0; k < k1; ++k) {
      const int kn = min(k + 2, k1);   // next row to fetch; at the end of the run the last row again (a cache hit)
      load_row(kn, nxt);
      float ab = 0.f, bb = 0.f;
#pragma unroll
      for (int v = 0; v < NV; ++v) Acc<T>::dot(prev[v], cur[v], ab, bb);
      ab = wave_sum(ab);
      bb = wave_sum(bb);
      const float cs = (pp > 0.f && bb > 0.f) ? ab / (sqrtf(pp) * sqrtf(bb)) : 0.f;
      if (lane == 0) {
        wout[k] = cs >= a.tau_seq ? a.c : 1.f;
        if (cout) cout[k] = cs;
      }
      pp = bb;
#pragma unroll
      for (int v = 0; v < NV; ++v) { prev[v] = cur[v]; cur[v] = nxt[v]; }
    }
  }
  if (run == runs_per_seq - 1 && lane == 0) {   // the last position has no successor
    wout[K - 1] = 1.f;
    if (cout) cout[K - 1] = 0.f;
  }
}

template <typename T>
hipError_t launch_t(cascade_ctx* ctx, const conv_weight_args* a) {
  const int row_bytes = a->hidden * (int)sizeof(T);
  const int nv = (row_bytes + 1023) / 1024;
  // pairs per wavefront: long runs re-read fewer boundary rows, short runs give more wavefronts in
  // flight; aim at eight wavefronts per compute unit, between 8 and 32 pairs each
  const long long pairs = (long long)a->n_seqs * (a->seq_len > 1 ? a->seq_len - 1 : 0);
  int RUN = (int)(pairs / (256 * 8));
  RUN = RUN < 8 ? 8 : (RUN > 32 ? 32 : RUN);
  const int runs_per_seq = a->seq_len > 1 ? (a->seq_len - 1 + RUN - 1) / RUN : 1;
  const long long waves = (long long)a->n_seqs * runs_per_seq;
  dim3 grid((unsigned)((waves + 3) / 4));
  KernelTimer t(ctx, CASCADE_K_WEIGHTS);
#define CASCADE_LAUNCH_CW(NV) CASCADE_TIMED_LAUNCH(t, (conv_weight_kernel<T, NV>), grid, dim3(256), 0, ctx->stream, *a, runs_per_seq, RUN)
  if (nv <= 1) CASCADE_LAUNCH_CW(1);
  else if (nv <= 2) CASCADE_LAUNCH_CW(2);
  else if (nv <= 4) CASCADE_LAUNCH_CW(4);
  else if (nv <= 8) CASCADE_LAUNCH_CW(8);
  else CASCADE_LAUNCH_CW(16);
#undef CASCADE_LAUNCH_CW
  return hipGetLastError();
}

}  // namespace

hipError_t launch_conv_weights(cascade_ctx* ctx, const conv_weight_args* a) {
  return a->dtype == CASCADE_BF16 ? launch_t<uint16_t>(ctx, a) : launch_t<float>(ctx, a);
}
