// Measurement aids: what this device actually sustains for a plain streaming read and for a
// register-only bf16 MFMA loop.  Benchmarks report kernel rooflines against the published peaks
// and, beside them, against these two measured ceilings.
#include "common.h"

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// Every lane reads 16 bytes per trip, consecutive lanes consecutive addresses, grid-stride over the
// buffer.  The xor of everything read is stored only if it equals a value the host picks so that
// the store practically never happens; the loads cannot be removed.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, long long n16, unsigned magic,
                                                          unsigned* __restrict__ sink) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long stride = (long long)gridDim.x * blockDim.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + 3 * stride < n16; i += 4 * stride) {
    u32x4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    acc ^= a ^ b ^ c ^ d;
  }
  for (; i < n16; i += stride) acc ^= src[i];
  unsigned x = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (x == magic) *sink = x;
}

// Eight independent 32x32x16 bf16 MFMA accumulator chains per wave, operands held in registers.
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, float* __restrict__ sink) {
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(float)((threadIdx.x + i) & 3);
    b[i] = (__bf16)(float)((threadIdx.x * 3 + i) & 1);
  }
  f32x16 acc[8];
  for (int j = 0; j < 8; ++j)
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
  for (int j = 0; j < 8; ++j)
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  if (s == -1.f) *sink = s;   // sums of non-negative products: never true
}

}  // namespace

extern "C" {

int cascade_measure_hbm_read(cascade_ctx* ctx, const void* buf, int64_t bytes, int32_t repeats, double* gb_per_s) {
  if (!ctx || !buf || !gb_per_s || bytes < 16 || repeats < 1 || repeats > 1000) return CASCADE_EINVAL;
  if (((uintptr_t)buf & 15) != 0) return CASCADE_EINVAL;
  const long long n16 = bytes / 16;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return CASCADE_EHIP;
  unsigned* sink = (unsigned*)(ctx->ws + 128);   // inside the 256-byte status block, never read by kernels
  const int grid = 8192;
  stream_read_kernel<<<grid, 256, 0, ctx->stream>>>((const u32x4*)buf, n16, 0x9e3779b9u, sink);   // warm-up
  (void)hipEventRecord(e0, ctx->stream);
  for (int r = 0; r < repeats; ++r) stream_read_kernel<<<grid, 256, 0, ctx->stream>>>((const u32x4*)buf, n16, 0x9e3779b9u, sink);
  (void)hipEventRecord(e1, ctx->stream);
  hipError_t e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess || ms <= 0.f) return CASCADE_EHIP;
  *gb_per_s = (double)n16 * 16.0 * repeats / (ms * 1e-3) / 1e9;
  return CASCADE_OK;
}

int cascade_measure_mfma_bf16(cascade_ctx* ctx, int32_t iters, double* tflop_per_s) {
  if (!ctx || !tflop_per_s || iters < 1 || iters > (1 << 20)) return CASCADE_EINVAL;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, ctx->device) != hipSuccess) return CASCADE_EHIP;
  const int grid = prop.multiProcessorCount * 8;   // 8 workgroups of 4 waves per compute unit
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return CASCADE_EHIP;
  float* sink = (float*)(ctx->ws + 192);
  mfma_loop_kernel<<<grid, 256, 0, ctx->stream>>>(16, sink);   // warm-up
  (void)hipEventRecord(e0, ctx->stream);
  mfma_loop_kernel<<<grid, 256, 0, ctx->stream>>>(iters, sink);
  (void)hipEventRecord(e1, ctx->stream);
  hipError_t e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess || ms <= 0.f) return CASCADE_EHIP;
  const double flops = (double)grid * 4.0 * iters * 8.0 * (2.0 * 32 * 32 * 16);
  *tflop_per_s = flops / (ms * 1e-3) / 1e12;
  return CASCADE_OK;
}

}  // extern "C"
