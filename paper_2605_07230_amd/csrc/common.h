// Shared declarations of the gfx950 tree-verification library (internal; the public ABI is
// include/cascade_verify.h).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/cascade_verify.h"

// ----------------------------------------------------------------------------------------------
// context
struct cascade_ctx {
  hipStream_t stream;
  cascade_limits lim;
  int device;
  int n_cu;               // compute units of the device (persistent kernels size their grids by it)
  char* ws;               // device workspace
  size_t ws_bytes;
  int* dev_status;        // one int at the start of ws: sticky precondition flag
  char* attn_ws;          // split-KV partials
  size_t attn_ws_bytes;
  char* hpack_ws;         // hidden states repacked into MFMA operand order, cond then uncond
  size_t hpack_ws_bytes;
  // optional per-kernel timing with HIP events on the ctx stream (cascade_set_kernel_timing)
  bool timing;
  hipEvent_t* ev;         // [CASCADE_K_COUNT][TIMING_RING][2], created on first enable
  int ev_used[CASCADE_K_COUNT];
};

enum { TIMING_RING = 2048 };

// Per-kernel timing: when it is on, a launch goes through hipExtLaunchKernelGGL with a start and a stop
// event taken from the context's ring, which receive the dispatch's own begin / end timestamps (no
// extra packets on the stream, so the figure is the kernel's duration as a profiler reports it).
struct KernelTimer {
  hipEvent_t e0, e1;
  KernelTimer(cascade_ctx* c, int id) : e0(nullptr), e1(nullptr) {
    if (c && c->timing && c->ev && c->ev_used[id] < TIMING_RING) {
      const int slot = c->ev_used[id]++;
      e0 = c->ev[(id * TIMING_RING + slot) * 2];
      e1 = c->ev[(id * TIMING_RING + slot) * 2 + 1];
    }
  }
  bool active() const { return e0 != nullptr; }
};
#define CASCADE_TIMED_LAUNCH(timer, kernel, grid, block, smem, stream, ...)                                  \
  do {                                                                                                       \
    if ((timer).active()) hipExtLaunchKernelGGL(kernel, grid, block, smem, stream, (timer).e0, (timer).e1, 0, __VA_ARGS__); \
    else hipLaunchKernelGGL(kernel, grid, block, smem, stream, __VA_ARGS__);                                  \
  } while (0)

// flags OR-ed into *dev_status by kernels
enum {
  CASCADE_FLAG_PARENT = 1,   // parent[i] >= i or < -1, or a second root
  CASCADE_FLAG_WIDTH = 2,    // more than CASCADE_MAX_WIDTH children
  CASCADE_FLAG_TOKEN = 4,    // token outside [0, vocab)
  CASCADE_FLAG_DEPTH = 8,    // path longer than max_depth
  CASCADE_FLAG_CAPACITY = 16, // kv_commit: a row's cache has no room for root + accepted path
  CASCADE_FLAG_PATH = 32,    // kv_commit: a path entry outside the row's tree, or a bad row_prompt
  CASCADE_FLAG_TREE_SIZE = 64  // a tree with more nodes than the bound the launch was sized for
};

// launchers (one translation unit each); all return hipError_t of the launch
hipError_t launch_tree_attn_f32(cascade_ctx* ctx, const tree_attn_args* a);
hipError_t launch_tree_attn_bf16(cascade_ctx* ctx, const tree_attn_args* a);
hipError_t launch_lmhead_f32(cascade_ctx* ctx, const lmhead_args* a);
hipError_t launch_lmhead_bf16(cascade_ctx* ctx, const lmhead_args* a);
hipError_t launch_row_stats(cascade_ctx* ctx, const lmhead_args* a);
hipError_t launch_pack_w(cascade_ctx* ctx, const void* w, int vocab, int hidden, void* w_packed);
hipError_t launch_accept(cascade_ctx* ctx, const accept_args* a);
hipError_t launch_select(cascade_ctx* ctx, const select_args* a);
hipError_t launch_select_residual(cascade_ctx* ctx, const select_args* a);
hipError_t launch_kv_commit(cascade_ctx* ctx, const kv_commit_args* a);
hipError_t launch_conv_weights(cascade_ctx* ctx, const conv_weight_args* a);

// ----------------------------------------------------------------------------------------------
// device helpers
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define WAVE 64

// Wave-wide scans and reductions on the DPP cross-lane network (no LDS traffic): a Hillis-Steele
// scan inside each row of 16 lanes (row_shr 1, 2, 4, 8), then the row totals are carried across
// rows with row_bcast:15 (into rows 1 and 3) and row_bcast:31 (into rows 2 and 3).  Lane 63 ends up
// holding the total.  Lanes with no source lane receive the operation's identity.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f32(float identity, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_i32(int identity, int v) {
  return __builtin_amdgcn_update_dpp(identity, v, CTRL, ROW_MASK, 0xf, false);
}
#define CASCADE_DPP_SCAN(v, OP, ID, FN)          \
  v = OP(v, FN<0x111, 0xf>(ID, v));              \
  v = OP(v, FN<0x112, 0xf>(ID, v));              \
  v = OP(v, FN<0x114, 0xf>(ID, v));              \
  v = OP(v, FN<0x118, 0xf>(ID, v));              \
  v = OP(v, FN<0x142, 0xa>(ID, v));              \
  v = OP(v, FN<0x143, 0xc>(ID, v));

__device__ __forceinline__ float op_add_f(float a, float b) { return a + b; }
__device__ __forceinline__ int op_add_i(int a, int b) { return a + b; }
__device__ __forceinline__ int op_min_i(int a, int b) { return min(a, b); }
__device__ __forceinline__ int op_max_i(int a, int b) { return max(a, b); }

__device__ __forceinline__ float wave_scan_incl_f(float v) {
  CASCADE_DPP_SCAN(v, op_add_f, 0.f, dpp_f32)
  return v;
}
__device__ __forceinline__ int wave_scan_incl_i(int v) {
  CASCADE_DPP_SCAN(v, op_add_i, 0, dpp_i32)
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  CASCADE_DPP_SCAN(v, op_add_f, 0.f, dpp_f32)
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  CASCADE_DPP_SCAN(v, fmaxf, -INFINITY, dpp_f32)
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ int wave_sum_i(int v) {
  CASCADE_DPP_SCAN(v, op_add_i, 0, dpp_i32)
  return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ int wave_min_i(int v) {
  CASCADE_DPP_SCAN(v, op_min_i, 0x7fffffff, dpp_i32)
  return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ int wave_max_i(int v) {
  CASCADE_DPP_SCAN(v, op_max_i, (int)0x80000000, dpp_i32)
  return __builtin_amdgcn_readlane(v, 63);
}

// Reductions across the four 16-lane rows of a wave (lanes l, l^16, l^32, l^48) with the gfx950
// row-swap instructions: v_permlane16_swap exchanges odd rows of its first operand with even rows
// of its second, v_permlane32_swap the upper half of the first with the lower half of the second.
// With both operands equal, the two results hold v[l] and v[l ^ 16] (resp. v[l ^ 32]) in every lane.
typedef unsigned cascade_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float rows4_max(float v) {
  cascade_u32x2 a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a.x), __uint_as_float(a.y));
  cascade_u32x2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b.x), __uint_as_float(b.y));
}
__device__ __forceinline__ float rows4_sum(float v) {
  cascade_u32x2 a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a.x) + __uint_as_float(a.y);
  cascade_u32x2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b.x) + __uint_as_float(b.y);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even float -> bf16 bits (NaN kept quiet)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// element loads that widen to float, for kernels templated on the storage type
template <typename T>
__device__ __forceinline__ float load_f32(const T* p);
template <>
__device__ __forceinline__ float load_f32<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_f32<uint16_t>(const uint16_t* p) { return bf16_bits_to_f32(*p); }
