// C ABI of the tree-verification library: context, argument validation, dispatch.
// Validation uses host-visible values only and happens before anything is enqueued.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>

#include "common.h"

namespace {

thread_local char g_hip_msg[256] = "no HIP error recorded";

int hip_fail(hipError_t e) {
  snprintf(g_hip_msg, sizeof(g_hip_msg), "HIP error %d: %s", (int)e, hipGetErrorString(e));
  return CASCADE_EHIP;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool bad_float(float x) { return isnan(x); }

}  // namespace

extern "C" {

const char* cascade_strerror(int status) {
  switch (status) {
    case CASCADE_OK: return "ok";
    case CASCADE_EINVAL: return "invalid argument (null pointer, negative size, NaN, bad enum)";
    case CASCADE_ESHAPE: return "shape exceeds the context limits or breaks a divisibility rule";
    case CASCADE_EDTYPE: return "dtype not supported by this call";
    case CASCADE_ENOMEM: return "workspace allocation failed";
    case CASCADE_EHIP: return g_hip_msg;
    case CASCADE_ETREE: return "a device-side precondition on the tree arrays was violated";
    default: return "unknown status";
  }
}

int cascade_create(cascade_ctx** out, const cascade_limits* lim, void* hip_stream) {
  if (!out) return CASCADE_EINVAL;
  *out = nullptr;
  if (!lim) return CASCADE_EINVAL;
  if (lim->max_rows <= 0 || lim->max_nodes_total <= 0 || lim->max_nodes_per_tree <= 0 || lim->max_prefix < 0 ||
      lim->n_heads <= 0 || lim->head_dim <= 0 || lim->hidden <= 0 || lim->vocab <= 0)
    return CASCADE_EINVAL;
  if (lim->max_nodes_per_tree > CASCADE_MAX_TREE || lim->vocab > CASCADE_MAX_VOCAB || lim->head_dim > 256 ||
      lim->max_nodes_per_tree > lim->max_nodes_total)
    return CASCADE_ESHAPE;
  cascade_ctx* c = new (std::nothrow) cascade_ctx;
  if (!c) return CASCADE_ENOMEM;
  memset(c, 0, sizeof(*c));
  c->stream = (hipStream_t)hip_stream;
  c->lim = *lim;
  hipError_t e = hipGetDevice(&c->device);
  if (e != hipSuccess) { delete c; return hip_fail(e); }
  e = hipDeviceGetAttribute(&c->n_cu, hipDeviceAttributeMultiprocessorCount, c->device);
  if (e != hipSuccess || c->n_cu <= 0) { delete c; return hip_fail(e != hipSuccess ? e : hipErrorInvalidDevice); }
  // split-KV partials: up to 16 splits, capped at 256 MiB (fewer splits are used if it does not fit)
  const size_t per_split = (size_t)lim->max_nodes_total * lim->n_heads * (lim->head_dim + 2) * sizeof(float);
  size_t attn = per_split * 16;
  const size_t cap = (size_t)256 << 20;
  if (attn > cap) attn = cap;
  c->attn_ws_bytes = align_up(attn, 256);
  // packed hidden states: two operands (cond, uncond), rows rounded up to 256, 2 bytes per element
  c->hpack_ws_bytes = align_up((size_t)2 * ((lim->max_nodes_total + 255) / 256 * 256) * lim->hidden * 2, 256);
  c->ws_bytes = 256 + c->attn_ws_bytes + c->hpack_ws_bytes;
  e = hipMalloc((void**)&c->ws, c->ws_bytes);
  if (e != hipSuccess) { delete c; (void)hipGetLastError(); return CASCADE_ENOMEM; }
  c->dev_status = (int*)c->ws;
  c->attn_ws = c->ws + 256;
  c->hpack_ws = c->attn_ws + c->attn_ws_bytes;
  e = hipMemsetAsync(c->ws, 0, 256, c->stream);
  if (e != hipSuccess) { (void)hipFree(c->ws); delete c; return hip_fail(e); }
  *out = c;
  return CASCADE_OK;
}

int cascade_set_kernel_timing(cascade_ctx* ctx, int enable) {
  if (!ctx) return CASCADE_EINVAL;
  if (enable && !ctx->ev) {
    const int n = CASCADE_K_COUNT * TIMING_RING * 2;
    ctx->ev = new (std::nothrow) hipEvent_t[n];
    if (!ctx->ev) return CASCADE_ENOMEM;
    for (int i = 0; i < n; ++i) {
      hipError_t e = hipEventCreate(&ctx->ev[i]);
      if (e != hipSuccess) {
        for (int j = 0; j < i; ++j) (void)hipEventDestroy(ctx->ev[j]);
        delete[] ctx->ev;
        ctx->ev = nullptr;
        return hip_fail(e);
      }
    }
  }
  ctx->timing = enable != 0;
  for (int k = 0; k < CASCADE_K_COUNT; ++k) ctx->ev_used[k] = 0;
  return CASCADE_OK;
}

int cascade_read_kernel_timing(cascade_ctx* ctx, int kernel_id, double* total_ms, int32_t* launches) {
  if (!ctx || !total_ms || !launches || kernel_id < 0 || kernel_id >= CASCADE_K_COUNT) return CASCADE_EINVAL;
  *total_ms = 0.0;
  *launches = 0;
  if (!ctx->ev) return CASCADE_OK;
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(e);
  double sum = 0.0;
  const int n = ctx->ev_used[kernel_id];
  for (int i = 0; i < n; ++i) {
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, ctx->ev[(kernel_id * TIMING_RING + i) * 2], ctx->ev[(kernel_id * TIMING_RING + i) * 2 + 1]);
    if (e != hipSuccess) return hip_fail(e);
    sum += ms;
  }
  *total_ms = sum;
  *launches = n;
  ctx->ev_used[kernel_id] = 0;
  return CASCADE_OK;
}

int cascade_destroy(cascade_ctx* ctx) {
  if (!ctx) return CASCADE_EINVAL;
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (ctx->ev) {
    for (int i = 0; i < CASCADE_K_COUNT * TIMING_RING * 2; ++i) (void)hipEventDestroy(ctx->ev[i]);
    delete[] ctx->ev;
  }
  hipError_t e2 = hipFree(ctx->ws);
  delete ctx;
  if (e != hipSuccess) return hip_fail(e);
  if (e2 != hipSuccess) return hip_fail(e2);
  return CASCADE_OK;
}

int64_t cascade_workspace_bytes(const cascade_ctx* ctx) { return ctx ? (int64_t)ctx->ws_bytes : 0; }

int cascade_device_status(cascade_ctx* ctx) {
  if (!ctx) return CASCADE_EINVAL;
  int flag = 0;
  hipError_t e = hipMemcpyAsync(&flag, ctx->dev_status, sizeof(int), hipMemcpyDeviceToHost, ctx->stream);
  if (e != hipSuccess) return hip_fail(e);
  e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(e);
  if (flag) {
    // cleared by a tiny kernel-free copy of a host zero (no memset node, so the call stays capturable-free)
    static const int zero = 0;
    e = hipMemcpyAsync(ctx->dev_status, &zero, sizeof(int), hipMemcpyHostToDevice, ctx->stream);
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return hip_fail(e);
    return CASCADE_ETREE;
  }
  return CASCADE_OK;
}

int tree_verify_attn(cascade_ctx* ctx, const tree_attn_args* a) {
  if (!ctx || !a) return CASCADE_EINVAL;
  if (!a->node_off || !a->parent || !a->prefix_len || !a->q || !a->k_tree || !a->v_tree || !a->out) return CASCADE_EINVAL;
  if (a->n_rows < 0 || a->n_nodes_total < 0 || a->max_nodes_per_tree < 0 || a->max_prefix_len < 0) return CASCADE_EINVAL;
  if (a->max_prefix_len > 0 && (!a->k_cache || !a->v_cache)) return CASCADE_EINVAL;
  if (a->dtype != CASCADE_F32 && a->dtype != CASCADE_BF16) return CASCADE_EDTYPE;
  if (a->n_heads <= 0 || a->n_kv_heads <= 0 || a->head_dim <= 0 || bad_float(a->scale) || a->scale < 0.f) return CASCADE_EINVAL;
  if (a->n_heads % a->n_kv_heads != 0) return CASCADE_ESHAPE;
  const cascade_limits& L = ctx->lim;
  if (a->n_rows > L.max_rows || a->n_nodes_total > L.max_nodes_total || a->max_nodes_per_tree > L.max_nodes_per_tree ||
      a->max_prefix_len > L.max_prefix || a->n_heads > L.n_heads || a->head_dim > L.head_dim)
    return CASCADE_ESHAPE;
  if (a->dtype == CASCADE_BF16) {
    if (a->head_dim != 64 && a->head_dim != 128) return CASCADE_ESHAPE;
    if ((a->cache_stride_row % 8) || (a->cache_stride_head % 8) || (a->cache_stride_pos % 8)) return CASCADE_ESHAPE;
  } else {
    if (a->head_dim > 256) return CASCADE_ESHAPE;
  }
  if (a->cache_stride_pos < a->head_dim && a->max_prefix_len > 1) return CASCADE_ESHAPE;
  if (a->n_rows == 0 || a->n_nodes_total == 0) return CASCADE_OK;
  hipError_t e = (a->dtype == CASCADE_BF16) ? launch_tree_attn_bf16(ctx, a) : launch_tree_attn_f32(ctx, a);
  return e == hipSuccess ? CASCADE_OK : hip_fail(e);
}

// --------------------------------------------------------------------------------------------
// tree_verify_attn_static: the same attention for callers that cannot allocate.  Everything the
// kernels need beyond inputs and outputs (the precondition flag word and the split-KV partials)
// lives in this file-scope device array instead of a context workspace.  Every GPU the library
// runs on holds its own copy at its own address until the process ends; the name below is only a
// host-side handle for hipGetSymbolAddress, never a pointer that may be handed to a kernel.
static __device__ __align__(256) unsigned char scratch[CASCADE_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_STATIC_DEVICES = 64;
unsigned char* g_scratch_ptr[MAX_STATIC_DEVICES];   // device address of `scratch`, per device (null until first use)
std::mutex g_scratch_mutex;

// first word of the scratch array: cleared before the launch, copied out after it
__global__ void static_status_kernel(int* flag, int* copy_to) {
  if (copy_to) *copy_to = *flag;
  else *flag = 0;
}

// device address of this device's copy of the array (looked up once per device, with that device current)
int static_scratch(int device, unsigned char** out) {
  if (device < 0 || device >= MAX_STATIC_DEVICES) return CASCADE_ESHAPE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (!ptr) return CASCADE_EHIP;
    g_scratch_ptr[device] = (unsigned char*)ptr;
  }
  *out = g_scratch_ptr[device];
  return CASCADE_OK;
}

}  // namespace

int tree_verify_attn_static(void* hip_stream, const tree_attn_args* a, int32_t* status_out) {
  if (!a) return CASCADE_EINVAL;
  if (a->n_rows < 0 || a->n_nodes_total < 0 || a->n_heads <= 0 || a->head_dim <= 0 || a->max_nodes_per_tree < 0 || a->max_prefix_len < 0)
    return CASCADE_EINVAL;
  // the stated maximum: beyond it not even two splits' partials fit the array
  if ((int64_t)a->n_nodes_total * a->n_heads > CASCADE_STATIC_MAX_QUERY_ROWS || a->head_dim > 128 ||
      a->max_nodes_per_tree > CASCADE_MAX_TREE)
    return CASCADE_ESHAPE;
  int device = -1;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return hip_fail(e);
  unsigned char* base = nullptr;
  int st = static_scratch(device, &base);
  if (st != CASCADE_OK) return st;
  // a context on the stack that points into the static array: no workspace of its own, no timing events
  cascade_ctx local;
  memset(&local, 0, sizeof(local));
  local.stream = (hipStream_t)hip_stream;
  local.device = device;
  local.lim.max_rows = a->n_rows;
  local.lim.max_nodes_total = a->n_nodes_total;
  local.lim.max_nodes_per_tree = a->max_nodes_per_tree;
  local.lim.max_prefix = a->max_prefix_len;
  local.lim.n_heads = a->n_heads;
  local.lim.head_dim = a->head_dim;
  local.ws = (char*)base;
  local.ws_bytes = CASCADE_STATIC_SCRATCH_BYTES;
  local.dev_status = (int*)base;
  local.attn_ws = (char*)base + 256;
  local.attn_ws_bytes = CASCADE_STATIC_SCRATCH_BYTES - 256;
  // the flag word keeps the previous call's value: cleared by a one-thread kernel (not a memset node, so
  // that a caller may capture the call into a graph)
  hipLaunchKernelGGL(static_status_kernel, dim3(1), dim3(1), 0, local.stream, local.dev_status, (int*)nullptr);
  e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e);
  st = tree_verify_attn(&local, a);   // same validation, same dispatch, same kernels
  if (st != CASCADE_OK) return st;
  if (status_out) {
    hipLaunchKernelGGL(static_status_kernel, dim3(1), dim3(1), 0, local.stream, local.dev_status, (int*)status_out);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
  }
  return CASCADE_OK;
}

int lmhead_softmax_cfg(cascade_ctx* ctx, const lmhead_args* a) {
  if (!ctx || !a) return CASCADE_EINVAL;
  if (!a->h_cond || !a->w || !a->logits || !a->row_max || !a->row_thr || !a->row_lse) return CASCADE_EINVAL;
  if (a->dtype != CASCADE_F32 && a->dtype != CASCADE_BF16) return CASCADE_EDTYPE;
  if (a->n_nodes < 0 || a->hidden <= 0 || a->vocab <= 0) return CASCADE_EINVAL;
  if (bad_float(a->cfg_scale) || bad_float(a->temperature) || !(a->temperature > 0.f)) return CASCADE_EINVAL;
  const cascade_limits& L = ctx->lim;
  if (a->n_nodes > L.max_nodes_total || a->hidden > L.hidden || a->vocab > L.vocab || a->vocab > CASCADE_MAX_VOCAB)
    return CASCADE_ESHAPE;
  if (a->w_layout != CASCADE_W_ROWMAJOR && a->w_layout != CASCADE_W_PACKED32) return CASCADE_EINVAL;
  if (a->cfg_mix != CASCADE_CFG_MIX_LOGITS && a->cfg_mix != CASCADE_CFG_MIX_HIDDEN) return CASCADE_EINVAL;
  if (a->dtype == CASCADE_BF16) {
    if ((a->hidden % 128) || (a->vocab % 64)) return CASCADE_ESHAPE;
  } else {
    if (a->hidden > 8192) return CASCADE_ESHAPE;
    if (a->w_layout != CASCADE_W_ROWMAJOR) return CASCADE_EDTYPE;
  }
  if (a->n_nodes == 0) return CASCADE_OK;
  hipError_t e = (a->dtype == CASCADE_BF16) ? launch_lmhead_bf16(ctx, a) : launch_lmhead_f32(ctx, a);
  if (e != hipSuccess) return hip_fail(e);
  e = launch_row_stats(ctx, a);
  return e == hipSuccess ? CASCADE_OK : hip_fail(e);
}

int cascade_pack_lmhead_w(cascade_ctx* ctx, const void* w, int32_t vocab, int32_t hidden, void* w_packed) {
  if (!ctx || !w || !w_packed || w == w_packed) return CASCADE_EINVAL;
  if (vocab <= 0 || hidden <= 0) return CASCADE_EINVAL;
  if ((vocab % 64) || (hidden % 128)) return CASCADE_ESHAPE;
  hipError_t e = launch_pack_w(ctx, w, vocab, hidden, w_packed);
  return e == hipSuccess ? CASCADE_OK : hip_fail(e);
}

int cascade_accept(cascade_ctx* ctx, const accept_args* a_in) {
  if (!ctx || !a_in) return CASCADE_EINVAL;
  accept_args local = *a_in;
  if (local.feature_space == CASCADE_FEATURES_LOGITS) {
    // similarity measured on the mixed logits: the same kernels with the logits rows as features
    local.h_cond = local.logits;
    local.h_dtype = CASCADE_F32;
    local.hidden = local.vocab;
  } else if (local.feature_space != CASCADE_FEATURES_HIDDEN) {
    return CASCADE_EINVAL;
  }
  const accept_args* a = &local;
  if (!a->node_off || !a->parent || !a->token || !a->h_cond || !a->logits || !a->row_thr || !a->row_lse || !a->q_tok ||
      !a->m_int || !a->m_conv || !a->cos_parent || !a->n_int || !a->n_conv)
    return CASCADE_EINVAL;
  if (a->h_dtype != CASCADE_F32 && a->h_dtype != CASCADE_BF16) return CASCADE_EDTYPE;
  if (a->n_prompts < 0 || a->n_nodes_total < 0 || a->hidden <= 0 || a->vocab <= 0) return CASCADE_EINVAL;
  if (bad_float(a->tau_pos) || bad_float(a->tau_seq)) return CASCADE_EINVAL;
  const cascade_limits& L = ctx->lim;
  const bool on_logits = a->feature_space == CASCADE_FEATURES_LOGITS;
  if (a->n_nodes_total > L.max_nodes_total || (!on_logits && a->hidden > L.hidden) || a->vocab > L.vocab) return CASCADE_ESHAPE;
  if (a->h_dtype == CASCADE_BF16 && (a->hidden % 8)) return CASCADE_ESHAPE;
  if (a->n_prompts == 0 || a->n_nodes_total == 0) return CASCADE_OK;
  hipError_t e = launch_accept(ctx, a);
  return e == hipSuccess ? CASCADE_OK : hip_fail(e);
}

int select_path(cascade_ctx* ctx, const select_args* a) {
  if (!ctx || !a) return CASCADE_EINVAL;
  if (!a->node_off || !a->parent || !a->token || !a->q_tok || !a->m_int || !a->m_conv || !a->n_int || !a->n_conv || !a->u ||
      !a->u_bonus || !a->logits || !a->row_thr || !a->row_lse || !a->accept_len || !a->emitted || !a->terminal || !a->tvd_used)
    return CASCADE_EINVAL;
  if (a->n_prompts < 0 || a->n_nodes_total < 0 || a->vocab <= 0 || a->max_depth < 0) return CASCADE_EINVAL;
  if (a->max_depth > 0 && !a->path_nodes) return CASCADE_EINVAL;
  if (a->mode != CASCADE_WALK_SEQUENTIAL && a->mode != CASCADE_WALK_LONGEST) return CASCADE_EINVAL;
  if (bad_float(a->eps_tvd) || a->eps_tvd < 0.f) return CASCADE_EINVAL;
  const cascade_limits& L = ctx->lim;
  if (a->n_nodes_total > L.max_nodes_total || a->vocab > L.vocab || a->max_depth > CASCADE_MAX_DEPTH) return CASCADE_ESHAPE;
  if (a->draft_dist) {
    if (a->mode != CASCADE_WALK_SEQUENTIAL) return CASCADE_EINVAL;
    if (a->vocab % 4) return CASCADE_ESHAPE;
    if (((uintptr_t)a->draft_dist | (uintptr_t)a->logits) & 15) return CASCADE_EINVAL;
  }
  if (a->n_prompts == 0) return CASCADE_OK;
  hipError_t e = a->draft_dist ? launch_select_residual(ctx, a) : launch_select(ctx, a);
  return e == hipSuccess ? CASCADE_OK : hip_fail(e);
}

int kv_commit(cascade_ctx* ctx, const kv_commit_args* a) {
  if (!ctx || !a) return CASCADE_EINVAL;
  if (!a->node_off || !a->row_prompt || !a->accept_len || !a->k_tree || !a->v_tree || !a->k_cache || !a->v_cache ||
      !a->prefix_len || !a->prefix_len_out || a->prefix_len == a->prefix_len_out)
    return CASCADE_EINVAL;
  if (a->dtype != CASCADE_F32 && a->dtype != CASCADE_BF16) return CASCADE_EDTYPE;
  if (a->n_rows < 0 || a->n_prompts < 0 || a->n_nodes_total < 0 || a->max_depth < 0 || a->n_layers < 0 || a->n_kv_heads <= 0 ||
      a->head_dim <= 0 || a->prefix_cap < 0)
    return CASCADE_EINVAL;
  if (a->max_depth > 0 && !a->path_nodes) return CASCADE_EINVAL;
  const int64_t e = a->dtype == CASCADE_BF16 ? 2 : 4;
  const int64_t strides[4] = {a->cache_stride_layer, a->cache_stride_row, a->cache_stride_head, a->cache_stride_pos};
  for (int i = 0; i < 4; ++i)
    if (strides[i] < 0 || (strides[i] * e) % 16) return CASCADE_ESHAPE;
  if ((a->head_dim * e) % 16 || a->cache_stride_pos < a->head_dim) return CASCADE_ESHAPE;
  if (((uintptr_t)a->k_tree | (uintptr_t)a->v_tree | (uintptr_t)a->k_cache | (uintptr_t)a->v_cache) & 15) return CASCADE_EINVAL;
  const cascade_limits& L = ctx->lim;
  if (a->n_rows > L.max_rows || a->n_nodes_total > L.max_nodes_total || a->max_depth > CASCADE_MAX_DEPTH) return CASCADE_ESHAPE;
  if ((int64_t)a->n_rows * (a->max_depth + 1) > 0x7fffffff || a->n_layers > 65535) return CASCADE_ESHAPE;
  if (a->n_rows == 0 || a->n_layers == 0) return CASCADE_OK;
  if (a->n_prompts == 0) return CASCADE_EINVAL;
  hipError_t err = launch_kv_commit(ctx, a);
  return err == hipSuccess ? CASCADE_OK : hip_fail(err);
}

int convergence_weights(cascade_ctx* ctx, const conv_weight_args* a) {
  if (!ctx || !a) return CASCADE_EINVAL;
  if (!a->features || !a->weights) return CASCADE_EINVAL;
  if (a->dtype != CASCADE_F32 && a->dtype != CASCADE_BF16) return CASCADE_EDTYPE;
  if (a->n_seqs < 0 || a->seq_len < 0 || a->hidden <= 0) return CASCADE_EINVAL;
  if (bad_float(a->tau_seq) || bad_float(a->c)) return CASCADE_EINVAL;
  const int64_t row_bytes = (int64_t)a->hidden * (a->dtype == CASCADE_BF16 ? 2 : 4);
  if ((row_bytes % 16) || row_bytes > 16384) return CASCADE_ESHAPE;
  if ((uintptr_t)a->features & 15) return CASCADE_EINVAL;
  if ((int64_t)a->n_seqs * ((a->seq_len + 7) / 8 + 1) > 0x3fffffff) return CASCADE_ESHAPE;
  if (a->n_seqs == 0 || a->seq_len == 0) return CASCADE_OK;
  hipError_t err = launch_conv_weights(ctx, a);
  return err == hipSuccess ? CASCADE_OK : hip_fail(err);
}

}  // extern "C"
