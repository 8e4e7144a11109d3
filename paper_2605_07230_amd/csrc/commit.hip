// kv_commit: append the root and the accepted path of every row's tree to that row's prefix cache,
// for all layers (Preliminaries: accepted tokens are appended to the prefix).  A pure gather /
// scatter of 16-byte pieces; one workgroup per (row, path slot, layer).
#include "common.h"

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

struct CommitParams {
  kv_commit_args a;
  int* dev_status;
  int row_vec;       // 16-byte pieces per node row (n_kv_heads * head_dim * elem / 16)
  int head_vec;      // 16-byte pieces per head
  long long sl, sr, sh, sp;   // cache strides in 16-byte pieces
  long long tree_layer_vec;   // 16-byte pieces per layer of k_tree / v_tree
};

__global__ __launch_bounds__(256) void kv_commit_kernel(CommitParams p) {
  const kv_commit_args& a = p.a;
  const int slots = a.max_depth + 1;
  const int s = blockIdx.x / slots, j = blockIdx.x % slots, layer = blockIdx.y;
  const int tid = threadIdx.x;
  const bool reporter = (j == 0 && layer == 0 && tid == 0);

  const int b = a.row_prompt[s];
  const int P = a.prefix_len[s];
  if (b < 0 || b >= a.n_prompts) {
    if (reporter) { atomicOr(p.dev_status, CASCADE_FLAG_PATH); a.prefix_len_out[s] = P; }
    return;
  }
  int n_acc = a.accept_len[b];
  if (n_acc < 0 || n_acc > a.max_depth) {
    if (reporter) { atomicOr(p.dev_status, CASCADE_FLAG_DEPTH); a.prefix_len_out[s] = P; }
    return;
  }
  if (P < 0 || P + 1 + n_acc > a.prefix_cap) {
    if (reporter) { atomicOr(p.dev_status, CASCADE_FLAG_CAPACITY); a.prefix_len_out[s] = P; }
    return;
  }
  if (reporter) a.prefix_len_out[s] = P + 1 + n_acc;
  if (j > n_acc) return;
  const int base = a.node_off[s], n_tree = a.node_off[s + 1] - base;
  const int node = (j == 0) ? 0 : a.path_nodes[(long long)b * a.max_depth + (j - 1)];
  if (node < 0 || node >= n_tree || base < 0 || base + node >= a.n_nodes_total) {
    if (layer == 0 && tid == 0) atomicOr(p.dev_status, CASCADE_FLAG_PATH);
    return;
  }
  const long long src_off = (long long)layer * p.tree_layer_vec + (long long)(base + node) * p.row_vec;
  const long long dst_off = (long long)layer * p.sl + (long long)s * p.sr + (long long)(P + j) * p.sp;
  const u32x4* ks = (const u32x4*)a.k_tree + src_off;
  const u32x4* vs = (const u32x4*)a.v_tree + src_off;
  u32x4* kd = (u32x4*)a.k_cache + dst_off;
  u32x4* vd = (u32x4*)a.v_cache + dst_off;
  for (int i = tid; i < p.row_vec; i += 256) {
    const int head = i / p.head_vec, within = i - head * p.head_vec;
    const u32x4 kx = ks[i], vx = vs[i];
    kd[(long long)head * p.sh + within] = kx;
    vd[(long long)head * p.sh + within] = vx;
  }
}

}  // namespace

hipError_t launch_kv_commit(cascade_ctx* ctx, const kv_commit_args* a) {
  const int e = a->dtype == CASCADE_BF16 ? 2 : 4;
  CommitParams p;
  p.a = *a;
  p.dev_status = ctx->dev_status;
  p.head_vec = a->head_dim * e / 16;
  p.row_vec = a->n_kv_heads * p.head_vec;
  p.sl = a->cache_stride_layer * e / 16;
  p.sr = a->cache_stride_row * e / 16;
  p.sh = a->cache_stride_head * e / 16;
  p.sp = a->cache_stride_pos * e / 16;
  p.tree_layer_vec = (long long)a->n_nodes_total * p.row_vec;
  dim3 grid((unsigned)(a->n_rows * (a->max_depth + 1)), (unsigned)a->n_layers);
  KernelTimer t(ctx, CASCADE_K_COMMIT);
  CASCADE_TIMED_LAUNCH(t, kv_commit_kernel, grid, dim3(256), 0, ctx->stream, p);
  return hipGetLastError();
}
