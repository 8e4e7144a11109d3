/*
 * cascade_verify.h — C ABI of the MI355X (gfx950) tree-verification step of CASCADE
 * speculative image decoding.
 *
 * One verification step = four calls, in this order, on one HIP stream:
 *
 *   tree_verify_attn    target attention of the drafted token tree against the prefix KV cache
 *   lmhead_softmax_cfg  final projection + classifier-free-guidance mix + top-k + softmax statistics
 *   cascade_accept      per-node quantities of the relaxed acceptance rule (Eq. 1, Eq. 2, Eq. 3)
 *   select_path         the walk of Alg. 2 (budget, acceptance test) and the correction step of Alg. 1
 *
 * and, between two steps, kv_commit appends the keys / values of the tokens that were kept to the
 * prefix cache.
 *
 * General conventions
 * -------------------
 *  - C99, no C++ types.  Every pointer inside an args struct is a DEVICE pointer unless its
 *    comment says HOST.  The args structs themselves and the ctx handle live on the host.
 *  - Ownership: the caller owns every buffer.  The library borrows them until the ctx stream has
 *    run the enqueued work.  Outputs are caller-allocated.  The library allocates device memory
 *    only inside cascade_create (one workspace, freed by cascade_destroy).
 *  - Asynchrony: every compute call enqueues kernels on the ctx stream and returns; it never
 *    synchronises the device.
 *  - Errors: 0 = CASCADE_OK, negative = cascade_status.  Errors detectable from host-visible
 *    arguments (null pointers, shapes, limits, dtype) are reported before anything is enqueued and
 *    leave outputs untouched.  HIP runtime failures give CASCADE_EHIP.  Preconditions on device
 *    arrays (below) cannot be seen by the host; kernels never read or write out of bounds because
 *    of them, they record a flag that cascade_device_status returns.
 *  - Packing: a *prompt* owns one token tree.  node_off[b]..node_off[b+1] are prompt b's nodes in
 *    the packed arrays; parent[] holds indices LOCAL to the tree; node 0 of each tree is its root
 *    (the last token already emitted), parent == -1, and parent[i] < i for i > 0.  Siblings are
 *    tried in ascending node index.  A node has at most CASCADE_MAX_WIDTH children.
 *  - With classifier-free guidance a prompt has two attention rows (conditional, unconditional)
 *    sharing the tree; attention is packed per ROW, the other three calls per PROMPT.
 */
#ifndef CASCADE_VERIFY_H
#define CASCADE_VERIFY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cascade_ctx cascade_ctx;   /* opaque; owns the workspace; bound to one HIP stream */

typedef enum {
  CASCADE_OK = 0,
  CASCADE_EINVAL = -1,    /* null pointer, negative size, NaN threshold, bad enum */
  CASCADE_ESHAPE = -2,    /* a size exceeds the ctx limits or breaks a divisibility rule */
  CASCADE_EDTYPE = -3,    /* dtype not supported by this call */
  CASCADE_ENOMEM = -4,    /* workspace allocation failed (cascade_create only) */
  CASCADE_EHIP = -5,      /* HIP runtime error; text via cascade_strerror(CASCADE_EHIP) */
  CASCADE_ETREE = -6      /* a device-side precondition was violated (cascade_device_status) */
} cascade_status;

typedef enum { CASCADE_F32 = 0, CASCADE_BF16 = 1 } cascade_dtype;

/* SEQUENTIAL is Alg. 2 as printed (siblings tried in order, first accepted child descends).
 * LONGEST simulates the same rule along every root-to-leaf path on its own and keeps the path
 * with the longest accepted prefix (ties: smallest leaf index). */
typedef enum { CASCADE_WALK_SEQUENTIAL = 0, CASCADE_WALK_LONGEST = 1 } cascade_walk_mode;

#define CASCADE_MAX_WIDTH 64      /* children per node */
#define CASCADE_MAX_TREE 1024     /* nodes per tree */
#define CASCADE_MAX_DEPTH 64      /* levels below the root */
#define CASCADE_MAX_VOCAB 65536   /* image(+text) vocabulary entries */

/* Upper bounds used to size the workspace.  All HOST values. */
typedef struct {
  int32_t max_rows;            /* attention rows S (2 per prompt with guidance) */
  int32_t max_nodes_total;     /* packed nodes over all rows */
  int32_t max_nodes_per_tree;  /* <= CASCADE_MAX_TREE */
  int32_t max_prefix;          /* prefix KV positions per row */
  int32_t n_heads;             /* query heads */
  int32_t head_dim;            /* 64 or 128 for bf16; any multiple of 4 up to 256 for f32 */
  int32_t hidden;
  int32_t vocab;               /* <= CASCADE_MAX_VOCAB */
} cascade_limits;

/* Allocates the workspace on the current device and binds the ctx to hip_stream (a hipStream_t
 * passed as void*; NULL = the default stream).  Returns CASCADE_OK and stores the handle, or a
 * negative status and stores NULL. */
int cascade_create(cascade_ctx** out, const cascade_limits* limits, void* hip_stream);
int cascade_destroy(cascade_ctx* ctx);
/* Static text for a status; for CASCADE_EHIP the text of the last HIP error seen by this thread. */
const char* cascade_strerror(int status);
/* Synchronises the ctx stream, returns CASCADE_OK or CASCADE_ETREE if any kernel since the last
 * call met a violated precondition (parent[i] >= i, more than CASCADE_MAX_WIDTH children, token
 * outside [0, vocab), tree deeper than max_depth, a tree with more nodes than the bound its launch was
 * sized for - tree_attn_args.max_nodes_per_tree, cascade_limits.max_nodes_per_tree - whose nodes are
 * then not verified: attention rows of such a tree are written as zeros with lse = -inf, acceptance
 * scalars beyond the bound as zeros, the walk sees only the nodes inside the bound; a kv_commit row
 * without room or with a path entry outside its tree), and clears the flag. */
int cascade_device_status(cascade_ctx* ctx);
/* Bytes of device workspace the ctx holds (HOST query). */
int64_t cascade_workspace_bytes(const cascade_ctx* ctx);

/* Optional per-kernel timing, for benchmarks.  When enabled, every launch of the kernels below
 * carries a start and a stop HIP event that receive the dispatch's own begin / end timestamps (at
 * most 2048 launches per kernel are kept between reads; later ones are not timed).  cascade_read_kernel_timing synchronises the
 * stream, returns the summed elapsed milliseconds and the number of timed launches of one kernel,
 * and resets that kernel's counter.  Timing is off by default and costs nothing when off. */
typedef enum {
  CASCADE_K_ATTN = 0,        /* tree attention main kernel */
  CASCADE_K_ATTN_MERGE = 1,  /* split-KV merge */
  CASCADE_K_LMHEAD = 2,      /* projection + guidance mix */
  CASCADE_K_ROW_STATS = 3,   /* row max / top-k threshold / log-sum-exp */
  CASCADE_K_ACCEPT = 4,
  CASCADE_K_SELECT = 5,
  CASCADE_K_COMMIT = 6,      /* kv_commit */
  CASCADE_K_WEIGHTS = 7,     /* convergence_weights */
  CASCADE_K_PACK = 8,        /* hidden-state repacking in front of the packed projection */
  CASCADE_K_COUNT = 9
} cascade_kernel_id;
int cascade_set_kernel_timing(cascade_ctx* ctx, int enable);
int cascade_read_kernel_timing(cascade_ctx* ctx, int kernel_id, double* total_ms, int32_t* launches);

/* Measurement aids for roofline reports (not part of the method): what this device sustains.
 * Both calls run a small kernel of their own on the ctx stream, wait for it, and return HOST
 * numbers.  cascade_measure_hbm_read streams `bytes` (>= 16, buf 16-byte aligned, DEVICE, only
 * read) `repeats` (1..1000) times with plain coalesced 16-byte loads and returns 1e9 bytes per
 * second; give it a buffer larger than the 256 MB last-level cache to measure HBM.
 * cascade_measure_mfma_bf16 runs `iters` (1..2^20) rounds of eight independent 32x32x16 bf16 MFMA
 * chains per wave, operands in registers, on 32 waves per compute unit, and returns 1e12 flop/s. */
int cascade_measure_hbm_read(cascade_ctx* ctx, const void* buf, int64_t bytes, int32_t repeats, double* gb_per_s);
int cascade_measure_mfma_bf16(cascade_ctx* ctx, int32_t iters, double* tflop_per_s);

/* ---------------------------------------------------------------------------------------------
 * tree_verify_attn — the target model's parallel pass over the drafted tree, one decoder layer's
 * attention (Preliminaries: the target evaluates all draft tokens in one parallel forward pass,
 * each conditioned on the prefix plus its own draft path; tree decoding with a tree mask).
 *
 * For row s, query head g (kv head g / (n_heads / n_kv_heads)) and node i of the row:
 *     J   = { prefix positions 0 .. prefix_len[s]-1 }  U  { tree nodes a : a ancestor of i, or a == i }
 *     out = sum_{j in J} softmax_j( scale * <q_i, k_j> ) * v_j
 * The ancestor mask is derived from parent[] on chip; it is never materialised in HBM.
 *
 * Layouts (element type = dtype; strides in ELEMENTS):
 *     q, out           [N, n_heads, head_dim]       contiguous, N = node_off[n_rows]
 *     k_tree, v_tree   [N, n_kv_heads, head_dim]    contiguous
 *     k_cache, v_cache element (s, kvh, pos, d) at s*cache_stride_row + kvh*cache_stride_head
 *                      + pos*cache_stride_pos + d   (d contiguous; strides multiples of 8 for bf16)
 *     lse              [N, n_heads] float32, log-sum-exp of the scaled scores over J; may be NULL
 * out is written in dtype (bf16: round to nearest even); accumulation and softmax are float32.
 */
typedef struct {
  int32_t n_rows;
  const int32_t* node_off;    /* [n_rows+1] DEVICE */
  const int32_t* parent;      /* [N] DEVICE, local indices */
  const int32_t* prefix_len;  /* [n_rows] DEVICE */
  int32_t n_nodes_total;      /* HOST copy of node_off[n_rows] */
  int32_t max_nodes_per_tree; /* HOST upper bound on any row's node count */
  int32_t max_prefix_len;     /* HOST upper bound on any prefix_len[s] */
  cascade_dtype dtype;
  int32_t n_heads, n_kv_heads, head_dim;
  float scale;                /* 0 => 1/sqrt(head_dim) */
  const void *q, *k_tree, *v_tree;
  const void *k_cache, *v_cache;
  int64_t cache_stride_row, cache_stride_head, cache_stride_pos;
  void* out;
  float* lse;                 /* nullable */
} tree_attn_args;
int tree_verify_attn(cascade_ctx* ctx, const tree_attn_args* args);

/* tree_verify_attn_static — tree_verify_attn for callers that cannot allocate device memory and so
 * cannot hold a cascade_ctx: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels, same results; the precondition flag and the
 * split-KV partials live in a static device array of CASCADE_STATIC_SCRATCH_BYTES that every GPU
 * the library runs on holds until the process ends.  The call allocates nothing and frees nothing.
 *   hip_stream   the hipStream_t (as void*) the kernels are enqueued on; NULL = the default stream
 *   status_out   DEVICE int32, nullable: receives 0, or the non-zero flag word if a tree precondition
 *                was violated during this call (what cascade_device_status reports for a ctx)
 * Limits: n_nodes_total * n_heads <= CASCADE_STATIC_MAX_QUERY_ROWS and head_dim <= 128, otherwise
 * CASCADE_ESHAPE and nothing is enqueued (the other checks are tree_verify_attn's).  Within the
 * limits the number of key splits is reduced to what fits the array.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two threads) race on it; calls on one stream, or otherwise ordered, are safe. */
#define CASCADE_STATIC_MAX_QUERY_ROWS 32768
#define CASCADE_STATIC_SCRATCH_BYTES (64u * 1024u * 1024u + 256u)
int tree_verify_attn_static(void* hip_stream, const tree_attn_args* args, int32_t* status_out);

/* ---------------------------------------------------------------------------------------------
 * lmhead_softmax_cfg — final projection at every tree node (Sec. 4.2: the O(hV) projection is
 * the dominant term), guidance mix, temperature, top-k and softmax statistics (App.
 * "Configuration Details": guidance scale 3 or 5, temperature 1, top-k 2000, top-p 1).
 *
 *     l_c = h_cond W^T,  l_u = h_uncond W^T            (float32 accumulation)
 *     g   = l_u + cfg_scale * (l_c - l_u)              (h_uncond == NULL:  g = l_c)
 *     g   = g / temperature
 *     row_thr = top_k-th largest g of the row          (top_k <= 0 or >= vocab: -inf, no filter)
 *     row_max = max_v g,  row_lse = log sum_{g_v >= row_thr} exp(g_v)
 * The node's target distribution is  q(v) = g_v >= row_thr ? exp(g_v - row_lse) : 0 ; it is not
 * materialised.  Raw conditional / unconditional logits are never written.
 *
 *     h_cond, h_uncond [n_nodes, hidden] dtype, contiguous;  w [vocab, hidden] dtype, contiguous
 *     logits [n_nodes, vocab] float32 (mixed, after temperature, before the filter)
 *     row_max, row_thr, row_lse [n_nodes] float32
 * bf16: hidden must be a multiple of 128 and vocab a multiple of 64.
 *
 * Weight layout.  CASCADE_W_ROWMAJOR: w is [vocab, hidden] as above.  CASCADE_W_PACKED32 (bf16
 * only): w was rewritten once, at model-load time, by cascade_pack_lmhead_w into MFMA operand
 * order: for every block of 32 vocabulary rows and every 16 hidden columns, 64 x 16 bytes where
 * entry l holds W[32*block + l%32][16*step + 8*(l/32) .. +7]; blocks of one 32-row group are
 * consecutive over the hidden dimension.  A wavefront then streams the matrix as contiguous
 * 1 KiB operand loads.  Same bytes, same values: results do not depend on the layout beyond
 * float32 summation order.
 *
 * Where the guidance mix is taken.  The projection is linear and has no bias, so
 *     l_u + s (l_c - l_u) = (h_u + s (h_c - h_u)) W^T :
 * CASCADE_CFG_MIX_LOGITS (0, the formula as written above) runs both products and mixes in the
 * projection's epilogue; CASCADE_CFG_MIX_HIDDEN mixes the two hidden rows of a node first (float32,
 * in the order u + s (c - u), rounded once to bf16) and runs ONE product over n_nodes rows - half
 * the multiplications.  The only difference is that one rounding of the mixed row: about 2^-9
 * relative per element, which shows in g as an error of a few 1e-3 of the row's largest |g| at
 * guidance scale 5 (inside the 2e-2 this library's bf16 results are held to).  Honoured for bf16
 * with CASCADE_W_PACKED32; every other case runs the two products.
 */
typedef enum { CASCADE_W_ROWMAJOR = 0, CASCADE_W_PACKED32 = 1 } cascade_w_layout;
typedef enum { CASCADE_CFG_MIX_LOGITS = 0, CASCADE_CFG_MIX_HIDDEN = 1 } cascade_cfg_mix;
/* Enqueues the repacking of a bf16 [vocab, hidden] matrix (DEVICE) into w_packed (DEVICE, same
 * byte size, must not alias w).  vocab % 64 == 0, hidden % 128 == 0. */
int cascade_pack_lmhead_w(cascade_ctx* ctx, const void* w, int32_t vocab, int32_t hidden, void* w_packed);

typedef struct {
  cascade_dtype dtype;
  int32_t n_nodes, hidden, vocab;
  const void* h_cond;
  const void* h_uncond;       /* nullable => no guidance */
  const void* w;
  cascade_w_layout w_layout;
  float cfg_scale, temperature;
  int32_t top_k;
  cascade_cfg_mix cfg_mix;    /* where the guidance mix is taken (see above); 0 = on the logits */
  float* logits;
  float *row_max, *row_thr, *row_lse;
} lmhead_args;
int lmhead_softmax_cfg(cascade_ctx* ctx, const lmhead_args* args);

/* ---------------------------------------------------------------------------------------------
 * cascade_accept — what the relaxed acceptance rule needs at every non-root node a with parent p
 * (Sec. 4.1 cosine similarity of target hidden states; Eq. 1 interchangeable set; Eq. 2
 * convergence set; Eq. 3 aggregated mass).  Q = the distribution of p (the one that verifies a):
 *
 *     q_tok[a]  = Q[token[a]]
 *     I_a = { siblings b != a : cos(F_a, F_b) >= tau_pos },  n_int[a]  = |I_a|
 *     C_a = { children b of a : cos(F_a, F_b) >= tau_seq },  n_conv[a] = |C_a|
 *     m_int[a]  = sum of Q[t] over distinct t in tokens(I_a) \ {token[a]}
 *     m_conv[a] = sum of Q[t] over distinct t in tokens(C_a) \ {token[a]} \ tokens(I_a)
 *     cos_parent[a] = cos(F_p, F_a)
 * F = rows of h_cond (the conditional row's final hidden state, the LM-head input), or, with
 * feature_space = CASCADE_FEATURES_LOGITS, the node's row of mixed logits (App. "Preliminary
 * Findings": cosine similarity of target logits as the alternative measure; h_cond, h_dtype and
 * hidden are then ignored).  cos is 0 when
 * a norm is 0.  A threshold > 1 disables that relaxation.  Root entries are written as 0.
 * Dot products and norms accumulate in float32.
 *
 *     node_off [n_prompts+1], parent/token [N] int32;  h_cond [N, hidden] h_dtype
 *     logits [N, vocab] float32 and row_thr/row_lse [N] as written by lmhead_softmax_cfg
 *     outputs [N]: q_tok, m_int, m_conv, cos_parent float32;  n_int, n_conv int32
 */
typedef enum { CASCADE_FEATURES_HIDDEN = 0, CASCADE_FEATURES_LOGITS = 1 } cascade_feature_space;
typedef struct {
  cascade_dtype h_dtype;
  int32_t n_prompts, n_nodes_total, hidden, vocab;
  const int32_t *node_off, *parent, *token;
  const void* h_cond;
  const float *logits, *row_thr, *row_lse;
  float tau_pos, tau_seq;
  float *q_tok, *m_int, *m_conv, *cos_parent;
  int32_t *n_int, *n_conv;
  cascade_feature_space feature_space;   /* 0 = hidden states */
} accept_args;
int cascade_accept(cascade_ctx* ctx, const accept_args* args);

/* ---------------------------------------------------------------------------------------------
 * select_path — Alg. 2's walk over the scalars of cascade_accept, then Alg. 1's correction step.
 *
 * SEQUENTIAL, per prompt:  cur = root, tvd = 0; at each level try the children a of cur in
 * ascending index:  q = q_tok[a];  if n_int[a] > 0 and tvd + m_int[a] <= eps_tvd: q += m_int[a],
 * tvd += m_int[a];  the same for (n_conv, m_conv);  a is accepted iff u[a]*draft_prob[a] < q
 * (Alg. 1's r < min(1, q/p) with 0 <= r < 1).  The first accepted child becomes cur; a level with
 * no accepted child, or a leaf, ends the walk.  The last token is drawn from the distribution of
 * cur with the tokens of the children rejected at that last level removed: the smallest v with
 * cumulative mass > u_bonus[b] * remaining mass (vocabulary order).
 * All compares and sums in float32.
 *
 * Residual walk (draft_dist != NULL; SEQUENTIAL only; vocab a multiple of 4): row a of draft_dist is
 * the full drafter distribution node a was drawn from.  The level starts with f = the distribution
 * of cur; the tried child a uses q = f[token[a]] and drafter probability draft_dist[a][token[a]]
 * (draft_prob is ignored), the relaxation masses unchanged; each rejection replaces f by Alg. 1's
 * residual norm([f - draft_dist[a]]_+) (f is kept if nothing would be left), so later siblings are
 * verified against what the earlier ones left over, and the last token is drawn from the final f
 * (no tokens are removed beyond that).  With one draft per level this is Alg. 1 exactly.
 *
 *     draft_prob [N] float32 (NULL => 1), u [N] float32 in [0,1), u_bonus [n_prompts] in [0,1)
 *     accept_len [n_prompts]; path_nodes [n_prompts, max_depth] local indices, -1 padded;
 *     emitted [n_prompts, max_depth+1]: accepted draft tokens, then the last token, -1 padded;
 *     terminal [n_prompts] local index of cur at the end; tvd_used [n_prompts] float32
 */
typedef struct {
  int32_t n_prompts, n_nodes_total, vocab, max_depth;
  cascade_walk_mode mode;
  const int32_t *node_off, *parent, *token;
  const float *q_tok, *m_int, *m_conv;
  const int32_t *n_int, *n_conv;
  const float* draft_prob;    /* nullable */
  const float* u;
  const float* u_bonus;
  float eps_tvd;
  const float *logits, *row_thr, *row_lse;
  int32_t *accept_len, *path_nodes, *emitted, *terminal;
  float* tvd_used;
  const float* draft_dist;    /* nullable; [N, vocab] => residual walk (see above) */
} select_args;
int select_path(cascade_ctx* ctx, const select_args* args);

/* ---------------------------------------------------------------------------------------------
 * kv_commit — after select_path: the tokens that are now part of the sequence get their keys and
 * values appended to the prefix cache, for every decoder layer (Preliminaries: accepted tokens are
 * appended to the prefix; iterative tree decoding forms the whole image sequence).  The root of a
 * tree is the token the previous step emitted last; its key / value were produced in this step, so
 * it goes first, then the accepted nodes in path order.  The last emitted token (correction or
 * bonus) has no key / value yet: it is the next tree's root.
 *
 * For row s with prompt b = row_prompt[s], P = prefix_len[s], n = accept_len[b]:
 *     node_0 = 0,  node_j = path_nodes[b, j-1]                       (j = 1 .. n)
 *     cache[layer, s, kvh, P + j, :] = tree[layer, node_off[s] + node_j, kvh, :]   for K and V
 *     prefix_len_out[s] = P + 1 + n
 * A row with P + 1 + n > prefix_cap is left untouched (prefix_len_out[s] = P) and a path entry
 * outside the row's tree is skipped; both set the flag cascade_device_status reports.
 * Pure copy: values are moved bit for bit.
 *
 *     k_tree, v_tree   [n_layers, N, n_kv_heads, head_dim] dtype, contiguous (N = node_off[n_rows])
 *     k_cache, v_cache element (layer, s, kvh, pos, d) at layer*cache_stride_layer +
 *                      s*cache_stride_row + kvh*cache_stride_head + pos*cache_stride_pos + d
 *                      (strides in ELEMENTS; head_dim and all strides multiples of 16 bytes)
 *     prefix_len_out   must not alias prefix_len
 */
typedef struct {
  int32_t n_rows, n_prompts;
  const int32_t* node_off;      /* [n_rows+1] DEVICE, row packing as in tree_verify_attn */
  const int32_t* row_prompt;    /* [n_rows] DEVICE (guidance rows of a prompt share its path) */
  const int32_t* accept_len;    /* [n_prompts] DEVICE, as written by select_path */
  const int32_t* path_nodes;    /* [n_prompts, max_depth] DEVICE, as written by select_path */
  int32_t max_depth;
  int32_t n_nodes_total;        /* HOST copy of node_off[n_rows] */
  cascade_dtype dtype;
  int32_t n_layers, n_kv_heads, head_dim;
  const void *k_tree, *v_tree;
  void *k_cache, *v_cache;
  int64_t cache_stride_layer, cache_stride_row, cache_stride_head, cache_stride_pos;
  int32_t prefix_cap;           /* positions allocated per (layer, row, kv head) */
  const int32_t* prefix_len;    /* [n_rows] DEVICE */
  int32_t* prefix_len_out;      /* [n_rows] DEVICE */
} kv_commit_args;
int kv_commit(cascade_ctx* ctx, const kv_commit_args* args);

/* ---------------------------------------------------------------------------------------------
 * convergence_weights — the weight mask of the drafter-training loss (Sec. "Enhancing Drafter
 * Performance", Eq. 4): over a full target-generated sequence, position k's soft cross-entropy
 * term is weighted by c when the consecutive target predictions (k, k+1) are in the convergence
 * set, i.e. cos(F_k, F_{k+1}) >= tau_seq (Eq. 2 between neighbours), and by 1 otherwise (c = 2 in
 * App. "Configuration Details").  The last position has no successor: weight 1.
 *
 *     features [n_seqs, seq_len, hidden] dtype, contiguous; hidden * sizeof(dtype) a multiple of 16
 *              and at most 16384 bytes
 *     weights  [n_seqs, seq_len] float32
 *     cos_next [n_seqs, seq_len] float32, cos(F_k, F_{k+1}); 0 at the last position; may be NULL
 * Dot products and norms accumulate in float32; cos is 0 when a norm is 0.
 */
typedef struct {
  cascade_dtype dtype;
  int32_t n_seqs, seq_len, hidden;
  const void* features;
  float tau_seq, c;
  float* weights;
  float* cos_next;            /* nullable */
} conv_weight_args;
int convergence_weights(cascade_ctx* ctx, const conv_weight_args* args);

#ifdef __cplusplus
}
#endif
#endif /* CASCADE_VERIFY_H */
