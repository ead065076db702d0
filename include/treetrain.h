/*
 * treetrain.h -- C ABI of the MI355X (gfx950) tree-attention hot path of "Tree Training".
 *
 * The library processes one DFS-serialised trajectory tree: every token of the tree appears once,
 * a node's tokens followed by its children's subtrees (paper Eq. 8).  In that order a node's
 * subtree is one contiguous token range, so the tree attention mask (Section "Attention Mask":
 * query i sees key j iff j <= i and both lie on a common root-to-leaf path) becomes a per-key
 * upper bound:
 *
 *        visible(i, j)  <=>  j <= i + n_prefix < kend[j]
 *
 * on the unified key axis [prefix keys ; own keys].  For own keys kend[j] = n_prefix + end of the
 * subtree of j's node; for cached prefix keys (partition boundaries, Section "Redundancy-Free Tree
 * Partitioning" and Appendix "Ancestor-Aware Attention Bias") kend[j] = INT32_MAX for ancestors of
 * the chunk and 0 for everything else in the cached slice.
 *
 * Conventions
 *   - All functions return a tt_status (0 = ok, < 0 = error); none throws or aborts.  The message
 *     for the last error on the calling thread is tt_last_error().
 *   - Arguments are validated on the host before anything is launched; a failed call launches
 *     nothing and writes nothing.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are GPU memory.  All buffers are
 *     owned by the caller; the library allocates no device memory.  Scratch comes from a
 *     caller-provided workspace (tt_tree_attn_workspace gives its size).
 *   - Device calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL = the null
 *     stream) and do not synchronise.
 *   - Inputs are const and never modified.  Outputs are overwritten, except the documented
 *     accumulators (dk_prefix_acc, dv_prefix_acc, loss_acc), which are added to.
 *   - Tensor layout is token-major: [tokens][heads][d] with d contiguous.  Query head h reads
 *     key/value head h / (hq / hkv).
 *   - Results are deterministic: the same inputs give bit-identical outputs from run to run
 *     (the paper reports exact run-to-run agreement, Appendix "Numerical Verification").
 */
#ifndef TREETRAIN_H
#define TREETRAIN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t tt_status;
#define TT_OK               0
#define TT_ERR_NULL        -1   /* a required pointer is NULL                                   */
#define TT_ERR_SHAPE       -2   /* a size is out of range or sizes are inconsistent             */
#define TT_ERR_TREE        -3   /* parent array is not a forest (out of range, self loop, cycle) */
#define TT_ERR_DTYPE       -4   /* unknown dtype code                                           */
#define TT_ERR_ALIGN       -5   /* a device pointer or stride breaks the alignment rule         */
#define TT_ERR_WORKSPACE   -6   /* workspace missing or too small                               */
#define TT_ERR_HIP         -7   /* the HIP runtime reported an error at launch                  */
#define TT_ERR_UNSUPPORTED -8   /* valid request that this build has no kernel for              */

#define TT_DTYPE_BF16 0
#define TT_DTYPE_FP32 1

/* tt_attn_desc.flags: run bf16 tensors through the slow fp32-arithmetic kernels instead of the
 * MFMA kernels (for cross-checks). */
#define TT_FLAG_REFERENCE_KERNELS 1

/* Keys per entry of the tile summaries (ktile_kend_min / ktile_kend_max). */
#define TT_KTILE 64

/* Message of the last failed call on this thread (library-owned, valid until the next call). */
const char* tt_last_error(void);
/* Library version as major*10000 + minor*100 + patch. */
int32_t tt_version(void);

/* ------------------------------------------------------------------------------------------
 * tt_tree_build_meta  (host only; needs no GPU)
 *
 * Turns a trajectory tree -- nodes with token-segment lengths, "Derivation" section -- into
 * everything the device calls need.
 *   DFS order and ranges        Eq. 8; children are visited in ascending input id.
 *   g_n, K                      number of root-to-leaf paths through node n / in total (one per
 *                               leaf; a zero-length leaf still counts).
 *   position ids                Eq. 9: total length of the strict ancestors + offset inside the
 *                               node; a root starts at its root_pos_offset (Appendix "Depth-Based
 *                               Position Offset": for a partition this is the ancestor-only depth
 *                               of the cut node's end, not the length of the cached slice).
 *   loss weights                Eq. 4: trained * g / K as one fp32 division.
 *   kend, tile summaries        the visibility bound above and its min/max per TT_KTILE keys; the
 *                               prefix region and the own region are tiled separately, each from
 *                               its own first key: n_ktiles = ceil(n_prefix/TT_KTILE) +
 *                               ceil(n_tokens/TT_KTILE).
 *
 * Inputs (host):
 *   parent[n_nodes]        parent node id, -1 for a root.  Any numbering; several roots allowed.
 *   seg_len[n_nodes]       tokens in the node, >= 0.
 *   trained[n_nodes]       1 = model output (gets a loss weight), 0 = input; NULL = all trained.
 *   root_pos_offset        NULL (= 0) or one value per root, in ascending root id.
 *   g_override, K_override NULL / 0, or the whole tree's g per node (input numbering) and K when
 *                          this forest is one partition of a larger tree.
 *   n_prefix               cached prefix keys in front of the own keys (0 = none).
 *   prefix_visible[n_prefix]  1 = ancestor of this chunk; NULL = all visible.
 * Outputs (host, caller-allocated; any may be NULL to skip it).  Per-node arrays are indexed by
 * DFS rank:
 *   dfs_order[n_nodes]     input id of the node at each DFS rank.
 *   node_start, node_end, subtree_end [n_nodes]   token ranges, own-sequence indices.
 *   node_parent[n_nodes]   DFS rank of the parent, -1 for roots.
 *   node_g[n_nodes]
 *   tok_node, tok_pos [n_tokens]
 *   tok_pred[n_tokens]     index of the token whose logits predict token t: t-1 inside a node,
 *                          the last token of the nearest non-empty ancestor at a node's first
 *                          token, -1 if there is none.
 *   tok_weight[n_tokens]   fp32.
 *   kend[n_prefix + n_tokens], ktile_kend_min, ktile_kend_max [n_ktiles].
 * Errors: TT_ERR_NULL, TT_ERR_SHAPE (negative sizes, total tokens + prefix >= 2^31 - 1),
 *   TT_ERR_TREE.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t n_nodes;
  int32_t n_tokens;   /* DFS length N                                  */
  int32_t n_leaves;   /* K                                             */
  int32_t n_roots;
  int32_t n_ktiles;   /* entries of the tile summaries                 */
} tt_meta_sizes;

tt_status tt_tree_meta_sizes(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                             int32_t n_prefix, tt_meta_sizes* out);

tt_status tt_tree_build_meta(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                             const uint8_t* trained, const int32_t* root_pos_offset,
                             const int32_t* g_override, int32_t K_override,
                             int32_t n_prefix, const uint8_t* prefix_visible,
                             int32_t* dfs_order, int32_t* node_start, int32_t* node_end,
                             int32_t* subtree_end, int32_t* node_parent, int32_t* node_g,
                             int32_t* tok_node, int32_t* tok_pos, int32_t* tok_pred,
                             float* tok_weight,
                             int32_t* kend, int32_t* ktile_kend_min, int32_t* ktile_kend_max);

/* ------------------------------------------------------------------------------------------
 * tt_tree_path_weights  (host only; needs no GPU)
 *
 * General per-token loss weights ("Derivation", last paragraph): with a weight w_k per
 * root-to-leaf path, lambda_t = sum of w_k over the paths through t; the loss is then the single
 * weighted sum over unique tokens that tt_tree_weighted_logprob computes.  tt_tree_build_meta's
 * tok_weight is the special case w_k = 1/K.
 *   scheme TT_WEIGHT_PATH_SUM         w_k = path_weight[k]; paths are numbered by the DFS order of
 *                                     their leaves (leaf_node[k] gives the leaf's input id)
 *          TT_WEIGHT_UNIFORM          lambda_t = 1 for every unique token
 *          TT_WEIGHT_PATH_TOKEN_MEAN  w_k = 1 / (K * trained tokens on path k): each branch's loss
 *                                     is its token mean, branches averaged; a branch without
 *                                     trained tokens has w_k = 0
 *   trained[n_nodes] or NULL (all trained): tokens of untrained nodes get weight 0.
 *   advantage[n_tokens] or NULL: per-token advantage in DFS order (policy-gradient objective,
 *                                l_t = -A_t log p), multiplied in as an fp32 product.
 * Outputs (host): tok_weight[n_tokens] fp32 in DFS order; leaf_node[n_leaves] or NULL.
 * Arithmetic: path sums in fp64, one rounding to fp32.
 * Errors: TT_ERR_NULL, TT_ERR_SHAPE, TT_ERR_TREE, TT_ERR_UNSUPPORTED (unknown scheme).
 * ------------------------------------------------------------------------------------------ */
#define TT_WEIGHT_PATH_SUM        0
#define TT_WEIGHT_UNIFORM         1
#define TT_WEIGHT_PATH_TOKEN_MEAN 2
tt_status tt_tree_path_weights(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                               const uint8_t* trained, int32_t scheme, const float* path_weight,
                               const float* advantage, float* tok_weight, int32_t* leaf_node);

/* ------------------------------------------------------------------------------------------
 * Tree attention (device).
 *
 * Forward, per query head:  S_ij = scale * <Q_i, K_j> on visible pairs, P = row softmax(S) in
 * fp32, O = P V, LSE_i = ln sum_j exp(S_ij).  Every query sees at least itself, so no row is
 * empty.  With this mask each token's output equals what plain causal attention over its own
 * root-to-leaf sequence gives (forward equivalence, Eq. 6).
 *
 * Backward:  D_i = <dO_i, O_i>, dP = dO V^T, dS = P o (dP - D), dQ = scale dS K,
 * dK = scale dS^T Q, dV = P^T dO; dK/dV are summed over the query heads of the group and over
 * every visible query, i.e. over all branches that pass through the key (Eq. 5).  Gradients for
 * cached prefix keys are ADDED in fp32 to dk_prefix_acc / dv_prefix_acc so that several child
 * partitions can accumulate into one buffer without bf16 rounding between them (Appendix
 * "Float32 Gradient Accumulation").
 *
 * dtype TT_DTYPE_BF16: bf16 tensors, bf16 MFMA with fp32 accumulation and fp32 softmax; d = 128.
 * dtype TT_DTYPE_FP32: fp32 tensors and arithmetic, any d <= 256 (slow reference-grade path).
 * Alignment: device pointers 16-byte aligned; token strides multiples of 8 elements.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t n_q;            /* own tokens N (queries; also the own keys)                     */
  int32_t n_prefix;       /* cached prefix keys P (0 = none)                               */
  int32_t hq, hkv, d;     /* query heads, key/value heads (hq % hkv == 0), head dim        */
  int32_t dtype;          /* TT_DTYPE_*: type of q, k, v, o, d_o, dq, dk, dv               */
  float   scale;          /* softmax scale, e.g. 1/sqrt(d)                                 */
  int32_t flags;          /* 0 or TT_FLAG_*                                                */
  int64_t q_stride_tok;   /* elements between consecutive tokens of q; 0 = hq*d            */
  int64_t k_stride_tok;   /* same for k_own; 0 = hkv*d                                     */
  int64_t v_stride_tok;   /* same for v_own; 0 = hkv*d                                     */
} tt_attn_desc;

/* Bytes of device workspace the forward (backward = 0) or backward (backward = 1) call needs;
 * 0 if the descriptor is invalid. */
size_t tt_tree_attn_workspace(const tt_attn_desc* desc, int32_t backward);

/* q [n_q][hq][d] (token stride q_stride_tok); k_own, v_own [n_q][hkv][d]; k_prefix, v_prefix
 * [n_prefix][hkv][d] contiguous, NULL iff n_prefix == 0; kend [n_prefix+n_q], kt_min, kt_max
 * [n_ktiles] int32 as written by tt_tree_build_meta (device copies).
 * Outputs: o [n_q][hq][d] contiguous, lse [hq][n_q] fp32 (natural log). */
tt_status tt_tree_attn_fwd(const tt_attn_desc* desc,
                           const void* q, const void* k_own, const void* v_own,
                           const void* k_prefix, const void* v_prefix,
                           const int32_t* kend, const int32_t* kt_min, const int32_t* kt_max,
                           void* o, float* lse,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Inputs as for the forward plus o, d_o [n_q][hq][d] contiguous and lse from the forward.
 * Outputs: dq [n_q][hq][d], dk_own, dv_own [n_q][hkv][d], contiguous, overwritten.
 * dk_prefix_acc, dv_prefix_acc [n_prefix][hkv][d] fp32, accumulated (+=); NULL iff n_prefix == 0.
 * Keys of the prefix with kend == 0 receive nothing. */
tt_status tt_tree_attn_bwd(const tt_attn_desc* desc,
                           const void* q, const void* k_own, const void* v_own,
                           const void* k_prefix, const void* v_prefix,
                           const int32_t* kend, const int32_t* kt_min, const int32_t* kt_max,
                           const void* o, const void* d_o, const float* lse,
                           void* dq, void* dk_own, void* dv_own,
                           float* dk_prefix_acc, float* dv_prefix_acc,
                           void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Tree partitioning (host planner + device driver)
 *
 * A tree that does not fit in one pass is cut into partitions (Section "Redundancy-Free Tree
 * Partitioning"): each a connected subtree, cut at node boundaries, at most `capacity` tokens,
 * every partition with one parent partition.  Each token is still computed once: a partition
 * attends to a cached slice of its parent partition's keys/values (Appendix "Zero-Overhead
 * Partition Boundaries"), gradients for those cached keys flow back in fp32.
 *
 * tt_tree_partition_plan (host only; needs no GPU)
 *   Packing rule (a deterministic greedy stand-in for the paper's bin-packing solver, which this
 *   library does not contain): partitions are opened in first-in-first-out order of their root
 *   nodes, the tree's roots first in ascending id.  A partition takes its root, then walks
 *   depth-first with children in ascending id; a child joins if the partition's running token
 *   count plus the child's own length is <= capacity, otherwise the edge is cut and the child is
 *   queued as a later partition's root.  A node longer than `capacity` forms a partition alone.
 *   Boundary bookkeeping for partition p whose root's parent node n_c lies in partition P:
 *     cached slice  = P's cached slice, then P's own tokens (P's DFS order) up to the end of n_c;
 *     visible flags = P's flags carried over, then 1 on the nodes of the path P.root .. n_c and
 *                     0 on everything else (Appendix "Ancestor-Aware Attention Bias");
 *     pos_offset    = pos_offset(P) + depth-based position of n_c's first token in P + |n_c|
 *                     (Appendix "Depth-Based Position Offset").
 *   Token indices are positions in the WHOLE tree's DFS serialisation (the order
 *   tt_tree_build_meta gives for the same parent / seg_len).
 * Outputs (host, caller-allocated, sizes from tt_tree_partition_sizes; any may be NULL):
 *   part_of_node[n_nodes]       partition of each node (input numbering)
 *   part_node_off[n_parts+1], part_nodes[n_nodes]   node ids per partition, in its DFS order
 *   part_parent[n_parts]        parent partition, -1 for a partition rooted at a tree root
 *   part_cut_node[n_parts]      n_c (input id), -1
 *   part_pos_offset[n_parts]
 *   part_tok_off[n_parts+1], own_tok[n_tokens]      own tokens per partition, its DFS order
 *   part_own_start[n_parts]     first own token if the partition's own tokens are one ascending run
 *                               of whole-tree indices (then no gather is needed), else -1
 *   part_prefix_start[n_parts]  the same for the cached slice (-1 also for an empty slice)
 *   part_prefix_off[n_parts+1], prefix_tok[sum_prefix], prefix_visible[sum_prefix]
 *   kend[sum_prefix + n_tokens] partition p's bounds on its [slice ; own] key axis start at
 *                               part_prefix_off[p] + part_tok_off[p]; same meaning as the kend of
 *                               tt_tree_build_meta called on the partition
 *   part_ktile_off[n_parts+1], kt_min, kt_max [sum_ktiles]   tile summaries per partition
 * Partitions are numbered parents first.
 * Errors: TT_ERR_NULL, TT_ERR_SHAPE (capacity < 1, negative sizes, overflow), TT_ERR_TREE.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t n_parts;
  int32_t n_tokens;         /* whole tree                                         */
  int32_t max_part_tokens;  /* most own tokens in one partition                   */
  int32_t max_prefix;       /* longest cached slice                               */
  int64_t sum_prefix;       /* entries of prefix_tok / prefix_visible             */
  int64_t sum_ktiles;       /* entries of kt_min / kt_max                         */
} tt_partition_sizes;

tt_status tt_tree_partition_sizes(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                                  int32_t capacity, tt_partition_sizes* out);

tt_status tt_tree_partition_plan(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                                 int32_t capacity,
                                 int32_t* part_of_node, int32_t* part_node_off, int32_t* part_nodes,
                                 int32_t* part_parent, int32_t* part_cut_node, int32_t* part_pos_offset,
                                 int32_t* part_tok_off, int32_t* own_tok,
                                 int64_t* part_prefix_off, int32_t* prefix_tok, uint8_t* prefix_visible,
                                 int32_t* kend, int64_t* part_ktile_off, int32_t* kt_min, int32_t* kt_max,
                                 int32_t* part_own_start, int32_t* part_prefix_start);

/* Partitioned tree attention (device): the whole tree in one call, one attention pass per
 * partition.  Tensors are whole-tree tensors in whole-tree DFS order, exactly as for
 * tt_tree_attn_fwd / tt_tree_attn_bwd with n_prefix = 0 (desc->n_q = plan->n_tokens,
 * desc->n_prefix = 0), and the results equal those calls' results up to floating-point summation
 * order.  Per partition the driver gathers the partition's rows and its cached slice, runs the
 * attention kernels with the plan's bounds, and scatters the results back; where the plan marks
 * the rows as one contiguous run (part_own_start / part_prefix_start) the kernels read and write
 * the whole-tree tensors in place instead.  The backward visits
 * partitions children first (Appendix "Backward Pass"), adds every partition's cached-key
 * gradients into whole-tree fp32 accumulators (Appendix "Float32 Gradient Accumulation") and
 * rounds dk / dv once at the end: dk = own-partition dk + accumulated cached-key gradients.
 *   plan: the offset tables and run starts are HOST arrays, the five index / bound arrays are DEVICE
 *   copies of the planner's outputs of the same names.
 * Errors: as the attention calls; TT_ERR_SHAPE if the plan's sizes disagree with desc. */
typedef struct {
  int32_t n_parts;
  int32_t n_tokens;
  const int32_t* part_tok_off;      /* host   [n_parts+1] */
  const int64_t* part_prefix_off;   /* host   [n_parts+1] */
  const int64_t* part_ktile_off;    /* host   [n_parts+1] */
  const int32_t* part_own_start;    /* host   [n_parts], or NULL = always gather */
  const int32_t* part_prefix_start; /* host   [n_parts], or NULL = always gather */
  const int32_t* own_tok;           /* device [n_tokens]  */
  const int32_t* prefix_tok;        /* device [sum_prefix] */
  const int32_t* kend;              /* device [sum_prefix + n_tokens] */
  const int32_t* kt_min;            /* device [sum_ktiles] */
  const int32_t* kt_max;            /* device [sum_ktiles] */
} tt_partition_plan;

/* Bytes of device workspace; 0 if desc or plan is invalid. */
size_t tt_tree_attn_partitioned_workspace(const tt_attn_desc* desc, const tt_partition_plan* plan,
                                          int32_t backward);

tt_status tt_tree_attn_partitioned_fwd(const tt_attn_desc* desc, const tt_partition_plan* plan,
                                       const void* q, const void* k, const void* v,
                                       void* o, float* lse,
                                       void* workspace, size_t workspace_bytes, void* stream);

tt_status tt_tree_attn_partitioned_bwd(const tt_attn_desc* desc, const tt_partition_plan* plan,
                                       const void* q, const void* k, const void* v,
                                       const void* o, const void* d_o, const float* lse,
                                       void* dq, void* dk, void* dv,
                                       void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * tt_tree_weighted_logprob (device)
 *
 * Per row r of the logits: lse_r = ln sum_v exp(z_rv), logp_r = z_r[target_r] - lse_r, and the
 * tree loss of Eq. 4, loss += sum_r weight_r * (-logp_r), where weight_r = g/K of the target
 * token (times an advantage for policy-gradient objectives, "Derivation" section).  The logits
 * are read from memory once.
 *   logits [n_rows][vocab], row stride `row_stride` elements (0 = vocab), dtype bf16 or fp32.
 *   target [n_rows] int32; a row whose target is negative or >= vocab is ignored: logp = 0, nothing
 *     is added to the loss (lse is still written).  The targets live in device memory, so they are
 *     not validated on the host; this rule is what the kernels do with an out-of-range value.
 *   weight [n_rows] fp32 or NULL (= 1).
 *   logp   [n_rows] fp32, required (also the staging for the deterministic reduction).
 *   lse    [n_rows] fp32 or NULL.
 *   loss_acc: one fp32, ADDED to (so that a long sequence can be processed in row chunks);
 *     NULL skips the reduction.  The caller zeroes it before the first chunk.
 * Alignment: logits aligned to its element size; rows that start on a 16-byte boundary (e.g. a
 *   16-byte aligned base and row_stride * sizeof(element) a multiple of 16) take the all-vector
 *   path, other rows peel a scalar head and tail.
 * ------------------------------------------------------------------------------------------ */
tt_status tt_tree_weighted_logprob(int64_t n_rows, int32_t vocab, int32_t dtype,
                                   const void* logits, int64_t row_stride,
                                   const int32_t* target, const float* weight,
                                   float* logp, float* lse, float* loss_acc, void* stream);

/* ------------------------------------------------------------------------------------------
 * tt_tree_weighted_logprob_bwd (device)
 *
 * Gradient of grad_scale * sum_r weight_r * (-logp_r) (Eq. 4 through l_t = -log softmax) with
 * respect to the logits:
 *   dlogits[r][v] = grad_scale * weight_r * (exp(z_rv - lse_r) - [v == target_r]),
 * exactly zero for ignored rows (target negative or >= vocab, the same rule as the forward;
 * lse[r] of such a row is not read).  One read of the logits, one write of the gradient.
 *   logits, target, weight as for tt_tree_weighted_logprob; lse [n_rows] fp32 from that call
 *   (required).  dlogits [n_rows][vocab], row stride `dlogits_row_stride` elements (0 = vocab),
 *   same dtype as the logits (bf16: round to nearest even); it may alias logits when the two
 *   strides are equal (every element is read before it is written, by the same thread).
 * Alignment: both arrays aligned to the element size; rows of which both the logits and the
 *   gradient start on a 16-byte boundary take the vector path, other rows a scalar path.
 * ------------------------------------------------------------------------------------------ */
tt_status tt_tree_weighted_logprob_bwd(int64_t n_rows, int32_t vocab, int32_t dtype,
                                       const void* logits, int64_t row_stride,
                                       const int32_t* target, const float* weight, const float* lse,
                                       float grad_scale, void* dlogits, int64_t dlogits_row_stride,
                                       void* stream);

/* ------------------------------------------------------------------------------------------
 * tt_tree_weighted_logprob_fwd_bwd (device)
 *
 * tt_tree_weighted_logprob and tt_tree_weighted_logprob_bwd in one pass, for the training step
 * that wants the loss of Eq. 4 and its gradient together: the logits are read from memory once
 * (a row stays on chip between the log-softmax statistics and the gradient; of a row longer than
 * 64 KB the rest is read a second time right behind the first).  Same results as the two calls
 * (the row sums are added in a different order: lse and logp agree to rounding).
 *   Arguments as for the two calls; logp and lse [n_rows] fp32 are both required; loss_acc may be
 *   NULL; grad_scale must be known beforehand (it usually is: 1, or 1 / accumulation steps).
 *   dlogits may alias logits when the strides are equal.
 * Alignment: when the logits' and the gradient's rows all start on 16-byte boundaries (aligned
 *   bases, row strides a multiple of 16 bytes) the one-pass kernel runs; otherwise the call runs
 *   the two passes one after the other.
 * ------------------------------------------------------------------------------------------ */
tt_status tt_tree_weighted_logprob_fwd_bwd(int64_t n_rows, int32_t vocab, int32_t dtype,
                                           const void* logits, int64_t row_stride,
                                           const int32_t* target, const float* weight, float grad_scale,
                                           float* logp, float* lse, float* loss_acc,
                                           void* dlogits, int64_t dlogits_row_stride, void* stream);

/* ------------------------------------------------------------------------------------------
 * tt_tree_rope (device)
 *
 * Rotary position embedding of a [n_tokens][n_heads][d] tensor (Q or K) with the tree position ids
 * tok_pos of tt_tree_build_meta (Eq. 9).  Rotate-half convention: for i in [0, d/2)
 *   angle = tok_pos[t] * theta_base^(-2i/d)
 *   y[i]       = x[i] cos(angle) - x[i + d/2] sin(angle)
 *   y[i + d/2] = x[i + d/2] cos(angle) + x[i] sin(angle)
 * inverse != 0 rotates by -angle (undoes the rotation; also the backward pass: feed dY, get dX).
 *   x, y: dtype bf16 or fp32, token strides in elements (0 = n_heads * d), heads and d contiguous;
 *   y may be x (in place) when the strides are equal.  tok_pos [n_tokens] int32, non-negative.
 *   d must be a multiple of 16 (bf16) / 8 (fp32), at most 1024; x, y 16-byte aligned, token strides a multiple of
 *   8 (bf16) / 4 (fp32) elements; n_heads * d <= 65536.
 * ------------------------------------------------------------------------------------------ */
tt_status tt_tree_rope(int64_t n_tokens, int32_t n_heads, int32_t d, int32_t dtype,
                       const void* x, int64_t x_stride_tok, const int32_t* tok_pos,
                       float theta_base, int32_t inverse, void* y, int64_t y_stride_tok, void* stream);

/* ------------------------------------------------------------------------------------------
 * Tree-correct causal convolution (device; host helper for the backward)
 *
 * The depthwise causal conv1d in front of an SSM (GDN) layer, Section "Implementation", paragraph
 * "SSM Layers (GDN)" (ii) and Appendix "Tree-Correct Causal Convolution": every token's window
 * holds the K-1 tokens that precede it on its own root-to-token sequence (not the K-1 tokens
 * before it in DFS order), zero before the start of a branch:
 *     y[t][c] = act( bias[c] + sum_{m=0..K-1} weight[c][K-1-m] * x[pred^m(t)][c] )
 * with pred = tok_pred of tt_tree_build_meta (pred^0(t) = t).  This equals the paper's
 * node-by-node procedure (parent's saved context prepended to each chunk) and a plain causal
 * conv1d run on every branch separately.
 *   x, y, dy, dx [n_tokens][channels], dtype bf16 or fp32, token strides in elements (0 = channels);
 *   weight [channels][K] fp32 (weight[c][K-1] multiplies the token itself), bias [channels] fp32
 *   or NULL; K in {2, 3, 4}; activation 0 = none, 1 = SiLU; channels a multiple of 8 (bf16) / 4.
 * Backward: dx (same dtype as x), dweight [channels][K] and dbias [channels] (fp32, overwritten;
 *   dbias may be NULL).  Successors of a token that do not directly follow it in DFS order (the
 *   second and later children of a branch point) are found through a small host-built list:
 *   tt_tree_conv_plan lists every token that has such successors (fix_tok, ascending), and for
 *   each, in CSR form (fix_off), the first token of every such run (fix_t) with its distance
 *   (fix_r, 1..K-1).  The device call takes device copies of the four arrays.
 *   Sums over tokens are taken in a fixed order: results are bit-reproducible.
 * Errors: TT_ERR_NULL, TT_ERR_SHAPE, TT_ERR_DTYPE, TT_ERR_ALIGN (16-byte pointers, strides a
 *   multiple of 8 / 4 elements), TT_ERR_UNSUPPORTED (K outside 2..4), TT_ERR_WORKSPACE.
 * ------------------------------------------------------------------------------------------ */
tt_status tt_tree_conv_fwd(int64_t n_tokens, int32_t channels, int32_t kernel_size, int32_t dtype,
                           int32_t activation, const void* x, int64_t x_stride_tok,
                           const float* weight, const float* bias, const int32_t* tok_pred,
                           void* y, int64_t y_stride_tok, void* stream);

/* Host: sizes, then contents, of the backward's successor list for kernel size K. */
tt_status tt_tree_conv_plan_sizes(int64_t n_tokens, const int32_t* tok_pred, int32_t kernel_size,
                                  int32_t* n_fix, int32_t* n_pairs);
tt_status tt_tree_conv_plan(int64_t n_tokens, const int32_t* tok_pred, int32_t kernel_size,
                            int32_t* fix_tok /* [n_fix] */, int32_t* fix_off /* [n_fix+1] */,
                            int32_t* fix_t /* [n_pairs] */, int32_t* fix_r /* [n_pairs] */);

size_t tt_tree_conv_bwd_workspace(int64_t n_tokens, int32_t channels, int32_t kernel_size, int32_t dtype);

tt_status tt_tree_conv_bwd(int64_t n_tokens, int32_t channels, int32_t kernel_size, int32_t dtype,
                           int32_t activation, const void* x, int64_t x_stride_tok,
                           const float* weight, const float* bias, const int32_t* tok_pred,
                           const void* dy, int64_t dy_stride_tok,
                           int32_t n_fix, const int32_t* fix_tok, const int32_t* fix_off,
                           const int32_t* fix_t, const int32_t* fix_r,
                           void* dx, int64_t dx_stride_tok, float* dweight, float* dbias,
                           void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * tt_tree_conv_bwd_static (device) -- tt_tree_conv_bwd for callers that cannot allocate
 *
 * For code that runs where device memory may not be allocated and no workspace can be brought in:
 * under HIP graph capture, in tight serving / training loops, in harnesses that forbid allocation.
 * Same arguments, same kernels and bit-identical results as tt_tree_conv_bwd, minus the workspace:
 * the per-tile partial sums of dweight / dbias go to an array of
 * TT_CONV_BWD_STATIC_SCRATCH_BYTES bytes that is part of the library's device code (every GPU the
 * library runs on holds one copy from the first use of the library on it until the process ends).
 * The call allocates and frees nothing.
 *   Limit: tt_tree_conv_bwd_workspace(n_tokens, channels, kernel_size, dtype) must not exceed
 *   TT_CONV_BWD_STATIC_SCRATCH_BYTES (e.g. 16 406 tokens x 8192 channels, K = 4, bf16 needs 42 MB);
 *   a larger shape is refused with TT_ERR_WORKSPACE before anything is launched.
 *   The scratch needs no clearing: every call overwrites the part it reads (one row per token tile).
 *   All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different
 *   streams, or threads) race on it and must be ordered by the caller; calls on one stream are safe.
 * Errors: as tt_tree_conv_bwd; TT_ERR_HIP if the array's device address cannot be obtained.
 * ------------------------------------------------------------------------------------------ */
#define TT_CONV_BWD_STATIC_SCRATCH_BYTES (64u << 20)
tt_status tt_tree_conv_bwd_static(int64_t n_tokens, int32_t channels, int32_t kernel_size, int32_t dtype,
                                  int32_t activation, const void* x, int64_t x_stride_tok,
                                  const float* weight, const float* bias, const int32_t* tok_pred,
                                  const void* dy, int64_t dy_stride_tok,
                                  int32_t n_fix, const int32_t* fix_tok, const int32_t* fix_off,
                                  const int32_t* fix_t, const int32_t* fix_r,
                                  void* dx, int64_t dx_stride_tok, float* dweight, float* dbias,
                                  void* stream);

/* ------------------------------------------------------------------------------------------
 * Gated delta rule with tree state routing, forward (device; host plan)
 *
 * The recurrent core of a GDN layer, Section "Implementation", paragraph "SSM Layers (GDN)" (i)
 * and Appendix "Tree-Aware SSM State Routing".  Per value head (key head = value head /
 * (hv / hk)), state S in R^{dk x dv}; token t with predecessor p = tok_pred[t] on its own
 * root-to-token sequence (S_p = 0 at the start of a branch):
 *     S~ = exp(g_t) S_p;   S_t = S~ + beta_t k_t (v_t - S~^T k_t)^T;   o_t = scale S_t^T q_t
 * i.e. a node's first token continues from the end state of its PARENT node, not from the
 * previous node in DFS order.  Computed in chunks of TT_GDN_CHUNK tokens that never cross a node
 * boundary (bf16 MFMA, fp32 accumulation, fp32 state).
 * tt_tree_gdn_plan (host): the chunk list in DFS order and, per chunk, where its entering state
 *   comes from and whether its leaving state must be kept:
 *     chunk_tok0, chunk_len [n_chunks]   first token (DFS index) and length (1..TT_GDN_CHUNK)
 *     chunk_src [n_chunks]   -2 = continues the previous chunk's sequence (state stays on chip),
 *                            -1 = zero state, >= 0 = saved state slot
 *     chunk_dst [n_chunks]   -1, or the slot the chunk's leaving state is saved to (nodes that
 *                            have two or more token-bearing child branches; EVERY such branch
 *                            starts from the slot, the one that follows directly included, so
 *                            that the branches are independent of each other)
 *     chunk_cap [n_chunks]   -1, or i when the chunk's leaving state is the end state of
 *                            capture_node[i]: the state a child partition starts from (Appendix
 *                            "SSM State Gateway": state extraction / injection).  A zero-length
 *                            capture node stands for its nearest token-bearing ancestor; two
 *                            capture nodes may not share a chunk.
 *   Zero-length nodes have no chunk; their children continue from the nearest token-bearing
 *   ancestor.
 * tt_tree_gdn_schedule (host): which parts of the chunk program may run side by side.  A segment
 *   is a maximal run of chunks whose state stays on chip (all but its first chunk have src = -2);
 *   it depends only on the segment that saved the slot its first chunk loads.  Level 0 holds the
 *   segments that start from the initial state, level l + 1 those whose slot a level-l segment
 *   saves: sibling subtrees land in one level and are walked by different workgroups at the same
 *   time, one launch per level.  Outputs, segments in level order (inside a level the longest
 *   first, ties in chunk order):
 *     seg_chunk0, seg_chunk1 [n_segments]  first chunk and one past the last chunk
 *     level_off [n_levels + 1]             segments of level l: level_off[l] .. level_off[l+1]-1
 *     slot_cons_off [n_slots + 1], slot_cons [n_consumers]   per slot, the segments that start
 *                                          from it, in chunk order (the backward sums their
 *                                          gradients in this order)
 *   The device calls take the schedule as tt_gdn_schedule (level_off stays a host array, the
 *   others are device copies); NULL = one set of workgroups walks all chunks in sequence order.
 * tt_tree_gdn_fwd (device): q, k [n_tokens][hk][128], v, o [n_tokens][hv][128] bf16 contiguous;
 *   g, beta [n_tokens][hv] fp32 (g <= 0: log of the decay); the chunk arrays are device
 *   copies of the plan (chunk_cap may be NULL = nothing captured).  initial_state [hv][128][128]
 *   fp32 or NULL (= 0): the state every root starts from (a partition's gateway state);
 *   state_out [n_capture][hv][128][128] fp32: end states of the capture nodes (NULL iff
 *   chunk_cap is NULL).  dk = dv = 128, hv a multiple of hk.  q and k are used as given
 *   (normalise them beforehand if the layer does).
 * Errors: TT_ERR_NULL, TT_ERR_SHAPE, TT_ERR_TREE, TT_ERR_ALIGN, TT_ERR_UNSUPPORTED (dims other
 *   than 128), TT_ERR_WORKSPACE.
 * ------------------------------------------------------------------------------------------ */
#define TT_GDN_CHUNK 64
typedef struct {
  int32_t n_segments, n_levels;
  const int32_t* level_off;       /* HOST   [n_levels + 1]                    */
  const int32_t* seg_chunk0;      /* device [n_segments]                      */
  const int32_t* seg_chunk1;      /* device [n_segments]                      */
  const int32_t* slot_cons_off;   /* device [n_slots + 1]   (backward only)   */
  const int32_t* slot_cons;       /* device [n_consumers]   (backward only)   */
} tt_gdn_schedule;
tt_status tt_tree_gdn_schedule_sizes(int32_t n_chunks, const int32_t* chunk_src, const int32_t* chunk_dst,
                                     int32_t n_slots, int32_t* n_segments, int32_t* n_levels,
                                     int32_t* n_consumers);
tt_status tt_tree_gdn_schedule(int32_t n_chunks, const int32_t* chunk_src, const int32_t* chunk_dst,
                               int32_t n_slots, int32_t* seg_chunk0, int32_t* seg_chunk1,
                               int32_t* level_off, int32_t* slot_cons_off, int32_t* slot_cons);
tt_status tt_tree_gdn_plan_sizes(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                                 int32_t* n_chunks, int32_t* n_slots);
tt_status tt_tree_gdn_plan(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                           int32_t n_capture, const int32_t* capture_node,
                           int32_t* chunk_tok0, int32_t* chunk_len, int32_t* chunk_src, int32_t* chunk_dst,
                           int32_t* chunk_cap);
size_t tt_tree_gdn_workspace(int32_t n_chunks, int32_t n_slots, int32_t hv);
tt_status tt_tree_gdn_fwd(int64_t n_tokens, int32_t hk, int32_t hv, int32_t dk, int32_t dv, float scale,
                          const void* q, const void* k, const void* v, const float* g, const float* beta,
                          int32_t n_chunks, const int32_t* chunk_tok0, const int32_t* chunk_len,
                          const int32_t* chunk_src, const int32_t* chunk_dst, int32_t n_slots,
                          const int32_t* chunk_cap, const tt_gdn_schedule* schedule,
                          const float* initial_state, float* state_out,
                          void* o, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Gated delta rule with tree state routing, backward (device)
 *
 * Vector-Jacobian product of tt_tree_gdn_fwd (same section and appendix): the recurrence run
 * backwards over the tree.  The gradient of a state that several child branches start from is
 * the sum of what they send back -- the gradient accumulation at the shared parent state of the
 * paper's "SSM Layers" paragraph -- which the chunk program provides: a chunk that started from a
 * saved-state slot adds the gradient of its entering state to that slot's gradient, and the
 * chunk that saved the slot picks the sum up (reverse DFS order sees every reader first).
 * Inputs as for the forward, plus d_o [n_tokens][hv][128] bf16.  The call recomputes the
 * per-chunk states itself (it does not need a preceding forward call or its workspace).
 * Outputs: dq, dk [n_tokens][hk][128] bf16 (summed over the hv / hk value heads of a key head in
 * fp32, then rounded once), dv [n_tokens][hv][128] bf16, dg, dbeta [n_tokens][hv] fp32.
 * Gateway (Appendix "SSM State Gateway"), all optional (NULL): initial_state as in the forward;
 * d_state_out [n_capture][hv][128][128] fp32, the upstream gradient of the captured end states
 * (what the child partitions' d_initial_state returned; needs chunk_cap);
 * d_initial_state [hv][128][128] fp32, overwritten with the gradient of the state the roots
 * start from.  Arithmetic: matrix products use bf16 operands with fp32 accumulation, like the
 * forward (state and state gradient stay fp32); the triangular solves and all element-wise work
 * are fp32.
 * Workspace, 16-byte aligned: tt_tree_gdn_bwd_workspace bytes let all heads run in one pass (about
 * 300 KB per chunk and value head, plus two fp32 [n_tokens][hv][128] arrays, 2 x n_slots saved
 * states per head and, with a schedule, one state gradient per segment and head; n_segments = 0
 * when the call gets no schedule).  The heads are independent up to the sum over the value heads
 * of a key head, so any size from tt_tree_gdn_bwd_workspace_min (one key head with its value heads
 * per pass) upwards is accepted: the call then runs in passes of as many key heads as fit -- less
 * memory for more launches and walks that fill less of the chip; results do not depend on it.
 * With a schedule the reverse walk also runs level by level (last level first): every segment
 * stores the gradient of the state it started from, and the chunk that saved a slot adds the
 * gradients of the slot's readers in the order of slot_cons -- a fixed order, no atomics.
 * Errors: as tt_tree_gdn_fwd.
 * ------------------------------------------------------------------------------------------ */
size_t tt_tree_gdn_bwd_workspace(int64_t n_tokens, int32_t n_chunks, int32_t n_slots, int32_t n_segments,
                                 int32_t hk, int32_t hv);
size_t tt_tree_gdn_bwd_workspace_min(int64_t n_tokens, int32_t n_chunks, int32_t n_slots, int32_t n_segments,
                                     int32_t hk, int32_t hv);
tt_status tt_tree_gdn_bwd(int64_t n_tokens, int32_t hk, int32_t hv, int32_t dk, int32_t dv, float scale,
                          const void* q, const void* k, const void* v, const float* g, const float* beta,
                          const void* d_o,
                          int32_t n_chunks, const int32_t* chunk_tok0, const int32_t* chunk_len,
                          const int32_t* chunk_src, const int32_t* chunk_dst, int32_t n_slots,
                          const int32_t* chunk_cap, const tt_gdn_schedule* schedule,
                          const float* initial_state, const float* d_state_out,
                          void* dq, void* dk_out, void* dv_out, float* dg, float* dbeta, float* d_initial_state,
                          void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Per-kernel timing (measurement aid; off by default).  When enabled, every kernel the library
 * launches is bracketed by HIP events on the launch stream.  tt_kernel_timing_read blocks until
 * the recorded events have completed and returns the totals since the last enable.
 * ------------------------------------------------------------------------------------------ */
#define TT_KERNEL_ATTN_FWD    0   /* bf16 MFMA forward                                   */
#define TT_KERNEL_LOSS_FUSED  1   /* loss forward + gradient in one pass over the logits  */
#define TT_KERNEL_ATTN_DKDV   2   /* bf16 MFMA dK/dV                                     */
#define TT_KERNEL_ATTN_DQ     3   /* bf16 MFMA dQ                                        */
#define TT_KERNEL_LOSS_ROWS   4   /* log-softmax + gather, one pass over the logits      */
#define TT_KERNEL_LOSS_SUM    5   /* weighted sum over rows                              */
#define TT_KERNEL_REF_FWD     6   /* fp32-arithmetic kernels                             */
#define TT_KERNEL_REF_BWD     7
#define TT_KERNEL_ATTN_PLAN   8   /* work decomposition of the dK/dV pass                */
#define TT_KERNEL_ATTN_REDUCE 9   /* sum of dK/dV partials of key tiles that were cut    */
#define TT_KERNEL_LOSS_BWD    10  /* gradient of the loss with respect to the logits     */
#define TT_KERNEL_ROPE        11  /* rotary position embedding                           */
#define TT_KERNEL_PART_GATHER  12  /* partition driver: row gathers                      */
#define TT_KERNEL_PART_SCATTER 13  /* partition driver: row scatters, accumulate, finalise */
#define TT_KERNEL_CONV_FWD     14  /* tree-correct causal convolution                    */
#define TT_KERNEL_CONV_BWD     15
#define TT_KERNEL_CONV_FIX     16  /* its branch-point fix-up and weight-gradient reduce */
#define TT_KERNEL_GDN_PREPARE  17  /* gated delta rule: per-chunk operands (parallel)     */
#define TT_KERNEL_GDN_SCAN     18  /* gated delta rule: state scan over the tree          */
#define TT_KERNEL_GDN_BWD_FSCAN  19  /* gated delta rule backward: forward walk that saves the states */
#define TT_KERNEL_GDN_BWD_RSCAN  20  /* reverse walk (state gradients)                              */
#define TT_KERNEL_GDN_BWD_FINISH 21  /* per-chunk gradients                                         */
#define TT_N_KERNELS          22
typedef struct {
  double  ms[TT_N_KERNELS];        /* summed kernel time in milliseconds */
  int64_t launches[TT_N_KERNELS];
} tt_kernel_times;
tt_status tt_kernel_timing_enable(int32_t on);     /* also resets the totals */
tt_status tt_kernel_timing_read(tt_kernel_times* out);

#ifdef __cplusplus
}
#endif
#endif /* TREETRAIN_H */
