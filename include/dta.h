/*
 * dta.h - C ABI of the MI355X (gfx950) dynamic-tree-attention library.
 *
 * The library computes causal softmax attention, forward and backward, over a
 * rollout prefix tree: every unique tree token's query attends to exactly the
 * keys/values on its root-to-node path (whole ancestor segments plus the causal
 * part of its own segment), so a prefix shared by many rollouts is computed
 * once, and the gradient of a shared key/value is the sum over all descendant
 * queries (paper section 3, problem formulation and equation 1; section 3.1,
 * push / leaf / pop steps; pseudocode appendix, FWD and BWD primitives).
 *
 * General rules
 *  - every function returns an int status (DTA_OK = 0, negative = error) unless
 *    stated otherwise; nothing throws, nothing aborts;
 *  - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *    memory of the current device; the caller owns every tensor and workspace,
 *    the library owns only dta_tree_t objects;
 *  - attention calls only enqueue work on the given HIP stream and do not
 *    synchronise it.  The first attention call on a tree (or an explicit
 *    dta_tree_attn_prepare) allocates and uploads the tree's device metadata
 *    (into a block of the library's own pool, by a copy on a stream the library owns; the call
 *    waits for that copy only, never for the caller's streams); later calls
 *    allocate nothing;
 *  - tensors are dense row-major [T, H, head_dim] with T = unique tree tokens in
 *    the packed DFS order defined by dta_tree_build;
 *  - a tree may be used from several host threads (its lazily built schedules are
 *    guarded); every attention call also records an event on its stream, which
 *    is how dta_tree_destroy knows when the device copies are free, so a tree
 *    must outlive any captured graph that replays calls made on it.
 */
#ifndef DTA_H_
#define DTA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dta_tree dta_tree_t; /* opaque */

enum {
  DTA_OK = 0,
  DTA_ERR_INVALID_ARG = -1, /* null pointer, n_nodes < 1, bad struct field         */
  DTA_ERR_BAD_TREE = -2,    /* parent out of range / self parent / cycle / seg_len<1 / > 2^31-1 tokens */
  DTA_ERR_UNSUPPORTED = -3, /* head_dim not in {64,128}, Hq % Hkv != 0, unknown dtype */
  DTA_ERR_ALLOC = -4,       /* host or device allocation failed                     */
  DTA_ERR_HIP = -5,         /* a HIP runtime call or kernel launch failed           */
  DTA_ERR_WORKSPACE = -6    /* workspace null or smaller than required              */
};

enum { DTA_F32 = 0, DTA_BF16 = 1 };

/* Integer facts about a tree (all counts exact, int64). */
typedef struct {
  int64_t n_nodes;
  int64_t n_tokens;            /* T: unique tree tokens = sum of seg_len                       */
  int64_t n_leaves;            /* rollouts: every root-to-leaf path is one sequence            */
  int64_t n_roots;
  int64_t max_path_tokens;     /* longest rollout, in tokens                                   */
  int64_t max_depth_nodes;     /* nodes on the deepest root-to-node path                       */
  int64_t rollout_tokens;      /* sum of leaf path lengths (dense training would process this) */
  int64_t rollout_tokens_full; /* same if every node ended a rollout (figure 1's full tree)    */
  int64_t unique_pairs;        /* sum over tokens of (position+1): (query, visible key) pairs  */
  int64_t dense_pairs;         /* sum over leaves of n(n+1)/2                                  */
  int64_t dense_pairs_full;    /* same with every node ending a rollout                        */
} dta_tree_info_t;

/* Borrowed host pointers into the tree object, valid until dta_tree_destroy.
 * Arrays indexed by node use the caller's node ids. */
typedef struct {
  const int32_t* dfs_order;        /* [n_nodes]   node id at each DFS preorder rank             */
  const int64_t* node_offset;      /* [n_nodes]   first packed token index of the node          */
  const int64_t* node_start_depth; /* [n_nodes]   tokens above the node on its root path        */
  const int64_t* subtree_tokens;   /* [n_nodes]   tokens in the node and all its descendants;   */
                                   /*             they occupy [offset, offset+subtree_tokens)   */
  const int64_t* anc_ptr;          /* [n_nodes+1] CSR pointer into anc_seg_*                    */
  const int64_t* anc_seg_off;      /* ancestor key intervals root->parent (packed token index), */
  const int64_t* anc_seg_len;      /*   adjacent intervals merged when contiguous               */
  const int32_t* token_kend;       /* [T] one past the last packed token that sees this key     */
} dta_tree_layout_t;

/* Tile schedule statistics for one head configuration (integer, host only). */
typedef struct {
  int64_t fwd_q_tile_tokens;   /* query tokens per forward work item                          */
  int64_t fwd_work_items;      /* forward query tiles (per kv head)                           */
  int64_t fwd_tile_pairs;      /* (padded query rows) x (keys streamed), summed over tiles    */
  int64_t bwd_kv_tile_tokens;  /* keys per backward dK/dV work item                           */
  int64_t bwd_work_items;
  int64_t bwd_tile_pairs;      /* (padded key cols) x (query rows streamed)                   */
  int64_t metadata_bytes;      /* what the first attention call copies to the device for this */
                               /* configuration: kend[] and the work lists                    */
} dta_schedule_info_t;

typedef struct {
  int32_t n_q_heads;
  int32_t n_kv_heads;   /* must divide n_q_heads; q head h uses kv head h / (n_q_heads/n_kv_heads) */
  int32_t head_dim;     /* 64 or 128                                                               */
  float softmax_scale;  /* multiplies q.k before the softmax; finite and nonzero, else INVALID_ARG   */
  int32_t dtype;        /* DTA_F32 or DTA_BF16: element type of q,k,v,o,dO,dq,dk,dv                */
} dta_attn_params_t;

/*
 * dta_tree_build - tree metadata from (parent, seg_len); host only, integer only.
 * A node is a token segment; parent[i] = -1 marks a root (several roots = a
 * forest of independent trees); seg_len[i] >= 1 tokens (paper section 3: nodes
 * are token segments, root-to-leaf paths are rollouts; path length is counted
 * in tokens).  Nodes are packed in DFS preorder, roots and children in
 * ascending node id (the paper leaves the DFS order free, section 4), so a
 * subtree is one contiguous token range.
 *   parent, seg_len : host, [n_nodes], read only during the call.
 *   flags           : must be 0.
 *   out             : receives a new tree; free it with dta_tree_destroy.
 * Errors: INVALID_ARG (null, n_nodes < 1, flags != 0), BAD_TREE, ALLOC.
 */
int dta_tree_build(const int32_t* parent, const int32_t* seg_len, int32_t n_nodes,
                   uint32_t flags, dta_tree_t** out);

/* Counts for reporting: C = rollout_tokens / n_tokens is the compression rate
 * of the paper's figure 1, S = 1 - 1/C its prefix-sharing rate. */
int dta_tree_info(const dta_tree_t* tree, dta_tree_info_t* out);

/*
 * dta_tree_layout - where every node's tokens sit in the packed tensors, and which
 * key intervals its queries see: the tree of token segments of the paper's
 * problem formulation (section 3) laid out in one DFS order (any DFS order of the
 * tree is valid, section 4).  A token of node u at in-node index j is row
 * node_offset[u] + j and has position node_start_depth[u] + j on its root path
 * (depth is counted in tokens, section 3.1, space complexity); its queries see
 * the intervals anc_seg_*[anc_ptr[u] .. anc_ptr[u+1]) (the segments of u's
 * ancestors, root first) and rows node_offset[u] .. node_offset[u] + j of u
 * itself.  Host only; the pointers are borrowed and stay valid until
 * dta_tree_destroy.
 */
int dta_tree_layout(const dta_tree_t* tree, dta_tree_layout_t* out);

/* Builds (and caches in the tree) the DFS tile schedule for this head
 * configuration and reports its size.  Host only. */
int dta_tree_schedule_info(dta_tree_t* tree, const dta_attn_params_t* params,
                           dta_schedule_info_t* out);

/* Frees host and device memory of the tree.  NULL is allowed.  Does not block:
 * the device copies are released once the attention calls already enqueued
 * for this tree have finished, so a tree may be destroyed right after its last
 * launch. */
void dta_tree_destroy(dta_tree_t* tree);

/* Bytes of device workspace dta_tree_attn_fwd (is_bwd = 0) or dta_tree_attn_bwd
 * (is_bwd != 0) needs; 0 on invalid arguments.  The workspace must be 256-byte
 * aligned; its contents need not be preserved between calls.  Calls that may
 * overlap in time (different streams) need a workspace each.  The forward's
 * (a few hundred bytes of work-queue counters in bf16 mode, none in fp32 mode)
 * is optional, see dta_tree_attn_fwd. */
size_t dta_tree_attn_workspace_bytes(const dta_tree_t* tree, const dta_attn_params_t* params,
                                     int is_bwd);

/* Optional: allocate and upload the tree's device metadata for this head
 * configuration now (waits for the upload only), so that later attention calls
 * only enqueue. */
int dta_tree_attn_prepare(dta_tree_t* tree, const dta_attn_params_t* params);

/*
 * dta_tree_attn_fwd - forward tree attention (the attention inside the paper's
 * FWD primitive, for every segment of the tree in one pass).
 * For token t, q head h, kv head g = h / (Hq/Hkv), with anc(t) the keys on t's
 * root path up to and including t:
 *   s_k = softmax_scale * q[t,h] . k[k,g]          for k in anc(t)
 *   lse[t,h] = ln sum_k exp(s_k)
 *   o[t,h]   = sum_k exp(s_k - lse[t,h]) * v[k,g]
 *   q : device [T,Hq,d]   k,v : device [T,Hkv,d]   (dtype per params)
 *   o : device [T,Hq,d] out, same dtype (round to nearest even)
 *   lse : device [T,Hq] fp32 out (natural log)
 *   workspace : device, >= dta_tree_attn_workspace_bytes(tree, params, 0) and 256-byte
 *               aligned, or NULL / smaller: then the launch hands one work item to
 *               each block instead of letting resident blocks draw items from
 *               queues, which is a few per cent slower on large inputs and gives
 *               the same bits
 *   hip_stream : a hipStream_t (NULL = default stream)
 * The tree is not const: the first call for a head configuration builds and caches
 * the tile schedule in it and, unless dta_tree_attn_prepare has done so, allocates
 * device memory for the tree's metadata and waits for its upload (see the general
 * rules above); later calls with the same configuration only enqueue.
 * bf16 mode multiplies in bf16 on the matrix cores and accumulates / does the
 * softmax in fp32; fp32 mode is fp32 throughout.
 */
int dta_tree_attn_fwd(dta_tree_t* tree, const dta_attn_params_t* params, const void* q,
                      const void* k, const void* v, void* o, float* lse, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/*
 * dta_tree_attn_bwd - backward tree attention (the attention inside the paper's
 * BWD primitive; gradients of all descendant rollouts are accumulated into a
 * shared key/value, pop step of section 3.1 and equation 1).
 * d_o is the upstream gradient per TREE token, already summed over the rollouts
 * sharing the token.  With p_tk = exp(s_tk - lse_t), D_t = d_o_t . o_t,
 * ds_tk = p_tk (d_o_t . v_k - D_t):
 *   dq[t,h] = scale * sum_{k in anc(t)} ds_tk k_k
 *   dk[k,g] = scale * sum_{h in group g} sum_{t : k in anc(t)} ds_tk q_t
 *   dv[k,g] =         sum_{h in group g} sum_{t : k in anc(t)} p_tk d_o_t
 *   q,k,v,o,d_o : device inputs as in forward; lse : device [T,Hq] fp32 from forward
 *   dq : device [T,Hq,d] out;  dk, dv : device [T,Hkv,d] out.  All three are
 *        OVERWRITTEN (each element written exactly once, no atomics).
 *   workspace : device, >= dta_tree_attn_workspace_bytes(tree, params, 1)
 * As for the forward, the first call for a head configuration may build the
 * schedule and allocate / upload the tree's device metadata.
 */
int dta_tree_attn_bwd(dta_tree_t* tree, const dta_attn_params_t* params, const void* q,
                      const void* k, const void* v, const void* o, const float* lse,
                      const void* d_o, void* dq, void* dk, void* dv, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/*
 * dta_tree_attn_bwd_stages - the same backward pass, restricted to the stages in
 * stage_mask, for callers that need only some gradients or that time the
 * launches one by one.  dta_tree_attn_bwd equals DTA_BWD_ALL.  DTA_BWD_DQ and
 * DTA_BWD_DKDV read what DTA_BWD_DELTA leaves in the workspace (the D values
 * and, in bf16 mode, lse rescaled for the kernels), so the delta stage must have
 * run on the same workspace, o, lse, d_o and softmax_scale before them.  In
 * bf16 mode a call that asks for DTA_BWD_DELTA and DTA_BWD_DQ together computes
 * D inside the dQ launch (no separate pass over o and d_o) and leaves the same
 * values in the workspace; results do not depend on how the stages are grouped.
 * Outputs of stages that are not selected are not touched (and may be NULL).
 */
enum { DTA_BWD_DELTA = 1, DTA_BWD_DQ = 2, DTA_BWD_DKDV = 4, DTA_BWD_ALL = 7 };
int dta_tree_attn_bwd_stages(dta_tree_t* tree, const dta_attn_params_t* params, const void* q,
                             const void* k, const void* v, const void* o, const float* lse,
                             const void* d_o, void* dq, void* dk, void* dv, void* workspace,
                             size_t workspace_bytes, void* hip_stream, uint32_t stage_mask);

/*
 * dta_tree_attn_bwd_noalloc - dta_tree_attn_bwd for callers that cannot allocate
 * device memory: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, results and bits as dta_tree_attn_bwd,
 * without the workspace: the scratch memory (row statistics, work-queue
 * counters, fp32 partial sums of split key tiles) is a device array of 160 MiB
 * that the library holds on every GPU it runs on until the process ends.  The
 * call allocates and frees nothing, on the host side of HIP or on the device:
 *  - the tree's device metadata for this head configuration must already be
 *    resident on the current device (dta_tree_attn_prepare, which may
 *    allocate, also resolves the scratch array's address on that device), else
 *    DTA_ERR_INVALID_ARG;
 *  - DTA_ERR_WORKSPACE, with a message on stderr, when
 *    dta_tree_attn_workspace_bytes(tree, params, 1) exceeds 160 MiB (trees of a
 *    few hundred thousand tokens need 35 to 130 MiB; one whose long shared
 *    prefix is cut into many partial sums, like the 16K-token root of the deep
 *    benchmark tree with its 468 MiB, does not fit);
 *  - every call on a GPU uses that GPU's one array, which keeps the previous
 *    call's contents: nothing in it needs to start from zero except the queue
 *    counters, which the call clears itself with a fill kernel, and calls that
 *    overlap in time on one GPU (two streams, two threads) race on it.  Order
 *    them on one stream or with events.
 */
int dta_tree_attn_bwd_noalloc(dta_tree_t* tree, const dta_attn_params_t* params, const void* q,
                              const void* k, const void* v, const void* o, const float* lse,
                              const void* d_o, void* dq, void* dk, void* dv, void* hip_stream);

/*
 * Segment calls: the attention inside the paper's FWD(l_start -> l_end) and BWD
 * primitives (pseudocode appendix, notation block), which its push / pop
 * traversal issues once per token segment (section 3.1; vanilla algorithm), and
 * once per chunk of a segment in the chunked pops of the optimised algorithm
 * (Pop_ByChunk).
 *
 *   [t_begin, t_end) : packed token rows of the call; non-empty and inside ONE
 *                      node's segment (a whole segment or a chunk of it), else
 *                      DTA_ERR_INVALID_ARG.
 *
 * dta_tree_attn_fwd_segment computes o and lse for these rows only.  The rows'
 * queries see the keys/values on their root path: the segments of the node's
 * ancestors, the node's tokens before the row, and the row itself.  Tensors are
 * the full packed [T, H, head_dim] tensors of dta_tree_attn_fwd (same layout,
 * alignment and ownership); of q, o, lse only the rows are read / written, of
 * k, v only rows on the root path up to t_end are read, so nothing else needs
 * to be valid yet (this is the paper's active stack: only the current path).
 *
 * dta_tree_attn_bwd_segment backpropagates the rows' attached gradient d_o
 * (rows [t_begin, t_end) of the per-tree-token dO): it writes dq for the rows
 * (final: a row's dQ depends on nothing else) and ADDS the rows' contributions
 * to dK and dV of every key they see into dk_acc / dv_acc, fp32
 * [T, n_kv_heads, head_dim] accumulators owned by the caller (zeroed by the
 * caller before the first call; rows of keys the call does not see are not
 * touched).  When all descendants of a key's node and the later rows of its own
 * segment have been popped, the key's accumulated gradient is final: running
 * the calls in the paper's pop order reproduces dta_tree_attn_bwd.  Calls
 * that add into the same accumulators must not overlap (same stream, or
 * ordered by events); within a call every key has one owner, so results are
 * bit-reproducible for a fixed sequence of calls.  o, lse: the forward results
 * of the rows.  workspace: as for dta_tree_attn_bwd (same size).
 */
int dta_tree_attn_fwd_segment(dta_tree_t* tree, const dta_attn_params_t* params, int64_t t_begin,
                              int64_t t_end, const void* q, const void* k, const void* v, void* o,
                              float* lse, void* workspace, size_t workspace_bytes,
                              void* hip_stream);
int dta_tree_attn_bwd_segment(dta_tree_t* tree, const dta_attn_params_t* params, int64_t t_begin,
                              int64_t t_end, const void* q, const void* k, const void* v,
                              const void* o, const float* lse, const void* d_o, void* dq,
                              float* dk_acc, float* dv_acc, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/*
 * Rollout sequences -> prefix tree, and load-balanced partitioning.  Host only,
 * integer only.
 *
 * dta_rollouts_build merges N token sequences into the prefix tree of the
 * paper's problem formulation (section 3): nodes are token segments, every
 * sequence is a root-to-node path, and a node ends exactly where sequences
 * branch or where one ends (a sequence contained in a longer one ends at an
 * interior node; equal sequences share their node).  Nodes are numbered in DFS
 * preorder with children in ascending order of their first token, i.e. in the
 * lexicographic order of the sequences, which is a valid DFS order of the tree
 * (section 4), so (parent, seg_len) passed to dta_tree_build are packed in
 * exactly this order and `tokens` is the packed token-id array.
 *   tokens      : host, concatenated token ids of all sequences.
 *   seq_offsets : host, [n_seqs + 1], seq_offsets[0] = 0, strictly increasing
 *                 (no empty sequence), else DTA_ERR_INVALID_ARG.
 *   out         : receives a new object; free it with dta_rollouts_destroy.
 * DTA_ERR_BAD_TREE if the tree would have more than 2^31 - 1 tokens.
 */
typedef struct dta_rollouts dta_rollouts_t;
typedef struct {
  int32_t n_seqs;
  int32_t n_nodes;
  int64_t n_tokens;         /* unique tree tokens                                              */
  const int32_t* parent;    /* [n_nodes]  tree arrays for dta_tree_build                       */
  const int32_t* seg_len;   /* [n_nodes]                                                       */
  const int32_t* tokens;    /* [n_tokens] token ids in the packed order                        */
  const int32_t* seq_node;  /* [n_seqs]   node at which input sequence i ends                  */
  const int32_t* order;     /* [n_seqs]   input index of the i-th sequence in lexicographic
                                          order (a proper prefix first, ties in input order)   */
  const int64_t* lcp;       /* [n_seqs]   common prefix length of the i-th and (i-1)-th
                                          sequence of that order; lcp[0] = 0                   */
} dta_rollouts_view_t;
int dta_rollouts_build(const int32_t* tokens, const int64_t* seq_offsets, int32_t n_seqs,
                       dta_rollouts_t** out);
/* Borrowed host pointers into the object, valid until dta_rollouts_destroy. */
int dta_rollouts_view(const dta_rollouts_t* rollouts, dta_rollouts_view_t* out);
void dta_rollouts_destroy(dta_rollouts_t* rollouts);

/*
 * dta_rollouts_partition - the paper's load-balanced DFS-contiguous partitioning
 * (section 4; pseudocode appendix): the sequences in lexicographic order are cut
 * into k contiguous groups such that the largest group cost is minimal, the cost
 * of a group being the tree tokens it needs (its first sequence, plus for every
 * further one its length minus the common prefix with its predecessor).  Binary
 * search on the cost bound with a greedy feasibility scan; if that yields fewer
 * than k groups, the first group with more than one sequence is split after its
 * first sequence until there are k.  1 <= k <= n_seqs, else DTA_ERR_INVALID_ARG.
 *   group_begin : host out, [k + 1]; group g is positions
 *                 [group_begin[g], group_begin[g+1]) of the lexicographic order.
 *   group_cost  : host out, [k], tree tokens of each group.
 */
int dta_rollouts_partition(const dta_rollouts_t* rollouts, int32_t k, int32_t* group_begin,
                           int64_t* group_cost);

/*
 * dta_tree_plan - the order in which the paper's optimised executor processes
 * a tree, as a list of operations and of the segment calls that carry them out.
 * Host only, integer only.
 *
 * Leaf order (pseudocode appendix, algorithm "Backward DFS Order"): bottom-up,
 * a leaf's tail is its depth in tokens; an internal node orders its children
 * leaf first, then by smaller tail (ties: smaller node id; the roots of a
 * forest are ordered the same way) and takes its first child's tail; the leaf
 * order of the DFS under these child orders, reversed, is leaf_order.
 *
 * Schedule (algorithm "Dynamic Tree Attention Backward", section 3.2): for each
 * leaf in that order, pop what the active stack does not share with it, forward
 * and push its suffix, and, where the next pop will leave part of the suffix on
 * the stack, a FWD-NoGrad anchor for that part; at the end pop everything.  A
 * pop of depths (lo, hi] is cut at evenly spaced boundaries at most `block`
 * tokens apart (block <= 0: never cut) and runs last chunk first, each chunk as
 * a recomputing forward followed by its backward.
 *
 * An operation works on depths [lo, hi) (0-based token positions) of the root
 * path of `leaf`; for pops that is the leaf that was pushed last.  calls[
 * call_ptr[i] .. call_ptr[i+1]) are operation i as rows [t_begin, t_end) of one
 * node each, ready for dta_tree_attn_fwd_segment (DTA_OP_FWD, DTA_OP_REFWD,
 * DTA_OP_FWD_NOGRAD) and dta_tree_attn_bwd_segment (DTA_OP_BWD); forwards list
 * the root side first, backwards the leaf side first.  Issued in this order on
 * zeroed accumulators the calls reproduce dta_tree_attn_fwd / _bwd.
 */
enum { DTA_OP_FWD = 0, DTA_OP_REFWD = 1, DTA_OP_BWD = 2, DTA_OP_FWD_NOGRAD = 3 };
typedef struct {
  int32_t op;      /* DTA_OP_*                                   */
  int32_t leaf;    /* node id of the leaf whose root path is meant */
  int64_t lo, hi;  /* depth range in tokens                       */
} dta_plan_op_t;
typedef struct {
  int32_t op;      /* DTA_OP_* of the operation it belongs to     */
  int32_t node;    /* node id                                     */
  int64_t t_begin, t_end;  /* packed rows, inside that node       */
} dta_plan_call_t;
typedef struct dta_plan dta_plan_t;
typedef struct {
  int32_t n_leaves;
  const int32_t* leaf_order;       /* [n_leaves] node ids                                  */
  int64_t n_ops;
  const dta_plan_op_t* ops;        /* [n_ops]                                              */
  const int64_t* call_ptr;         /* [n_ops + 1]                                          */
  int64_t n_calls;
  const dta_plan_call_t* calls;    /* [n_calls]                                            */
  int64_t n_fwd;                   /* regular forwards = n_leaves                          */
  int64_t n_fwd_nograd;            /* anchors, at most n_leaves                            */
  int64_t n_chunks;                /* popped chunks (one REFWD and one BWD each)           */
  int64_t max_stack_tokens;        /* longest active stack = longest root-to-leaf path     */
} dta_plan_view_t;
int dta_tree_plan(const dta_tree_t* tree, int64_t block, dta_plan_t** out);
/* Borrowed host pointers into the plan, valid until dta_plan_destroy. */
int dta_plan_view(const dta_plan_t* plan, dta_plan_view_t* out);
void dta_plan_destroy(dta_plan_t* plan);

/* Static, human-readable name of a status code. */
const char* dta_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* DTA_H_ */
