/*
 * c2t.h — C ABI of the MI355X (gfx950) implementation of the per-layer hot path of
 * C2T classifier-based token-tree construction (arXiv 2502.13652).
 *
 * One draft phase is Algorithm 1 of the paper: starting from the root token, each
 * iteration takes the draft model's logits for every node of the current tree layer
 * ("frontier"), keeps the TopK most probable children per node (Sec. 4.2.2, purpose 1),
 * gives each child the features joint probability P (Eq. 1), entropy H of the
 * distribution it was drawn from (Eq. 2, first line, natural log) and depth d,
 * scores it with the two-layer ReLU FFN classifier C = sigmoid(F(P,H,d)) (Eq. 3,
 * Sec. 4.1), drops children with C <= beta (first pruning, Sec. 4.2.1), keeps the
 * `max_frontier` most confident survivors (second pruning, Sec. 4.2.2, purpose 2)
 * within a total node budget (EAGLE-2's N, Sec. 2.2), and appends them to the tree.
 * The draft-model call between layers is the caller's: it reads the new frontier
 * with c2t_get_frontier, runs its model, and hands the logits to c2t_expand_layer.
 * c2t_finalize_tree emits what tree attention (Sec. 2.2) needs for verification.
 *
 * Conventions
 *  - Every pointer is tagged [host] or [device] below.  The library never allocates,
 *    frees or synchronises device memory: the caller owns all of it, including the
 *    workspace, and passes the stream (a hipStream_t as void*, NULL = default stream)
 *    that every kernel of a call is enqueued on.  Calls return after enqueueing.
 *  - Every call on a context is made with the workspace's device current, and calls on one
 *    context are not thread-safe (one draft phase at a time per context; use one context per
 *    stream for concurrent phases).
 *  - Return value: 0 = C2T_OK, negative = error (c2t_strerror).  Argument and state
 *    errors are found on the host before anything is enqueued.  Data errors (NaN or
 *    +inf logits, a row with no finite logit) never fail a call: the row yields no
 *    candidates and bit 0 of that sequence's status word is set.
 *  - Call order per draft phase: c2t_reset, then at most max_depth x c2t_expand_layer,
 *    then c2t_finalize_tree; anything else is C2T_ERR_STATE.
 *  - Ties: a row's TopK is ordered by (logit desc, token id asc); survivors of a layer
 *    are ranked by (classifier logit z desc, token id asc, parent slot asc).
 *  - Decisions are taken on the classifier's pre-sigmoid logit z in fp32:
 *    C > beta  <=>  z > logit(beta), logit(beta) rounded once to fp32 (beta = 0 keeps all).
 */
#ifndef C2T_H
#define C2T_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct c2t_ctx c2t_ctx; /* opaque, host memory */

enum { C2T_F32 = 0, C2T_BF16 = 1 };

enum {
  C2T_OK = 0,
  C2T_ERR_INVALID_ARG = -1, /* NULL pointer, value out of range                        */
  C2T_ERR_UNSUPPORTED = -2, /* misaligned logits / stride, size above a compiled limit */
  C2T_ERR_WORKSPACE = -3,   /* workspace NULL, misaligned (256 B) or too small         */
  C2T_ERR_STATE = -4,       /* call out of order, classifier not set                   */
  C2T_ERR_HIP = -5,         /* a HIP runtime call failed (launch, event)                */
  C2T_ERR_NOMEM = -6        /* host memory for the context could not be allocated      */
};

/* Limits compiled into the kernels. */
#define C2T_MAX_TOP_K 64
#define C2T_MAX_FRONTIER 64
#define C2T_MAX_HIDDEN 256
#define C2T_MAX_BUDGET 1024
#define C2T_MAX_CANDIDATES 2048 /* max_frontier * top_k */
#define C2T_MAX_HISTORY 32768   /* max_depth * max_frontier * top_k with rerank = 1 */

typedef struct {
  int32_t batch;        /* B: independent sequences                                   */
  int32_t vocab;        /* V: logits per row, >= top_k                                */
  int32_t max_frontier; /* F: nodes expanded per layer (second pruning width)         */
  int32_t top_k;        /* K: children scored per frontier node                       */
  int32_t max_depth;    /* D = d_max of Algorithm 1                                   */
  int32_t budget;       /* N: max candidate nodes per sequence, root excluded         */
  int32_t hidden;       /* h: classifier hidden width                                 */
  int32_t logits_dtype; /* C2T_F32 or C2T_BF16                                        */
  float beta;           /* 0 <= beta < 1                                              */
  int32_t entropy_top_m; /* 0: entropy over the full vocabulary (Eq. 2, line 1);
                            M > 0: over the M most probable tokens, with the probabilities
                            of the full softmax (Eq. 2, line 2).  Rows that have to be split
                            over workgroups (fp32 rows of more than 49152 logits, bf16 rows of
                            more than 262144) are gone over once more by one workgroup for it  */
  int32_t rerank;        /* 1: keep every scored candidate of every layer in the workspace so that
                            c2t_finalize_tree_reranked can be called (max_depth * max_frontier *
                            top_k <= C2T_MAX_HISTORY); 0: only the tree                          */
} c2t_config;

/* Caller-owned [device] output buffers of c2t_finalize_tree, N = budget.
 * Node order is breadth first, within a layer by rank.  Entries >= n_nodes[b] are
 * written as tokens/parent -1, position 0, reals 0, mask 0. */
typedef struct {
  int32_t* tokens;     /* [B][N] token id of each candidate node                       */
  int32_t* parent;     /* [B][N] node index of the parent, -1 = child of the root      */
  int32_t* position;   /* [B][N] depth + 1 (offset from the root token)                */
  float* conf;         /* [B][N] C = sigmoid(z)                                        */
  float* joint_prob;   /* [B][N] P, Eq. 1                                              */
  float* entropy;      /* [B][N] H of the row the node was drawn from, Eq. 2           */
  int32_t* n_nodes;    /* [B]                                                          */
  uint8_t* mask;       /* [B][N][N] mask[i][j] = 1 iff j == i or j is an ancestor of i;
                          the root is not a slot (every node attends to it)            */
  uint32_t* status;    /* [B] bit 0: a consumed row held NaN / +inf / no finite logit;
                          bit 1 (informational): a bf16 row took the slower two-pass
                          path (a logit >= 2^7 or in (-2^10, -2^7]; one value held by
                          more than 65535 logits; logits below 2^-25 in magnitude, -inf
                          or <= -2^10 among the K largest)                             */
} c2t_tree_out;

/* Bytes of device workspace a context of this configuration needs.  [host] out. */
int c2t_workspace_bytes(const c2t_config* cfg, size_t* out);

/* Create a context over a caller-owned [device] workspace (256-byte aligned, at least
 * c2t_workspace_bytes).  The workspace must stay valid until c2t_destroy.  [host] out. */
int c2t_create(const c2t_config* cfg, void* dev_workspace, size_t workspace_bytes, c2t_ctx** out);
void c2t_destroy(c2t_ctx* ctx);

/* Classifier parameters of Eq. 3, [host] pointers.  The values travel to the workspace as the
 * arguments of small kernels enqueued on `stream` (one per 240 floats of the 5h + 1): they are read
 * before the call returns, so the host arrays may be reused or freed at once, the call never blocks
 * on the device and never touches pageable memory asynchronously, it orders with the layer kernels
 * of the same stream like any other launch, and it may be repeated at any time between draft phases.  W1 is [h][3] with input order
 * (P, H, d); b1 [h]; w2 [h]; b2 scalar.  z = b2 + sum_j w2[j] * relu(W1[j].(P,H,d) + b1[j]),
 * evaluated in fp32 as a fixed chain of fused multiply-adds, j ascending. */
int c2t_set_classifier(c2t_ctx* ctx, const float* W1, const float* b1, const float* w2, float b2,
                       void* stream);

/* Start a draft phase (Algorithm 1, first four lines): tree = {root}, frontier = {root},
 * P_root = 1, depth 0, every sequence's node count and status cleared. */
int c2t_reset(c2t_ctx* ctx, void* stream);

/* One iteration of Algorithm 1's loop for every sequence.
 * logits [device]: [B][F][row_stride_elems] of the configured dtype; row f of sequence b is
 * the draft model's output for frontier slot f.  Only rows f < n_frontier[b] are read
 * (one row per sequence in the first layer).  The base address must be 16-byte aligned and
 * row_stride_elems >= vocab a multiple of 16 bytes, else C2T_ERR_UNSUPPORTED.
 * Effects: appends the kept children to the tree, replaces the frontier by them. */
int c2t_expand_layer(c2t_ctx* ctx, const void* logits, int64_t row_stride_elems, void* stream);

/* [device] pointers into the workspace describing the current frontier, valid until the
 * next reset/expand: tokens [B][F] (token id of each frontier node; -1 for the root slot),
 * parent_slot [B][F] (slot, in the previous frontier, of the node's parent: which of the
 * previous rows it was drawn from), n_frontier [B] (0 = this sequence's loop has ended:
 * Algorithm 1's guard "exists C_i > beta").  Any of the three out-pointers may be NULL. */
int c2t_get_frontier(c2t_ctx* ctx, const int32_t** tokens, const int32_t** parent_slot,
                     const int32_t** n_frontier);

/* Every candidate given a confidence in the last expanded layer, [device] pointers into the
 * workspace, arrays [B][F*K] indexed slot*K + rank_in_row (entries of unused slots are stale):
 * token, p (generation probability), P, H, z, kept (1 = appended to the tree); n_cand [B].
 * Any out-pointer may be NULL. */
int c2t_get_candidates(c2t_ctx* ctx, const int32_t** n_cand, const int32_t** token, const float** p,
                       const float** P, const float** H, const float** z, const int32_t** kept);

/* Emit the verification inputs of the tree built so far into caller-owned [device] buffers
 * (every field of `out` non-NULL). */
int c2t_finalize_tree(c2t_ctx* ctx, const c2t_tree_out* out, void* stream);

/* EAGLE-2-style reranking (Sec. 2.2: all candidate nodes are reranked and the top N selected),
 * for a context created with rerank = 1: over every candidate that was given a confidence in any
 * layer of this draft phase, kept by the prunings or not, the n_out (1..C2T_MAX_BUDGET) best by the
 * smallest classifier logit on the candidate's path from the root (itself included).  That score
 * never increases along a path, so with the order (score desc, depth asc, scoring order asc: slot,
 * then rank in the row) every selected candidate's parent is selected before it: the result is a
 * tree for any classifier, and the plain top-n_out by confidence for one that is monotone along
 * paths (EAGLE-2's joint probability).  `out` as for c2t_finalize_tree with N = n_out; nodes in
 * selection order.  Same place in the call order as c2t_finalize_tree. */
int c2t_finalize_tree_reranked(c2t_ctx* ctx, const c2t_tree_out* out, int32_t n_out, void* stream);

/* For callers that cannot allocate device memory or hand over a workspace slice for scratch (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * reranking as c2t_finalize_tree_reranked, same arguments, same results, but the kernel's scratch
 * (one int32 per history entry, batch * max_depth * max_frontier * top_k of them) lives in a static
 * device array inside the library instead of the context's workspace.  The call allocates nothing
 * and frees nothing.  Limit: at most C2T_STATIC_RERANK_ENTRIES history entries, else
 * C2T_ERR_UNSUPPORTED; C2T_ERR_HIP if the array's device address cannot be obtained.  Every call on
 * one GPU, from any context, uses that GPU's one array: calls that overlap on a GPU (different
 * streams, or graphs replayed concurrently) race and must be serialised by the caller; calls on
 * different GPUs are independent.  Nothing needs clearing between calls: the kernel writes every
 * scratch entry before it reads it. */
#define C2T_STATIC_RERANK_ENTRIES (4 * 1024 * 1024)   /* 16 MiB of device memory per GPU, held until the process ends */
int c2t_finalize_tree_reranked_static(c2t_ctx* ctx, const c2t_tree_out* out, int32_t n_out, void* stream);

/* Per-launch accounting for benchmarks: [device] pointer to int32 [max_depth + 1];
 * entry l = number of logits rows layer l's expand consumed (sum over sequences of
 * n_frontier), filled as the layers run. */
int c2t_get_layer_rows(c2t_ctx* ctx, const int32_t** layer_rows);

/* Launch-shape override for experiments: number of workgroups a logits row is split over
 * in the first layer (one row per sequence) and in later layers; 0 = library default.
 * C2T_ERR_UNSUPPORTED below the minimum the vocabulary needs.
 * By default a launch of few long bf16 rows (at most 128 rows of at least 65,536 logits, e.g. a
 * single sequence's layer or a batch's first layer) lets several workgroups on otherwise idle CUs
 * count one row together: they add their histograms up through the workspace before the row's one
 * epilogue, so the results are those of an unshared row.  A count set here (1 included) is taken
 * literally and switches that off for the layers it is set for. */
int c2t_set_row_splits(c2t_ctx* ctx, int32_t first_layer, int32_t other_layers);

/* Workgroups that work on one logits row in the first layer's launch and in the later layers'
 * launches as the context stands: the split count, or the number of workgroups that share a row
 * (see c2t_set_row_splits).  [host] outputs; either may be NULL. */
int c2t_get_row_workgroups(const c2t_ctx* ctx, int32_t* first_layer, int32_t* other_layers);

/* Optional timing of the layer kernel with HIP events attached to each launch on the caller's
 * stream (they take the kernel's own begin and end).  c2t_profile_enable creates `capacity` event
 * pairs (host resources; 0 disables and destroys them).  After the caller has synchronised the
 * stream, c2t_profile_read writes the duration in milliseconds of each launch recorded since the
 * last read to ms[0..*n) ([host], capacity given in *n on entry) and forgets them.
 * Attaching the events costs the host about 20 us a launch; c2t_profile_sample(every, first)
 * attaches them only to the launches of draft phases first, first + every, first + 2 every, ...
 * (phases are counted in c2t_reset calls since c2t_profile_enable, from 0); every >= 1,
 * 0 <= first < every, else C2T_ERR_INVALID_ARG; default: every phase. */
int c2t_profile_enable(c2t_ctx* ctx, int32_t capacity);
int c2t_profile_sample(c2t_ctx* ctx, int32_t every, int32_t first);
int c2t_profile_read(c2t_ctx* ctx, float* ms, int32_t* n);

/* Plain streaming read of `bytes` (multiple of 16) of [device] memory, summed into one
 * uint32 at [device] out: the practical HBM read ceiling to compare the logits pass with. */
int c2t_stream_read(const void* dev_ptr, size_t bytes, uint32_t* dev_out, void* stream);

/* The same for `rows` rows of `row_bytes` (multiple of 16) each, `row_stride_bytes` (multiple of 16,
 * >= row_bytes) apart in [device] memory, read the way the logits pass reads them (one workgroup
 * per row): the ceiling for that access pattern. */
int c2t_stream_read_rows(const void* dev_ptr, int32_t rows, size_t row_bytes, size_t row_stride_bytes,
                         uint32_t* dev_out, void* stream);

/* Profiling build only (the library compiled with -DC2T_PHASE_TIMES; paper_2502_13652_amd/phase_times.py
 * builds and drives it): copies to [host] out, for the first n_workgroups (<= 8192) workgroups of the
 * layer kernel's launches so far, 16 uint64 each: the 100 MHz wall-clock time at which the workgroup's
 * first thread last passed each phase boundary (start, end of its own stream, histogram complete, sums,
 * K-th largest value, cells listed, cells re-read, top K ranked, row scored and handed over, sequence
 * ticket taken, sequence pruned, four steps inside the sequence's pruning, split row merged; unused slots keep
 * their previous value).  Synchronises the device.
 * The normal build returns C2T_ERR_UNSUPPORTED. */
int c2t_phase_times_read(uint64_t* out, int32_t n_workgroups);

const char* c2t_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* C2T_H */
