/*
 * specpipe.h -- C ABI of the SpecPipe stage library for AMD MI355X (gfx950).
 *
 * One pipeline stage of SpecPipe (arXiv 2504.04104): the stage's decoder layers
 * run on newly inserted nodes of the dynamic speculative token tree
 * ("node-wise computation", Sec. 3.3.2, Algorithm 1 lines 1-3), and pruning
 * propagation compacts the tree tables and the KV cache once a token has been
 * verified (Sec. 3.2 "to-subtree pruning", Sec. 3.3.2, Algorithm 1 lines 5-7).
 *
 * Numbering.  The paper's tree has the last verified token as root tau_1.  Here
 * that root is the last token of the committed context ("prefix"), and only the
 * speculative tokens are numbered: node k of a request is the paper's
 * tau_(k+2); parent -1 means "child of the root".  Parents always have a
 * smaller index than their children.  depth(k) = 0 for children of the root.
 * A request's committed context has prefix_len tokens (root included) and its
 * tree has n_live nodes; node k's K/V rows live in cache slot
 * slot_base + prefix_len + k, and it stands for sequence position
 * prefix_len + depth(k) (each tree level is one future position, Sec. 3.2).
 *
 * Memory.  Every device byte is owned by the caller: weights, the KV slab, the
 * table arena and the workspace are passed in as device pointers and must stay
 * valid until sp_stage_destroy().  The library allocates no device memory of
 * its own and creates no streams (the HIP graphs sp_stage_forward may build hold
 * whatever the runtime needs for them: up to 256 instantiated graphs per stage, one per distinct call
 * shape, each of 9-10 kernel nodes per layer, i.e. some tens of kilobytes of host and device memory
 * per graph that the HIP runtime allocates at the capturing call).  All device work of a call is enqueued
 * on the stream passed to it, in call order; calls return without waiting for
 * the GPU unless stated.  Host arrays passed in are read before the call returns.
 * One stream should carry all calls of a stage: the workspace, the page tables
 * and the device copy of a call's plan are reused from call to call.
 *
 * KV slab layout (element type = config dtype), index order slowest to fastest:
 *     [layer][K=0|V=1][kv_head][slot][d_head]
 * with `kv_slots` slots per head.  K rows are stored rotated (post-RoPE).  A
 * request owns the slot range [slot_base, slot_base + capacity).  One K or V
 * row of one token is n_kv_heads * d_head elements, i.e. 2*8*128*2 B = 4096 B
 * per token per layer for the 70B shape in bf16 (Sec. 4.5, Table 1).
 *
 * Weights: every matrix is [out_features][in_features] row-major (y = x W^T), in
 * the config dtype.  wqkv stacks the query rows, then the key rows, then the
 * value rows; wgu stacks the gate rows, then the up rows.
 *
 * Errors: every call returns SP_OK (0) or a negative sp_status; on error the
 * state is unchanged.  A handle is not thread-safe.
 */
#ifndef SPECPIPE_H
#define SPECPIPE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SP_VERSION 1
#define SP_MAX_TREE_NODES 256   /* live speculative nodes per request            */
#define SP_MAX_BATCH_REQ 64     /* requests per sp_stage_forward / *_batch call   */
#define SP_ANC_WORDS 4          /* 64-bit words of one ancestor-bitmask row       */

typedef struct sp_stage sp_stage;
typedef void* sp_stream;        /* a hipStream_t; NULL = the default stream */

typedef enum sp_status {
  SP_OK = 0,
  SP_E_INVALID = -1,      /* null pointer, bad size, bad config                       */
  SP_E_CAPACITY = -2,     /* tree, slot range, batch or workspace too small           */
  SP_E_BAD_PARENT = -3,   /* parent not in {-1} U [0, index of the child)             */
  SP_E_BAD_REQ = -4,      /* request id out of range or not initialised               */
  SP_E_BAD_NODE = -5,     /* node index outside the live tree                         */
  SP_E_ORDER = -6,        /* forward / accept of a node whose path has not been forwarded */
  SP_E_PENDING = -7,      /* a prune awaits sp_kv_compact (or none does)              */
  SP_E_HIP = -8,          /* a HIP runtime call failed; see sp_last_hip_error()       */
  SP_E_UNSUPPORTED = -9   /* shape or dtype the kernels do not cover                  */
} sp_status;

typedef enum sp_dtype { SP_F32 = 0, SP_BF16 = 1 } sp_dtype;
typedef enum sp_prune_mode { SP_ACCEPT = 0, SP_DROP = 1, SP_CLEAR = 2 } sp_prune_mode;

/* sp_config.flags */
#define SP_FLAG_SIMPLE_KERNELS 1u   /* use the plain (non-MFMA) kernels for every step */
#define SP_FLAG_PACKED_WEIGHTS 2u   /* wqkv, wo, wgu, wd were re-laid by sp_pack_weights() (bf16 MFMA path only) */
#define SP_FLAG_NO_GRAPHS 8u        /* never replay HIP graphs inside sp_stage_forward (see there) */
#define SP_FLAG_PAGED_KV 4u         /* requests hold their cache in pages of page_slots slots (see below) */

typedef struct sp_config {
  int32_t n_layers;
  int32_t d_model;
  int32_t n_q_heads;
  int32_t n_kv_heads;      /* divides n_q_heads; query head h reads KV head h / (n_q/n_kv) */
  int32_t d_head;          /* even, multiple of 8, <= 256 */
  int32_t d_ff;
  float rms_eps;
  float rope_theta;        /* angle of pair t at position p: p * theta^(-2t/d_head); pairs (t, t+d_head/2) */
  int32_t dtype;           /* sp_dtype: storage type of weights, hidden rows and KV */
  int32_t max_requests;
  int32_t max_tree_nodes;  /* <= SP_MAX_TREE_NODES */
  int32_t max_batch_nodes; /* most rows (sum of n_nodes) one sp_stage_forward call may carry */
  int64_t kv_slots;        /* slots per (layer, K|V, head) plane of the slab */
  uint32_t flags;
  int32_t page_slots;      /* SP_FLAG_PAGED_KV: slots per page, a power of two in [32, 4096] that divides kv_slots */
} sp_config;

/* Device pointers of one layer's weights. */
typedef struct sp_layer_weights {
  const void* wqkv;    /* [(n_q + 2 n_kv) * d_head][d_model] */
  const void* wo;      /* [d_model][n_q * d_head]            */
  const void* wgu;     /* [2 * d_ff][d_model]: gate, then up */
  const void* wd;      /* [d_model][d_ff]                    */
  const void* norm1;   /* [d_model] gain of the attention RMSNorm */
  const void* norm2;   /* [d_model] gain of the FFN RMSNorm       */
} sp_layer_weights;

typedef struct sp_sizes {
  size_t kv_bytes;         /* KV slab */
  size_t tables_bytes;     /* per-request tree tables and prune maps */
  size_t workspace_bytes;  /* activations and partial results of one forward call */
  size_t kv_plane_bytes;   /* bytes between consecutive kv_heads   */
  size_t kv_row_bytes;     /* bytes of one (slot, head) row = d_head * element size */
} sp_sizes;

typedef struct sp_buffers {
  void* kv;        size_t kv_bytes;
  void* tables;    size_t tables_bytes;
  void* workspace; size_t workspace_bytes;
} sp_buffers;

/* Host copy of one request's tables, for tests and debugging (Sec. 3.2: I, P and M;
 * M is held as one ancestor bitmask per node: bit j of anc[i] is M[i][j]). */
typedef struct sp_tree_view {
  int32_t prefix_len;
  int32_t n_live;
  int32_t parent[SP_MAX_TREE_NODES];
  int32_t depth[SP_MAX_TREE_NODES];
  int32_t token[SP_MAX_TREE_NODES];
  float prob[SP_MAX_TREE_NODES];
  uint64_t anc[SP_MAX_TREE_NODES][SP_ANC_WORDS];
  int32_t pred[SP_MAX_TREE_NODES];   /* the model's next token after the node, -1 while unknown */
  int32_t root_pred;                 /* ... after the committed context, -1 while unknown      */
} sp_tree_view;

/* Output head of the last stage (device pointers; storage type of the config).  With
 * SP_FLAG_PACKED_WEIGHTS the vocabulary matrix is expected in the re-laid order too
 * (sp_pack_matrix). */
typedef struct sp_head_weights {
  const void* norm;     /* [d_model] gain of the final RMSNorm   */
  const void* wvocab;   /* [vocab][d_model]                      */
  int32_t vocab;
  int32_t reserved;
} sp_head_weights;

/* ---- set-up ---------------------------------------------------------------- */

/* Buffer sizes a stage of this config needs: the device state {E_i, M_i, KV_i} that Algorithm 1
 * gives every device (hidden rows in flight, tree tables, KV cache) plus the scratch of one
 * forward call.  Pure host arithmetic. */
int sp_stage_query_sizes(const sp_config* cfg, sp_sizes* out);

/* Load-time re-layout of one layer's four projection matrices (bf16) into the order the
 * matrix-core kernels read them in: per strip of 16 output rows and per step of 32 inputs,
 * one contiguous 1 KB block holding, for lane l of a wave, the 8 values
 * W[strip*16 + l%16][step*32 + (l/16)*8 .. +8].  It changes no value and no result, only
 * how many bytes each wave load fetches contiguously.  `in` and `out` hold device pointers;
 * `out` buffers are caller-allocated, of the same sizes, and distinct from `in`.  norm1 and
 * norm2 are not touched (pass the originals to sp_stage_create).  Create the stage with
 * SP_FLAG_PACKED_WEIGHTS to use the result.  Errors: SP_E_UNSUPPORTED unless dtype is bf16
 * and d_model, d_ff are multiples of 32. */
int sp_pack_weights(const sp_config* cfg, const sp_layer_weights* in, const sp_layer_weights* out,
                    sp_stream stream);

/* The same re-layout for one [n_rows][n_cols] bf16 matrix (n_rows % 16 == 0, n_cols % 32 == 0):
 * used for the vocabulary matrix of the output head. */
int sp_pack_matrix(const void* in /*device*/, void* out /*device, distinct*/, int32_t n_rows, int32_t n_cols,
                   sp_stream stream);

/* Builds a stage: one device of the pipeline with its share of the model's layers and the state
 * {E_i, M_i, KV_i} of Algorithm 1 ("Input": each device holds hidden states, a copy of the tree mask
 * and its KV cache; Sec. 3.3.2).  `layers` is a host array of n_layers entries holding device
 * pointers.  Buffers must be at least as large as sp_stage_query_sizes() says and
 * 256-byte aligned.  The tables buffer is initialised on `stream`. */
int sp_stage_create(const sp_config* cfg, const sp_layer_weights* layers, const sp_buffers* buffers,
                    sp_stream stream, sp_stage** out);
void sp_stage_destroy(sp_stage* stage);

/* Declares request `req` and its initial device state (Algorithm 1, "Input": KV_i holds the
 * committed context, M_i is the mask of a tree that holds only the root): it owns slots
 * [slot_base, slot_base+capacity) of every plane, of which the first prefix_len (>= 1: the root) already hold the rotated K
 * and V of the committed context for every layer.  Its tree becomes empty.  May be
 * called again to reset a request. */
int sp_request_init(sp_stage* stage, int32_t req, int64_t slot_base, int32_t capacity,
                    int32_t prefix_len, sp_stream stream);

/* Paged cache (SP_FLAG_PAGED_KV; SpecPipe-DB stores its cache PagedAttention-style, Sec. 4
 * "Implementation").  The slab is cut into kv_slots / page_slots pages; the library hands
 * them out: a request holds the pages of its first prefix_len + n_live logical slots, in
 * any physical order.  Logical slot s of a request lives in physical slot
 * page[s / page_slots] * page_slots + s % page_slots of every (layer, K|V, head) plane.
 * sp_request_init takes slot_base = 0 and capacity = the most logical slots the request may
 * reach; it takes the pages of the committed context, whose K and V the caller then writes
 * at the physical slots sp_request_pages reports.  sp_tree_insert takes further pages as
 * the tree grows (SP_E_CAPACITY if none is free: nothing changes), sp_kv_compact returns the
 * pages past the compacted rows, sp_request_release returns all.  Page bookkeeping is host
 * state; the device tables are updated in stream order, so one stream must carry all calls
 * of a stage. */
int sp_request_pages(const sp_stage* stage, int32_t req, int32_t* pages_out /*host, nullable*/,
                     int32_t max_pages, int32_t* n_pages_out /*host, nullable*/);
/* Ends a request (both storage modes): its pages, if any, return to the allocator. */
int sp_request_release(sp_stage* stage, int32_t req, sp_stream stream);
/* Pages not held by any request (SP_E_INVALID for a null stage). */
int sp_stage_free_pages(const sp_stage* stage);

/* ---- the hot path ------------------------------------------------------------ */

/* Layer appending (Sec. 3.2): appends n_new nodes to request `req`.  parents[k] is
 * -1, a live node, or one of this call's earlier nodes.  The new nodes get indices
 * n_live .. n_live+n_new-1 in argument order (*first_index_out = old n_live); pass
 * them sorted by parent order to keep the paper's level-by-level indexing.  tokens
 * (I) and probs (P) are carried, compacted and returned but never interpreted; NULL
 * stores zeros.  Errors: SP_E_CAPACITY (tree or slot range full), SP_E_BAD_PARENT,
 * SP_E_BAD_REQ, SP_E_PENDING. */
int sp_tree_insert(sp_stage* stage, int32_t req, int32_t n_new, const int32_t* parents /*host*/,
                   const int32_t* tokens /*host, nullable*/, const float* probs /*host, nullable*/,
                   int32_t* first_index_out /*host, nullable*/, sp_stream stream);

/* The same for several requests in one launch (dynamic batching, Sec. 4 "Implementation"):
 * request req_ids[i] appends n_new[i] nodes; parents / tokens / probs hold the nodes of all
 * requests back to back in that order; first_index_out[i] = index of request i's first new
 * node.  Every request is validated before anything changes.  Requests must be distinct. */
int sp_tree_insert_batch(sp_stage* stage, int32_t n_req, const int32_t* req_ids /*host*/,
                         const int32_t* n_new /*host*/, const int32_t* parents /*host*/,
                         const int32_t* tokens /*host, nullable*/, const float* probs /*host, nullable*/,
                         int32_t* first_index_out /*host, nullable*/, sp_stream stream);

/* Node-wise computation (Algorithm 1 lines 1-3): runs every layer of the stage on
 * nodes [first_node[i], first_node[i]+n_nodes[i]) of request req_ids[i], i < n_req,
 * under the tree mask: a node attends to its request's committed context and to
 * itself and its ancestors.  x_in / x_out: device, [sum n_nodes][d_model] in the
 * config dtype, rows ordered by (position in req_ids, node index); they may alias.
 * The nodes' K and V rows are written to the slab.  A node's parent must have been
 * forwarded before or be part of this call (SP_E_ORDER).  A request may appear once.
 * Launch overhead: when a call has the same shape (rows, attention work items) as an
 * earlier one, its launches except the first and the last are replayed from a HIP graph
 * captured the second time that shape was seen; results are identical.  The call stays
 * eager on a stream that cannot be captured (the default stream: pass a stream of your
 * own), while the stream is being captured by the caller, while sp_profile_begin
 * brackets fall into it, or with SP_FLAG_NO_GRAPHS. */
int sp_stage_forward(sp_stage* stage, int32_t n_req, const int32_t* req_ids /*host*/,
                     const int32_t* first_node /*host*/, const int32_t* n_nodes /*host*/,
                     const void* x_in /*device*/, void* x_out /*device*/, sp_stream stream);

/* Pruning propagation, table part (Sec. 3.2, Algorithm 1 lines 5 and 7).
 * SP_ACCEPT(node): the verified token is `node`.  The path root..node joins the
 *   committed context (prefix_len grows by depth(node)+1 = *n_commit_out); the strict
 *   descendants of `node` stay as the tree, re-indexed by rank; children of `node`
 *   get parent -1; depths shrink by n_commit.
 * SP_DROP(node): `node` and its descendants leave the tree; nothing is committed.
 * SP_CLEAR: every speculative node leaves (a pipeline stall, Algorithm 1 lines 8-9: the true
 *   token then enters as a level of its own); `node` is ignored; nothing is committed.
 * On SP_ACCEPT the prediction stored for `node` becomes the root's (see sp_stage_verify_head).
 * Computes the keep flags from the mask column, their prefix sums, and the compacted
 * tables on the device, and leaves the old->new map there for sp_kv_compact, which
 * must be the next call for this request.  Outputs are computed on the host mirror.
 * SP_ACCEPT needs the whole path root..node to have been forwarded at this stage (its K/V rows
 * become committed context): SP_E_ORDER otherwise. */
int sp_tree_prune(sp_stage* stage, int32_t req, int32_t mode, int32_t node,
                  int32_t* n_live_out /*host, nullable*/, int32_t* n_commit_out /*host, nullable*/,
                  sp_stream stream);

/* Pruning propagation, cache part (Algorithm 1 line 6): K and V rows of the kept
 * nodes -- for SP_ACCEPT the mask is row(node) OR col(node), so the committed path
 * comes first -- move, in order, to the slots right after the old committed context,
 * for every layer.  If x_rows != NULL it holds n_rows hidden rows [n_rows][d_model]
 * (device) of nodes row_nodes[] (host; indices from before the prune, ascending):
 * rows whose node is outside col(node) (resp. inside the dropped subtree) are
 * removed in place (Algorithm 1 line 5).  *n_rows_out = surviving rows;
 * row_nodes_out[i] = new index of the node of surviving row i (-1 for the accepted
 * node itself, which is now the root).  Clears the pending state. */
int sp_kv_compact(sp_stage* stage, int32_t req, void* x_rows /*device, nullable*/, int32_t n_rows,
                  const int32_t* row_nodes /*host*/, int32_t* n_rows_out /*host, nullable*/,
                  int32_t* row_nodes_out /*host, nullable*/, sp_stream stream);

/* The same two steps for several requests in one launch each (dynamic batching,
 * Sec. 4 "Implementation").  Entries with modes[i] < 0 are skipped. */
int sp_tree_prune_batch(sp_stage* stage, int32_t n, const int32_t* req_ids, const int32_t* modes,
                        const int32_t* nodes, int32_t* n_live_out /*nullable*/,
                        int32_t* n_commit_out /*nullable*/, sp_stream stream);
int sp_kv_compact_batch(sp_stage* stage, int32_t n, const int32_t* req_ids, sp_stream stream);

/* Fixed-width expansion of the tree bottom (Sec. 3.3.3, "Fixed-width tree"): for each of the
 * n_bottom nodes bottom_nodes[] (host; live nodes in ascending order, or the single entry -1
 * for the root of an empty tree) the token source proposes k candidates, cand_tokens /
 * cand_probs (device, [n_bottom][k]; a negative token marks an absent candidate).  A
 * candidate's cumulative probability is its own probability times the probabilities stored in
 * the tables for the bottom node and its ancestors (float32, multiplied from the root
 * downwards).  The w candidates with the highest cumulative probability are kept -- an earlier
 * candidate wins a tie -- and written in parent order, ready for sp_tree_insert:
 * out_parents / out_tokens / out_probs (device, room for w entries) and *out_count (device).
 * n_bottom * k <= 4096 and w <= 256, else SP_E_CAPACITY.  Asynchronous on `stream`. */
int sp_tree_expand(sp_stage* stage, int32_t req, int32_t n_bottom, const int32_t* bottom_nodes /*host*/,
                   int32_t k, const int32_t* cand_tokens /*device*/, const float* cand_probs /*device*/,
                   int32_t w, int32_t* out_parents /*device*/, int32_t* out_tokens /*device*/,
                   float* out_probs /*device*/, int32_t* out_count /*device*/, sp_stream stream);

/* ---- verification on the last stage (Algorithm 1, "verify new token"; Sec. 3.4) ----- */

/* Next-token prediction of tree nodes from their outputs of the last decoder layer:
 *   pred = argmax_v ( RMSNorm(x; head->norm, rms_eps) . head->wvocab[v] ),
 * the lowest v among equal maxima (top-1 validation).  Rows of `x` (device, [sum n][d_model],
 * 16-byte aligned) are in the order of sp_stage_forward: request by request, nodes
 * first_node[i] .. first_node[i] + n_nodes[i] - 1, which must have been forwarded
 * (else SP_E_ORDER).  The prediction of every row is stored in its node's table entry and,
 * if the pointers are given, written to pred_out[row] / the winning logit to max_out[row]
 * (device).  The vocabulary matrix is read once; logits are not materialised on the bf16
 * matrix-core path (vocab % 64 == 0), otherwise they take vocab * rows floats of the
 * workspace (SP_E_CAPACITY if that does not fit).  Uses the stage's workspace: do not
 * overlap with sp_stage_forward on another stream. */
int sp_stage_verify_head(sp_stage* stage, const sp_head_weights* head, int32_t n_req,
                         const int32_t* req_ids /*host*/, const int32_t* first_node /*host*/,
                         const int32_t* n_nodes /*host*/, const void* x /*device*/,
                         int32_t* pred_out /*device, nullable*/, float* max_out /*device, nullable*/,
                         sp_stream stream);

/* For callers that cannot allocate device memory or hand over a workspace at the time of the call
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * sp_stage_verify_head with its intermediate buffers -- row descriptors, the normalised rows and the
 * per-tile (value, index) pairs or logits -- in a fixed array of SP_NOALLOC_SCRATCH_BYTES inside the
 * library's device image instead of the stage's workspace.  Same arguments, same results, same
 * errors, plus SP_E_CAPACITY when the call carries more than SP_NOALLOC_MAX_ROWS rows or its buffers
 * (rows * d_model * 6 bytes in bf16, plus rows * vocab / 32 floats on the matrix-core path or
 * rows * vocab floats otherwise) exceed the array.  Calls no allocating routine.  Every GPU the
 * library has created a stage on holds one such array until the process ends; all calls on a GPU
 * share it, each call overwrites what it reads before reading it (nothing has to start at zero),
 * and calls that overlap on one GPU (different streams) race. */
#define SP_NOALLOC_MAX_ROWS 64
#define SP_NOALLOC_SCRATCH_BYTES (8u << 20)
int sp_stage_verify_head_noalloc(sp_stage* stage, const sp_head_weights* head, int32_t n_req,
                                 const int32_t* req_ids /*host*/, const int32_t* first_node /*host*/,
                                 const int32_t* n_nodes /*host*/, const void* x /*device*/,
                                 int32_t* pred_out /*device, nullable*/, float* max_out /*device, nullable*/,
                                 sp_stream stream);

/* Declares the model's token after the committed context of a request whose tree the
 * last stage has not fed yet (after prefill or a stall).  Later it follows the accepts. */
int sp_request_set_root_pred(sp_stage* stage, int32_t req, int32_t token, sp_stream stream);

/* The verified token of each request: nodes_dev[i] (device) = the first child of the root
 * whose token equals the root's prediction, -1 if none does (stall) or the prediction is
 * unknown.  If nodes_host != NULL the result is also copied there asynchronously on
 * `stream` (pinned memory advised); it is valid once the stream has been synchronised.
 * The caller then issues sp_tree_prune(SP_ACCEPT, node), or SP_CLEAR and an insert of the
 * predicted token on a miss. */
int sp_tree_match(sp_stage* stage, int32_t n, const int32_t* req_ids /*host*/, int32_t* nodes_dev /*device*/,
                  int32_t* nodes_host /*host, nullable*/, sp_stream stream);

/* Pruning propagation decided on the device: sp_tree_prune + sp_kv_compact (without hidden rows) for the
 * listed requests, the verified node of request i read by the prune kernel from nodes_dev[i * stride]
 * (device; the output of sp_tree_match with stride 1, of sp_stage_verify_lossy with stride 2): a live node is
 * accepted (SP_ACCEPT), -1 clears the tree (SP_CLEAR: the stall of Algorithm 1, after which the caller
 * inserts the true token).  Nothing waits for the host between verification and pruning (Sec. 3.4, "Input
 * more than one tree-level", names GPU-CPU synchronisation as what makes verification of several levels
 * slow); the call also queues a copy of the nodes to pinned host memory, and the library's host-side view of
 * these requests (prefix_len, n_live, parents; the pages they hold) catches up at the next call that names
 * one of them, which waits for that copy if it has not arrived.  The verified nodes must have been forwarded
 * at this stage (as they have when verification follows their forward).  Not for use under stream capture.
 * Errors: SP_E_BAD_REQ, SP_E_PENDING, SP_E_INVALID (repeated request, stride not 1 or 2). */
int sp_tree_prune_verified(sp_stage* stage, int32_t n, const int32_t* req_ids /*host*/,
                           const int32_t* nodes_dev /*device*/, int32_t stride, sp_stream stream);

/* Lossy verification (Sec. 3.4, "Lossless and Lossy Acceleration").  x_root [n][d_model]
 * (device, the stage's dtype) holds, for each listed request, the last decoder layer's output of
 * the node that is now the root (the caller keeps that row of sp_stage_forward's x_out from the
 * call that forwarded the node).  The large model's distribution after the root is
 * softmax(RMSNorm(x_root) W_vocab^T); candidates are the root's children.
 *   SP_VERIFY_RELAXED: the child whose token has the highest probability (the first such child);
 *                      -1 only if the root has no child with a token inside the vocabulary.
 *   SP_VERIFY_TOP_P:   children whose token is in the top-p set (tokens in descending probability,
 *                      equal ones by ascending id, up to and including the one at which the running
 *                      sum reaches top_p, 0 < top_p <= 1) are acceptable; of those the child with the
 *                      highest draft probability (the first such child), -1 if none is acceptable.
 * result_dev (device, 2n ints): [2i] = the verified node of req_ids[i] or -1, [2i+1] = the model's
 * top-1 token, which is also stored as the root's prediction (so a miss continues as in the
 * lossless flow: SP_CLEAR, then an insert of that token).  If result_host != NULL the 2n ints are
 * also copied there asynchronously on `stream`.  The probabilities are formed in float32; a child
 * whose cumulative mass lies within rounding of top_p may fall on either side.
 * Errors: SP_E_INVALID (mode, top_p, repeated request), SP_E_BAD_REQ, SP_E_PENDING,
 * SP_E_CAPACITY (n rows of vocab logits plus scratch exceed the workspace). */
typedef enum sp_verify_mode { SP_VERIFY_RELAXED = 1, SP_VERIFY_TOP_P = 2 } sp_verify_mode;
int sp_stage_verify_lossy(sp_stage* stage, const sp_head_weights* head, int32_t n, const int32_t* req_ids /*host*/,
                          const void* x_root /*device*/, int32_t mode, float top_p, int32_t* result_dev /*device*/,
                          int32_t* result_host /*host, nullable*/, sp_stream stream);

/* Stochastic verification (Sec. 4.3, "Stochastic Decoding": temperature 0.6, candidates collected until
 * their probabilities reach 0.9 or 80 have been taken).  x_root as for sp_stage_verify_lossy.  The token
 * after the root of req_ids[i] is drawn from softmax(RMSNorm(x_root[i]) W_vocab^T / temperature): candidates
 * in descending probability (equal ones by ascending id) up to and including the one at which the running
 * sum reaches top_p, at most top_k (<= SP_MAX_SAMPLE_TOP_K) of them; with C_j the running sums over the
 * m candidates, candidate j is drawn iff C_(j-1) <= u[i] * C_m < C_j, u[i] in [0, 1) supplied by the caller
 * (host array: the library draws no random numbers).  The drawn token takes the place of the top-1 token:
 * result_dev[2i] = the first child of the root that carries it, -1 if none does (a stall, continue as in the
 * lossless flow), result_dev[2i+1] = the token, which is also stored as the root's prediction.
 * Probabilities and running sums are float32; a draw within rounding of a boundary may fall on either side.
 * Errors: SP_E_INVALID (temperature <= 0, top_p outside (0, 1], top_k outside [1, SP_MAX_SAMPLE_TOP_K], u
 * outside [0, 1), repeated request), SP_E_BAD_REQ, SP_E_PENDING, SP_E_CAPACITY (n rows of logits exceed the
 * workspace). */
#define SP_MAX_SAMPLE_TOP_K 128
int sp_stage_verify_sample(sp_stage* stage, const sp_head_weights* head, int32_t n, const int32_t* req_ids /*host*/,
                           const void* x_root /*device*/, float temperature, float top_p, int32_t top_k,
                           const float* u /*host, n*/, int32_t* result_dev /*device, 2n*/,
                           int32_t* result_host /*host, nullable*/, sp_stream stream);

/* ---- inspection ------------------------------------------------------------- */

/* Copies a request's device tables to the host.  Waits for `stream`. */
int sp_tree_read(sp_stage* stage, int32_t req, sp_tree_view* out /*host*/, sp_stream stream);

/* Host mirror of a request's counters; no GPU access. */
int sp_request_info(const sp_stage* stage, int32_t req, int32_t* prefix_len, int32_t* n_live,
                    int32_t* n_forwarded);

/* Per-kernel timing.  After sp_profile_begin(kind), every launch of that kernel
 * kind is bracketed by HIP events on its stream (at most max_launches of them);
 * sp_profile_end waits for the last event and returns the launch count and the sum
 * of their durations. */
typedef enum sp_kernel_kind {
  SP_K_NONE = 0, SP_K_GEMM_QKV = 1, SP_K_GEMM_O = 2, SP_K_GEMM_GATEUP = 3, SP_K_GEMM_DOWN = 4,
  SP_K_ATTENTION = 5, SP_K_ATTENTION_MERGE = 6, SP_K_KV_COMPACT = 7, SP_K_TREE_PRUNE = 8,
  SP_K_TREE_INSERT = 9, SP_K_NORM = 10, SP_K_ROPE_KV = 11, SP_K_VERIFY_HEAD = 12, SP_K_KIND_COUNT = 13
} sp_kernel_kind;
int sp_profile_begin(sp_stage* stage, int32_t kind, int32_t max_launches);
/* After sp_profile_begin: sample.  Launches of that kind inside sp_stage_forward are taken
 * call by call: every `every`-th call has all its launches of the kind bracketed, the other
 * calls none (outside sp_stage_forward: one launch in `every`).  The events open a gap of a
 * few microseconds around the launch they bracket and keep the call from replaying its
 * graph, so a timed run samples instead of bracketing every launch. */
int sp_profile_sample_every(sp_stage* stage, int32_t every);
int sp_profile_end(sp_stage* stage, int32_t* n_launches, float* total_ms);

const char* sp_strerror(int status);
int sp_version(void);
int sp_last_hip_error(const sp_stage* stage);

#ifdef __cplusplus
}
#endif
#endif /* SPECPIPE_H */
