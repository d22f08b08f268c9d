// Host-callable launchers of the HIP kernels.  Each enqueues on `st` and returns
// the launch status; none synchronises.
#pragma once
#include "sp_device.h"

struct KvGeom {
  char* kv;              // slab
  size_t plane_bytes;    // bytes between consecutive kv heads: kv_slots * row_bytes
  int row_bytes;         // d_head * element size
  int n_layers;
  int n_kv_heads;
  // Paged storage (SpecPipe-DB keeps its cache in pages, Sec. 4 "Implementation"): request r's
  // logical slot s lives in physical slot page_table[r * pt_stride + (s >> pg_shift)] << pg_shift
  // | (s & mask).  Null: a request owns the contiguous range that starts at its base slot.
  const int* page_table;
  int pt_stride;
  int pg_shift;
};

// Physical slot of a request's logical slot (base is the request's first slot when contiguous, 0 when paged).
__device__ __forceinline__ size_t sp_phys_slot(const KvGeom& g, int req, long long base, int lslot) {
  if (!g.page_table) return (size_t)(base + lslot);
  const int page = g.page_table[(size_t)req * g.pt_stride + (lslot >> g.pg_shift)];
  return ((size_t)page << g.pg_shift) | (size_t)(lslot & ((1 << g.pg_shift) - 1));
}

// ---- tree tables -------------------------------------------------------------
hipError_t sp_launch_tables_clear(ReqMeta* meta, ReqTables* tables, int n_req, hipStream_t st);
hipError_t sp_launch_request_init(ReqMeta* meta, ReqTables* tables, int req, long long base, int cap, int P,
                                  hipStream_t st);
// first_slot: cache slot of the first new node (host mirror: base + prefix_len + n_live)
hipError_t sp_launch_tree_insert(ReqMeta* meta, ReqTables* tables, const InsertArgs& a, KvGeom g, hipStream_t st);
// dev_nodes (nullable, device): item i accepts node dev_nodes[i * dev_stride] if it is a live node and clears
// the tree otherwise; the modes and nodes of `b` are then ignored (entries with mode < 0 are still skipped)
hipError_t sp_launch_tree_prune(ReqMeta* meta, ReqTables* tables, const PruneBatch& b, const int* dev_nodes,
                                int dev_stride, hipStream_t st);
hipError_t sp_launch_pages_set(int* page_table, int pt_stride, int req, int first, int n, const int* pages /*host*/,
                               hipStream_t st);
// out[i] (device) = verified root child of request reqs[i], or -1
hipError_t sp_launch_tree_match(const ReqMeta* meta, const ReqTables* tables, int n, const int* reqs, int* out,
                                hipStream_t st);
hipError_t sp_launch_tree_expand(const ReqTables* tables, const ExpandArgs& a, const int* cand_tok,
                                 const float* cand_prob, int* out_parent, int* out_token, float* out_prob,
                                 int* out_count, hipStream_t st);
hipError_t sp_launch_set_root_pred(ReqMeta* meta, int req, int token, hipStream_t st);

// ---- lossy verification (sp_verify.hip) -------------------------------------------
// xn = rmsnorm(x) * gain for M rows (no residual stream, no row descriptors)
hipError_t sp_launch_row_norm(int dtype, const void* x, const void* gain, void* xn, int M, int d, float eps,
                              hipStream_t st);
// floats of scratch sp_launch_verify_lossy needs for n rows of V logits
size_t sp_lossy_scratch_floats(int n, int V);
// mode 1 relaxed, 2 top-p; logits [n][V]; out[2i] = verified node of reqs[i] or -1, out[2i+1] = top-1 token
hipError_t sp_launch_verify_lossy(ReqMeta* meta, const ReqTables* tables, const float* logits, int n, const int* reqs,
                                  int V, int mode, float top_p, float* scratch, int* out, hipStream_t st);
// stochastic verification: out[2i] = verified node of reqs[i] or -1, out[2i+1] = the token drawn at u[i]
hipError_t sp_launch_verify_sample(ReqMeta* meta, const ReqTables* tables, const float* logits, int n, const int* reqs,
                                   int V, float temperature, float top_p, int top_k, const float* u /*host*/, int* out,
                                   hipStream_t st);
hipError_t sp_launch_kv_compact(const ReqMeta* meta, const ReqTables* tables, const PruneBatch& b, KvGeom g,
                                void* rows /*nullable: hidden rows of the one request, same launch*/,
                                size_t row_stride_bytes, int row_bytes, const RowList* l, hipStream_t st);

// A forward call's requests (segments) and the split of its attention work, made on the host.
struct AttnPlan {          // host-made split of a forward call's attention work
  int n_seg;
  int qt;                  // 16-row query tiles per wave: 1 or 2
  int units_total;         // partial-result units: sum over split segments of chunks * rows * n_q
  int total_items;         // sum over segments of q_blocks * chunks
  int any_split;           // some segment has more than one chunk: the merge kernel must run
  int seg_item0[SP_BATCH + 1];   // first work item of each segment
  int seg_chunks[SP_BATCH];
  int seg_clen[SP_BATCH];  // slots per chunk of the segment (multiple of 32)
  int seg_qblocks[SP_BATCH];
  int seg_unit0[SP_BATCH];
  int seg_row0[SP_BATCH];  // first row of the call that belongs to the segment
  int seg_rows[SP_BATCH];
  int seg_req[SP_BATCH];
  int seg_first[SP_BATCH]; // first node of the segment
  int seg_P[SP_BATCH];     // host mirror of prefix length and live nodes
  int seg_T[SP_BATCH];
  long long seg_base[SP_BATCH];
};

// ---- elementwise / row kernels --------------------------------------------------
// Rows enter the stage: row descriptors and rotary tables (cs: [rows][d_head], cos then sin),
// h = x, xn = rmsnorm(h) * gain.
// The segment fields of `plan` say which request and node each row belongs to; if plan_dev is given the
// whole plan is also stored there for the attention kernels of the call.
hipError_t sp_launch_enter_norm(int dtype, const void* x, const AttnPlan& plan, AttnPlan* plan_dev /*nullable*/,
                                const ReqMeta* meta, const ReqTables* tables, RowInfo* rows, float* cs, int d_head,
                                float theta, float* h, const void* gain, void* xn, int M, int d, float eps,
                                hipStream_t st);

// h += sum_s part[s]; xn = rmsnorm(h) * gain
hipError_t sp_launch_add_norm(int dtype, float* h, const float* part, int S, size_t part_stride,
                              const void* gain, void* xn, int M, int d, float eps, hipStream_t st);
// q,k rotated, v copied; q -> qbuf [M][n_q*d_head]; k,v -> slab rows
hipError_t sp_launch_rope_kv(int dtype, const float* part, int S, size_t part_stride, const RowInfo* rows,
                             const float* cs, void* qbuf, KvGeom g, int layer, int M, int n_q, int n_kv,
                             int d_head, hipStream_t st);
// top-1 token per row from per-tile (value, index) pairs or from plain logits; also written to tables[..].pred
hipError_t sp_launch_argmax_rows(bool pairs, const float* part, int n_items, const FwdBatch& b, ReqTables* tables,
                                 int* pred_out /*nullable*/, float* max_out /*nullable*/, hipStream_t st);
hipError_t sp_launch_silu_mul(int dtype, const float* gu, void* act, int M, int F, hipStream_t st);
hipError_t sp_launch_finish(int dtype, const float* h, const float* part, int S, size_t part_stride, void* out,
                            int M, int d, hipStream_t st);

// ---- GEMM: out[s][m][n] (f32) = sum over the s-th K slice of X[m][k] * W[n][k] -----
hipError_t sp_launch_gemm_simple(int dtype, const void* X, const void* W, float* out, int M, int N, int K,
                                 hipStream_t st);
// bf16 MFMA kernels.  Returns the split count used in *S_out (partials [S][M][N]).  packed: the
// weights are in MFMA fragment order (sp_launch_pack_weights).
hipError_t sp_launch_gemm_bf16(const bf16_t* X, const bf16_t* W, bool packed, float* out, int M, int N, int K,
                               int max_split, size_t part_capacity_floats, int* S_out, hipStream_t st,
                               bool resident = false);
// act[m][f] = silu(X Wg^T) * (X Wu^T), W = [gate rows ; up rows]
hipError_t sp_launch_gemm_argmax_bf16(const bf16_t* X, const bf16_t* W, bool packed, float* pairs, int M, int V, int K,
                                      size_t pair_capacity_floats, int* tiles_out, hipStream_t st);
hipError_t sp_launch_gemm_gateup_bf16(const bf16_t* X, const bf16_t* W, bool packed, bf16_t* act, int M, int F,
                                      int K, int n_cu, hipStream_t st);
// Many rows (M > 128): workgroups of 128 rows x 256 columns, weights kept in registers per wave.
// Needs N % 256 == 0 (gate/up: F % 128 == 0) and K % 64 == 0.
hipError_t sp_launch_gemm_wide(const bf16_t* X, const bf16_t* W, bool packed, float* out, int M, int N, int K,
                               int n_cu, size_t part_capacity_floats, int* S_out, hipStream_t st);
hipError_t sp_launch_gemm_wide_gateup(const bf16_t* X, const bf16_t* W, bool packed, bf16_t* act, int M, int F, int K,
                                      hipStream_t st);
// [N][K] row-major bf16 -> MFMA fragment order (N % 16 == 0, K % 32 == 0, out != in)
hipError_t sp_launch_pack_weights(const void* in, void* out, int N, int K, hipStream_t st);

// ---- tree attention -------------------------------------------------------------
hipError_t sp_launch_attn_simple(int dtype, const void* q, const RowInfo* rows, const ReqTables* tables, KvGeom g,
                                 int layer, void* out, int M, int n_q, int n_kv, int d_head, hipStream_t st);

// plan: host copy (grid sizes); plan_dev: the device copy the kernels read
hipError_t sp_launch_attn_bf16(const bf16_t* q, const ReqTables* tables, KvGeom g, int layer, const AttnPlan& plan,
                               const AttnPlan* plan_dev, float* part /*workspace*/, bf16_t* out, int M, int n_q,
                               int n_kv, int d_head, hipStream_t st);
