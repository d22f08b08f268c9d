// Shared device-side definitions of the SpecPipe stage library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define SP_T 256          // tree capacity per request (== SP_MAX_TREE_NODES)
#define SP_W 4            // 64-bit words per ancestor-bitmask row
#define SP_BATCH 64       // requests per batched call (== SP_MAX_BATCH_REQ)

typedef uint16_t bf16_t;  // raw bfloat16 bits

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(8))) unsigned short u16x8_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;   // a 16-byte register quad

// ---- per-request device state -------------------------------------------------
// Counters of a request.  Written by the request-init, insert and prune kernels,
// read by the forward kernels; the host keeps a mirror only to validate arguments
// and to size launches.
struct ReqMeta {
  long long base;   // first cache slot of the request
  int cap;          // slots it owns
  int P;            // committed tokens (root included)
  int T;            // live speculative nodes
  int root_pred;    // the model's token after the committed context, -1 while unknown
};

// Tree tables of a request (Sec. 3.2: I, P, M) plus the map the last prune left
// for the cache compaction.  anc[i] holds row i of M as a bitmask: bit j set iff
// j == i or node j is an ancestor of node i.
struct ReqTables {
  int parent[SP_T];
  int depth[SP_T];
  int token[SP_T];
  float prob[SP_T];
  int pred[SP_T];         // the model's next token after the node, -1 until the last stage has seen it
  unsigned long long anc[SP_T][SP_W];
  // pending compaction: cache rows [0, n_kv_keep) of the tree region take the rows
  // of old nodes kv_src[0..n_kv_keep); rows below first_moved stay where they are.
  int pend_n_kv_keep;
  int pend_first_moved;
  int pend_P_old;
  int pend_T_old;
  short kv_src[SP_T];
  short tab_new[SP_T];    // old node -> new node index, -1 if it left the tables
};

// One row of a forward call.
struct RowInfo {
  long long base;   // request's first slot
  int req;
  int node;
  int pos;          // sequence position = P + depth
  int P;
  int T;
  int seg;          // index of the request inside the call
};

// A forward call's requests, passed to kernels by value.
struct FwdBatch {
  int n_req;
  int n_rows;
  int req[SP_BATCH];
  int first[SP_BATCH];
  int n[SP_BATCH];
  int row0[SP_BATCH];
};

// Arguments of one insert launch, passed by value: up to SP_T new nodes spread over up to
// SP_BATCH requests; request i owns entries [row0[i], row0[i+1]) and appends them after its
// t0[i] live nodes, in cache slots first_slot[i]...
struct InsertArgs {
  int n_req;
  short req[SP_BATCH];
  short t0[SP_BATCH];
  short row0[SP_BATCH + 1];
  long long first_slot[SP_BATCH];   // base + prefix_len + t0 (logical slot prefix_len + t0 when paged)
  short parent[SP_T];
  int token[SP_T];
  float prob[SP_T];
};

struct PruneBatch {
  int n;
  int req[SP_BATCH];
  int mode[SP_BATCH];    // <0: skip
  int node[SP_BATCH];
};

#define SP_SAMPLE_MAX_K 128  // most candidates of a stochastic verification (== SP_MAX_SAMPLE_TOP_K)
#define SP_EXPAND_MAX 4096   // candidates of one fixed-width expansion (bottom tokens x k)

struct ExpandArgs {      // by value
  int req;
  int n_bottom;
  int k;
  int w;
  short bottom[SP_T];    // node whose children are proposed, ascending; -1 = the root (empty tree)
};

struct RowList {         // source rows of an in-place row compaction, by value
  int n_keep;
  int first_moved;
  short src[SP_T];
};

// ---- bf16 <-> f32 ---------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// round-to-nearest-even in hardware (v_cvt_pk_bf16_f32)
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// max / sum over the four lanes l, l^16, l^32, l^48 (the lanes that share an MFMA column)
__device__ __forceinline__ float quad_rows_max(float v) {
  auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float quad_rows_sum(float v) {
  auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

template <typename T> struct Elt;
template <> struct Elt<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elt<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
