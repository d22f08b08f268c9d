// Tree tables on the device: layer appending, prune flags + prefix sums + table
// compaction, and the in-place row gather that compacts the KV cache and the
// in-flight hidden rows.  (Sec. 3.2; Sec. 3.3.2 "pruning propagation"; Algorithm 1
// lines 5-7.)
#include "sp_launch.h"

// 256-bit rows live in four registers; select the word without indexing memory.
__device__ __forceinline__ void set_bit(unsigned long long (&b)[SP_W], int idx) {
#pragma unroll
  for (int w = 0; w < SP_W; ++w) b[w] |= ((idx >> 6) == w) ? (1ull << (idx & 63)) : 0ull;
}
__device__ __forceinline__ bool test_bit(const unsigned long long (&b)[SP_W], int idx) {
  unsigned long long word = 0ull;
#pragma unroll
  for (int w = 0; w < SP_W; ++w) word = ((idx >> 6) == w) ? b[w] : word;
  return (word >> (idx & 63)) & 1ull;
}

// -----------------------------------------------------------------------------
__global__ void k_tables_clear(ReqMeta* meta, ReqTables* tables, int n_req) {
  int r = blockIdx.x;
  if (r >= n_req) return;
  ReqTables& t = tables[r];
  for (int i = threadIdx.x; i < SP_T; i += blockDim.x) {
    t.parent[i] = -1; t.depth[i] = 0; t.token[i] = 0; t.prob[i] = 0.f; t.pred[i] = -1;
    for (int w = 0; w < SP_W; ++w) t.anc[i][w] = 0ull;
    t.kv_src[i] = 0; t.tab_new[i] = -1;
  }
  if (threadIdx.x == 0) {
    t.pend_n_kv_keep = 0; t.pend_first_moved = 0; t.pend_P_old = 0; t.pend_T_old = 0;
    ReqMeta m; m.base = 0; m.cap = 0; m.P = 0; m.T = 0; m.root_pred = -1;
    meta[r] = m;
  }
}

__global__ void k_request_init(ReqMeta* meta, ReqTables* tables, int req, long long base, int cap, int P) {
  if (threadIdx.x == 0) {
    ReqMeta m; m.base = base; m.cap = cap; m.P = P; m.T = 0; m.root_pred = -1;
    meta[req] = m;
    ReqTables& t = tables[req];
    t.pend_n_kv_keep = 0; t.pend_first_moved = 0; t.pend_P_old = P; t.pend_T_old = 0;
  }
}

// Layer appending for the requests of a call (blockIdx.y).  Block x = 0: thread k owns the
// request's new node T0+k.  Its ancestor row is its own bit, the bits of the parents it
// reaches inside this call, and the stored row of the first parent that existed before the
// call (nothing if it reaches the root).  Blocks x = 1..: one per (layer, K|V, head) plane;
// they clear the new nodes' cache rows, so that every slot below prefix_len + n_live always
// holds finite numbers (a masked key still enters the matrix-core product with weight zero).
__global__ void __launch_bounds__(SP_T) k_tree_insert(ReqMeta* meta, ReqTables* tables, InsertArgs a, KvGeom g) {
  const int item = blockIdx.y;
  const int req = a.req[item];
  const int r0 = a.row0[item], n_new = a.row0[item + 1] - r0;
  if (blockIdx.x > 0) {
    char* plane = g.kv + (size_t)(blockIdx.x - 1) * g.plane_bytes;
    const int u16 = g.row_bytes >> 4;
    const int n16 = n_new * u16;
    for (int i = threadIdx.x; i < n16; i += blockDim.x) {
      const int row = i / u16, u = i - row * u16;
      const size_t slot = sp_phys_slot(g, req, 0, (int)a.first_slot[item] + row);   // first_slot includes the base
      reinterpret_cast<uint4*>(plane + slot * g.row_bytes)[u] = make_uint4(0u, 0u, 0u, 0u);
    }
    return;
  }
  ReqTables& t = tables[req];
  const int T0 = a.t0[item];
  const int k = threadIdx.x;
  if (k < n_new) {
    unsigned long long bits[SP_W] = {0ull, 0ull, 0ull, 0ull};
    const int self = T0 + k;
    set_bit(bits, self);
    int cur = a.parent[r0 + k];
    int up = 0;
    while (cur >= T0) {
      set_bit(bits, cur);
      cur = a.parent[r0 + cur - T0];
      ++up;
    }
    int dep = up;
    if (cur >= 0) {
#pragma unroll
      for (int w = 0; w < SP_W; ++w) bits[w] |= t.anc[cur][w];
      dep = t.depth[cur] + up + 1;
    }
    t.parent[self] = a.parent[r0 + k];
    t.depth[self] = dep;
    t.token[self] = a.token[r0 + k];
    t.prob[self] = a.prob[r0 + k];
    t.pred[self] = -1;
#pragma unroll
    for (int w = 0; w < SP_W; ++w) t.anc[self][w] = bits[w];
  }
  if (threadIdx.x == 0) meta[req].T = T0 + n_new;
}

// Prune flags from the mask column, wave-level prefix sums (ballot + popcount,
// wave64), compacted tables written in place, and the old->new map for the cache.
// dev_nodes (nullable): the verified node of every item, left on the device by the match or the lossy
// verification kernel: node >= 0 is accepted, anything else clears the tree (a stall).
__global__ void __launch_bounds__(SP_T) k_tree_prune(ReqMeta* meta, ReqTables* tables, PruneBatch b,
                                                      const int* dev_nodes, int dev_stride) {
  const int item = blockIdx.x;
  int mode = b.mode[item];
  if (mode < 0) return;
  const int req = b.req[item];
  ReqTables& t = tables[req];
  const int T = meta[req].T;
  const int P = meta[req].P;
  int node = b.node[item];
  if (dev_nodes != nullptr) {
    node = dev_nodes[(size_t)item * dev_stride];
    mode = (node >= 0 && node < T) ? 0 : 2;
  }
  const int r = mode == 2 ? 0 : node;                // mode 2 (clear) names no node
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

  __shared__ unsigned long long s_tab[SP_W], s_kv[SP_W], s_path[SP_W];
  __shared__ short s_new[SP_T];

  if (tid < SP_W) s_path[tid] = t.anc[r][tid];
  const bool live = tid < T;
  unsigned long long my[SP_W] = {0ull, 0ull, 0ull, 0ull};
  int par = -1, dep = 0, tok = 0, prd = -1;
  float prb = 0.f;
  if (live) {
#pragma unroll
    for (int w = 0; w < SP_W; ++w) my[w] = t.anc[tid][w];
    par = t.parent[tid]; dep = t.depth[tid]; tok = t.token[tid]; prb = t.prob[tid]; prd = t.pred[tid];
  }
  __syncthreads();
  const bool in_col = live && test_bit(my, r);                               // tid is r or below r
  const bool on_path = live && ((s_path[tid >> 6] >> (tid & 63)) & 1ull);   // tid is r or above r
  bool keep_tab, keep_kv;
  if (mode == 0)      { keep_tab = in_col && tid != r; keep_kv = in_col || on_path; }
  else if (mode == 1) { keep_tab = live && !in_col;    keep_kv = keep_tab; }
  else                { keep_tab = false;              keep_kv = false; }       // clear: the root alone stays

  const unsigned long long bt = __ballot(keep_tab), bk = __ballot(keep_kv);
  if (lane == 0) { s_tab[wave] = bt; s_kv[wave] = bk; }
  __syncthreads();
  const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  int pre_tab = __popcll(bt & below), pre_kv = __popcll(bk & below);
  int n_tab = 0, n_kv = 0;
#pragma unroll
  for (int w = 0; w < SP_W; ++w) {
    const int ct = __popcll(s_tab[w]), ck = __popcll(s_kv[w]);
    if (w < wave) { pre_tab += ct; pre_kv += ck; }
    n_tab += ct; n_kv += ck;
  }
  int n_commit = 0;
  if (mode == 0) {
#pragma unroll
    for (int w = 0; w < SP_W; ++w) n_commit += __popcll(s_path[w]);
  }
  s_new[tid] = keep_tab ? (short)pre_tab : (short)-1;
  __syncthreads();     // every thread has read its old entries; the map is complete

  if (keep_tab) {
    const int np = (par >= 0 && s_new[par] >= 0) ? (int)s_new[par] : -1;
    unsigned long long nrow[SP_W] = {0ull, 0ull, 0ull, 0ull};
#pragma unroll
    for (int w = 0; w < SP_W; ++w) {
      unsigned long long bits = my[w] & s_tab[w];
      while (bits) {
        const int j = __ffsll((long long)bits) - 1;
        bits &= bits - 1;
        const int nj = s_new[w * 64 + j];
        set_bit(nrow, nj);
      }
    }
    t.parent[pre_tab] = np;
    t.depth[pre_tab] = dep - n_commit;
    t.token[pre_tab] = tok;
    t.prob[pre_tab] = prb;
    t.pred[pre_tab] = prd;
#pragma unroll
    for (int w = 0; w < SP_W; ++w) t.anc[pre_tab][w] = nrow[w];
  }
  // the accepted node is the new root: its prediction is what the next step verifies against
  if (mode == 0 && tid == r) meta[req].root_pred = prd;
  if (keep_kv) t.kv_src[pre_kv] = (short)tid;
  t.tab_new[tid] = s_new[tid];
  if (tid == 0) {
    // rows before the first dropped one keep their slot
    int first = T;
#pragma unroll
    for (int w = SP_W - 1; w >= 0; --w) {
      unsigned long long live_w = 0ull;
      const int lo = w * 64;
      if (T > lo) live_w = (T - lo >= 64) ? ~0ull : ((1ull << (T - lo)) - 1ull);
      const unsigned long long gone = live_w & ~s_kv[w];
      if (gone) first = lo + __ffsll((long long)gone) - 1;
    }
    t.pend_n_kv_keep = n_kv;
    t.pend_first_moved = first;
    t.pend_P_old = P;
    t.pend_T_old = T;
    meta[req].P = P + n_commit;
    meta[req].T = n_tab;
  }
}

// -----------------------------------------------------------------------------
// In-place stable row gather on one "stream" of rows: destination row j takes
// source row src[j] >= j.  A workgroup owns the stream.  It works through the
// destinations in ascending batches; inside a batch every source is in registers
// before the first store.  Later batches only read sources beyond the rows a batch
// writes (src[j] >= j), so no row is overwritten before it is read.
// phys (nullable): row index -> physical row of the stream (paged cache); else rows are consecutive.
template <int R>
__device__ __forceinline__ void gather_inplace(char* stream, size_t row_stride, int slice_bytes, int first,
                                               int n_keep, const short* src, const int* phys = nullptr) {
  const int U = slice_bytes >> 4;                 // 16-byte units per row slice
  const int rows_per_pass = blockDim.x / U;
  const int u = threadIdx.x % U, rr = threadIdx.x / U;
  const bool active = rr < rows_per_pass;
  // every moved row is read once and written once: both carry the non-temporal hint
  for (int b0 = first; b0 < n_keep; b0 += rows_per_pass * R) {
    u32x4_t regs[R];
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int dst = b0 + i * rows_per_pass + rr;
      const bool in = active && dst < n_keep;
      const int s = in ? (int)src[dst] : 0;
      const bool mv = in && s != dst;
      // rows that stay (or lanes without a row) read the stream's first bytes and drop them
      const size_t srow = phys ? (size_t)phys[mv ? s : 0] : (size_t)s;
      const u32x4_t v = __builtin_nontemporal_load(
          reinterpret_cast<const u32x4_t*>(stream + (mv ? srow * row_stride + (size_t)u * 16 : 0)));
      regs[i] = mv ? v : (u32x4_t){0u, 0u, 0u, 0u};
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int dst = b0 + i * rows_per_pass + rr;
      if (active && dst < n_keep) {
        const int s = src[dst];
        const size_t drow = phys ? (size_t)phys[dst] : (size_t)dst;
        if (s != dst)
          __builtin_nontemporal_store(regs[i], reinterpret_cast<u32x4_t*>(stream + drow * row_stride + (size_t)u * 16));
      }
    }
    __syncthreads();
  }
}

// Column slices of in-flight hidden rows that ride along with a cache compaction (one request):
// workgroups past the cache planes take one slice each.
struct RowsJob {
  char* rows;              // nullptr: none
  size_t row_stride;
  int n_slices, slice_bytes, last_slice_bytes;
};

__device__ __forceinline__ void rows_compact_slice(const RowsJob& j, const RowList& l, int slice, short* s_src) {
  for (int i = threadIdx.x; i < l.n_keep; i += blockDim.x) s_src[i] = l.src[i];
  __syncthreads();
  gather_inplace<16>(j.rows + (size_t)slice * j.slice_bytes, j.row_stride,
                     slice == j.n_slices - 1 ? j.last_slice_bytes : j.slice_bytes, l.first_moved, l.n_keep, s_src);
}

// grid = (layers * 2 * kv_heads [+ row slices], batch items): one workgroup per (plane, request).
template <bool WITH_ROWS>
__global__ void __launch_bounds__(256) k_kv_compact(const ReqMeta* meta, const ReqTables* tables, PruneBatch b,
                                                     KvGeom g, RowsJob rj, RowList rl) {
  __shared__ short s_src[SP_T];
  const int planes = g.n_layers * 2 * g.n_kv_heads;
  if (WITH_ROWS && (int)blockIdx.x >= planes) {
    rows_compact_slice(rj, rl, blockIdx.x - planes, s_src);
    return;
  }
  const int item = blockIdx.y;
  if (b.mode[item] < 0) return;
  const int req = b.req[item];
  const ReqTables& t = tables[req];
  __shared__ int s_phys[SP_T];
  const int n_keep = t.pend_n_kv_keep, first = t.pend_first_moved;
  for (int i = threadIdx.x; i < n_keep; i += blockDim.x) s_src[i] = t.kv_src[i];
  if (g.page_table)       // physical slot of every row of the old tree region
    for (int i = threadIdx.x; i < t.pend_T_old; i += blockDim.x) s_phys[i] = (int)sp_phys_slot(g, req, 0, t.pend_P_old + i);
  __syncthreads();
  if (first >= n_keep) return;
  const size_t plane = blockIdx.x;      // (layer*2 + kv) * n_kv_heads + head
  if (g.page_table) {
    gather_inplace<16>(g.kv + plane * g.plane_bytes, (size_t)g.row_bytes, g.row_bytes, first, n_keep, s_src, s_phys);
  } else {
    char* stream = g.kv + plane * g.plane_bytes + (size_t)(meta[req].base + t.pend_P_old) * g.row_bytes;
    gather_inplace<16>(stream, (size_t)g.row_bytes, g.row_bytes, first, n_keep, s_src);
  }
}

// ---- launchers -------------------------------------------------------------------
hipError_t sp_launch_tables_clear(ReqMeta* meta, ReqTables* tables, int n_req, hipStream_t st) {
  hipLaunchKernelGGL(k_tables_clear, dim3(n_req), dim3(256), 0, st, meta, tables, n_req);
  return hipGetLastError();
}
hipError_t sp_launch_request_init(ReqMeta* meta, ReqTables* tables, int req, long long base, int cap, int P,
                                  hipStream_t st) {
  hipLaunchKernelGGL(k_request_init, dim3(1), dim3(64), 0, st, meta, tables, req, base, cap, P);
  return hipGetLastError();
}
hipError_t sp_launch_tree_insert(ReqMeta* meta, ReqTables* tables, const InsertArgs& a, KvGeom g, hipStream_t st) {
  hipLaunchKernelGGL(k_tree_insert, dim3(1 + g.n_layers * 2 * g.n_kv_heads, a.n_req), dim3(SP_T), 0, st, meta, tables,
                     a, g);
  return hipGetLastError();
}
// -----------------------------------------------------------------------------
// Verification of the root's successor (Algorithm 1, "verify new token"; top-1 rule of
// Sec. 3.4): the verified node is the first child of the root whose token is the
// model's token after the committed context; -1 if no child carries it (pipeline stall)
// or the prediction is not known yet.  One workgroup per request, thread t = node t.
struct MatchBatch {
  int n;
  int req[SP_BATCH];
};

__global__ void __launch_bounds__(SP_T) k_tree_match(const ReqMeta* meta, const ReqTables* tables, MatchBatch b,
                                                      int* out) {
  const int item = blockIdx.x;
  const int req = b.req[item];
  const ReqTables& t = tables[req];
  const ReqMeta m = meta[req];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  __shared__ int s_first[SP_W];
  const bool hit = tid < m.T && m.root_pred >= 0 && t.parent[tid] == -1 && t.token[tid] == m.root_pred;
  const unsigned long long bal = __ballot(hit);
  if (lane == 0) s_first[wave] = bal ? wave * 64 + (__ffsll((long long)bal) - 1) : -1;
  __syncthreads();
  if (tid == 0) {
    int node = -1;
#pragma unroll
    for (int w = SP_W - 1; w >= 0; --w) if (s_first[w] >= 0) node = s_first[w];
    out[item] = node;
  }
}

__global__ void k_set_root_pred(ReqMeta* meta, int req, int token) {
  if (threadIdx.x == 0 && blockIdx.x == 0) meta[req].root_pred = token;
}

hipError_t sp_launch_tree_match(const ReqMeta* meta, const ReqTables* tables, int n, const int* reqs, int* out,
                                hipStream_t st) {
  MatchBatch b;
  b.n = n;
  for (int i = 0; i < n; ++i) b.req[i] = reqs[i];
  hipLaunchKernelGGL(k_tree_match, dim3(n), dim3(SP_T), 0, st, meta, tables, b, out);
  return hipGetLastError();
}
hipError_t sp_launch_set_root_pred(ReqMeta* meta, int req, int token, hipStream_t st) {
  hipLaunchKernelGGL(k_set_root_pred, dim3(1), dim3(64), 0, st, meta, req, token);
  return hipGetLastError();
}

// -----------------------------------------------------------------------------
// Fixed-width expansion (Sec. 3.3.3 "Fixed-width tree"): candidate c = (bottom token c / k,
// proposal c % k) has cumulative probability P[ancestors, root first] * P[bottom] * p(c),
// multiplied in that order in float32.  The w largest are kept (an earlier candidate wins a
// tie) and come out in candidate order, which is parent order (Sec. 3.2 "Layer appending").
// One workgroup of 1024 threads; a candidate's rank is the number of candidates that beat it.
__global__ void __launch_bounds__(1024) k_tree_expand(const ReqTables* tables, ExpandArgs a, const int* cand_tok,
                                                       const float* cand_prob, int* out_parent, int* out_token,
                                                       float* out_prob, int* out_count) {
  constexpr int PER = SP_EXPAND_MAX / 1024;          // candidates per thread at most
  // sort key of a candidate: probability bits (non-negative floats order like their bit patterns) above
  // the complemented index, so that one 64-bit comparison decides "beats": larger probability, or the
  // same probability and an earlier place.  0 = absent.
  __shared__ __attribute__((aligned(16))) unsigned long long s_key[SP_EXPAND_MAX];
  __shared__ unsigned char s_sel[SP_EXPAND_MAX];
  __shared__ int s_wave[16];
  __shared__ float s_prob[SP_T], s_base[SP_T];
  constexpr int EXPAND_CAND = 1024;                  // keys the short ranking can hold
  __shared__ unsigned long long s_cand[EXPAND_CAND], s_bound[16];
  __shared__ unsigned s_ncand;
  const ReqTables& t = tables[a.req];
  const int C = a.n_bottom * a.k;
  const int C16 = (C + 15) & ~15;                    // the ranking sweep reads 16 keys at a time
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  // the path product of every bottom token, once: the nodes' probabilities go to LDS first, so that the
  // walk down a path is a chain of LDS reads, not of memory round trips
  if (tid < SP_T) s_prob[tid] = t.prob[tid];
  __syncthreads();
  if (tid < a.n_bottom) {
    const int node = a.bottom[tid];
    float base = 1.f;
    if (node >= 0) {
      unsigned long long anc[SP_W];
#pragma unroll
      for (int w = 0; w < SP_W; ++w) anc[w] = t.anc[node][w];
#pragma unroll
      for (int w = 0; w < SP_W; ++w) {
        unsigned long long bits = anc[w];
        while (bits) {                              // ascending index = from the root downwards
          const int j = w * 64 + __ffsll((long long)bits) - 1;
          bits &= bits - 1;
          base = base * s_prob[j];
        }
      }
    }
    s_base[tid] = base;
  }
  __syncthreads();
  for (int c = tid; c < C16; c += 1024) {
    unsigned long long key = 0ull;
    if (c < C && cand_tok[c] >= 0) {
      const float cum = s_base[c / a.k] * cand_prob[c];
      // negative or NaN probabilities are outside the contract; they rank as absent
      key = cum >= 0.f ? ((unsigned long long)__float_as_uint(cum + 0.f) << 32) | (unsigned long long)(0xffffffffu - (unsigned)c)
                       : 0ull;
    }
    s_key[c] = key;
  }
  __syncthreads();
  // Which candidates are among the w largest.  A bound first: a wave takes the ceil(w / 16) largest of its
  // threads' best keys; those are 16 * ceil(w / 16) >= w distinct candidates, so the smallest of them (t0) is
  // at most the w-th largest key.  Only the keys >= t0 (a few more than w on spread-out probabilities) are
  // then ranked against each other.  If they do not fit the list, every key is ranked against all keys.
  const int per_rank = (C + 1023) / 1024;            // uniform: slots this launch uses
  unsigned long long mykey[PER];
  unsigned long long best = 0ull;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int c = tid + i * 1024;
    mykey[i] = c < C ? s_key[c] : 0ull;
    best = mykey[i] > best ? mykey[i] : best;
    if (c < C) s_sel[c] = 0;
  }
  {
    unsigned long long cur = best, kept = 0ull;
    const int rounds = (a.w + 15) >> 4;
    for (int r = 0; r < rounds; ++r) {
      kept = cur;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const unsigned long long other = __shfl_xor(kept, o, 64);
        kept = other > kept ? other : kept;
      }
      if (kept == 0ull) break;                        // fewer present candidates than rounds: no bound from this wave
      const unsigned long long holders = __ballot(cur == kept);     // keys are distinct: one lane
      if (lane == (int)__builtin_ctzll(holders)) cur = 0ull;
    }
    if (lane == 0) s_bound[wave] = kept;
    if (tid == 0) s_ncand = 0u;
  }
  __syncthreads();
  unsigned long long t0 = s_bound[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) t0 = s_bound[w] < t0 ? s_bound[w] : t0;
#pragma unroll
  for (int i = 0; i < PER; ++i)
    if (i < per_rank && mykey[i] != 0ull && mykey[i] >= t0) {
      const unsigned p = atomicAdd(&s_ncand, 1u);
      if (p < EXPAND_CAND) s_cand[p] = mykey[i];
    }
  __syncthreads();
  const int n_cand = (int)s_ncand;
  if (n_cand <= EXPAND_CAND) {
    for (int i = tid; i < n_cand; i += 1024) {
      const unsigned long long k = s_cand[i];
      int rank = 0;
      for (int j = 0; j < n_cand; ++j) rank += s_cand[j] > k ? 1 : 0;
      if (rank < a.w) s_sel[0xffffffffu - (unsigned)(k & 0xffffffffull)] = 1;
    }
  } else {
    // one sweep over all keys, sixteen per step so that eight LDS reads are in flight (absent keys are 0
    // and beat nobody)
    int rank[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) rank[i] = 0;
    for (int o = 0; o < C16; o += 16) {
      unsigned long long kk[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) kk[j] = s_key[o + j];
#pragma unroll
      for (int i = 0; i < PER; ++i)
        if (i < per_rank) {
#pragma unroll
          for (int j = 0; j < 16; ++j) rank[i] += kk[j] > mykey[i] ? 1 : 0;
        }
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int c = tid + i * 1024;
      if (c < C) s_sel[c] = (mykey[i] != 0ull && rank[i] < a.w) ? 1 : 0;
    }
  }
  __syncthreads();
  // ordered compaction: thread t owns candidates [t*per, (t+1)*per); exclusive scan of the counts
  const int per = (C + 1023) / 1024;
  const int lo = min(tid * per, C), hi = min(lo + per, C);
  int mine = 0;
  for (int c = lo; c < hi; ++c) mine += s_sel[c];
  int incl = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int v = __shfl_up(incl, off, 64);
    if (lane >= off) incl += v;
  }
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  int pos = incl - mine;
  for (int w = 0; w < wave; ++w) pos += s_wave[w];
  for (int c = lo; c < hi; ++c) {
    if (!s_sel[c]) continue;
    out_parent[pos] = a.bottom[c / a.k];
    out_token[pos] = cand_tok[c];
    out_prob[pos] = cand_prob[c];
    ++pos;
  }
  if (tid == 1023) *out_count = pos;
}

hipError_t sp_launch_tree_expand(const ReqTables* tables, const ExpandArgs& a, const int* cand_tok,
                                 const float* cand_prob, int* out_parent, int* out_token, float* out_prob,
                                 int* out_count, hipStream_t st) {
  hipLaunchKernelGGL(k_tree_expand, dim3(1), dim3(1024), 0, st, tables, a, cand_tok, cand_prob, out_parent, out_token,
                     out_prob, out_count);
  return hipGetLastError();
}

// Writes page ids into a request's page table (host-side allocator decisions, by value).
struct PageSet {
  int req;
  int first;       // first logical page written
  int n;
  int page[512];
};
__global__ void k_pages_set(int* page_table, int pt_stride, PageSet p) {
  for (int i = threadIdx.x; i < p.n; i += blockDim.x) page_table[(size_t)p.req * pt_stride + p.first + i] = p.page[i];
}
hipError_t sp_launch_pages_set(int* page_table, int pt_stride, int req, int first, int n, const int* pages,
                               hipStream_t st) {
  for (int done = 0; done < n; done += 512) {
    PageSet p;
    p.req = req; p.first = first + done; p.n = n - done < 512 ? n - done : 512;
    for (int i = 0; i < p.n; ++i) p.page[i] = pages[done + i];
    hipLaunchKernelGGL(k_pages_set, dim3(1), dim3(256), 0, st, page_table, pt_stride, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t sp_launch_tree_prune(ReqMeta* meta, ReqTables* tables, const PruneBatch& b, const int* dev_nodes,
                                int dev_stride, hipStream_t st) {
  hipLaunchKernelGGL(k_tree_prune, dim3(b.n), dim3(SP_T), 0, st, meta, tables, b, dev_nodes, dev_stride);
  return hipGetLastError();
}
static RowsJob rows_job(void* rows, size_t row_stride_bytes, int row_bytes) {
  // slices of 256 bytes and a last narrower one (a multiple of 16 by construction: d_model % 8 == 0)
  RowsJob j;
  j.rows = (char*)rows;
  j.row_stride = row_stride_bytes;
  j.slice_bytes = 256;
  j.n_slices = (row_bytes + 255) / 256;
  j.last_slice_bytes = row_bytes - (j.n_slices - 1) * 256;
  return j;
}
// rows != nullptr (one request only): the hidden rows are compacted by the same launch
hipError_t sp_launch_kv_compact(const ReqMeta* meta, const ReqTables* tables, const PruneBatch& b, KvGeom g,
                                void* rows, size_t row_stride_bytes, int row_bytes, const RowList* l, hipStream_t st) {
  const int planes = g.n_layers * 2 * g.n_kv_heads;
  if (rows && l && b.n == 1) {
    const RowsJob j = rows_job(rows, row_stride_bytes, row_bytes);
    hipLaunchKernelGGL(k_kv_compact<true>, dim3(planes + j.n_slices, 1), dim3(256), 0, st, meta, tables, b, g, j, *l);
  } else {
    RowsJob j;
    j.rows = nullptr; j.row_stride = 0; j.n_slices = 0; j.slice_bytes = 0; j.last_slice_bytes = 0;
    RowList none;
    none.n_keep = 0; none.first_moved = 0;
    hipLaunchKernelGGL(k_kv_compact<false>, dim3(planes, b.n), dim3(256), 0, st, meta, tables, b, g, j, none);
  }
  return hipGetLastError();
}
