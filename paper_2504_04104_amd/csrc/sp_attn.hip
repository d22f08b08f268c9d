// Tree-masked attention on the matrix cores (Sec. 2.1 attention, Sec. 2.2 and 3.3.2
// tree mask), bf16, d_head = 128, grouped-query.
//
// A workgroup of eight waves owns one (request, KV head, block of query rows, chunk of
// cache slots).  Its waves cut the chunk into eight runs of 32-slot tiles; each wave
// streams the K and V rows of its run from HBM exactly once for all query rows of the
// block (the g query heads of the group times the tree nodes), keeps an online softmax,
// and the eight states are folded together through LDS.  If the request's whole cache
// range is one chunk the block's output is final; otherwise an un-normalised partial
// (running max, sum, output) is left per query row and a second kernel merges the chunks.
// The committed context is visible to every node; a tree slot is visible to a node iff its
// bit is set in the node's ancestor mask.
//
// MFMA use (v_mfma_f32_16x16x32_bf16, D[4*(l/16)+i][l%16]):
//   S^T = K Q^T : A = 16 slots x 32 d (16 B per lane, read from an LDS copy of the K tile),
//                 B = 32 d x 16 query rows (registers, loaded once).
//   O^T = V^T P^T: B = P^T is exactly the S^T registers of two 16-slot tiles (the
//                 contraction order over the 32 slots is free, so no shuffle is
//                 needed); A = V^T needs 8 slots per lane for one d, which is read
//                 from an LDS copy of the V tile, two d columns per 32-bit read.
#include "sp_launch.h"

#define DH 128
#define VS 272            // LDS row stride of the V tile in bytes (256 + 16)
#define AW 8              // waves per workgroup
#define VT_BYTES (32 * VS)

struct AttnArgs {
  const bf16_t* q;          // [M][n_q][DH]
  const ReqTables* tables;
  KvGeom g;
  int layer, n_q, n_kv;
  float* part_o;            // [units][DH], followed by [units][2] (running max, sum)
  bf16_t* out;              // [M][n_q][DH]
  const AttnPlan* plan;     // device copy of the call's plan (written by the kernel that opens the forward)
};

// STREAM: every request of the call has a single block of query rows, so each K/V row is read by one workgroup
// only; the loads then carry the non-temporal hint and the rows pass through the caches without staying.
// The K rows take the same way as the V rows: loaded as whole 256-byte rows (a load instruction covers four rows)
// into an LDS tile of the wave, from which the MFMA A fragments are read.  Loaded straight from global memory in
// A-fragment order an instruction would cover 64 bytes of each of 16 rows and every 128-byte line would be asked
// for twice: a workgroup alone on its CU streams 8 KB tiles at 48 (non-temporal) or 84 GB/s (ordinary loads) in
// whole rows against 26 or 34 GB/s in quarter rows, and the ragged batch's attention went from 78 to 68 us.
template <int QT, bool PAGED, bool STREAM>
__global__ void __launch_bounds__(64 * AW) k_attn_bf16(AttnArgs a) {
  const AttnPlan& plan = *a.plan;
  // V (and K) tiles of the eight waves; the same bytes later carry the states being folded
  // (eight waves x QT x 8 d-tiles x 64 lanes x 16 B = QT * 64 KB).
  constexpr int FOLD_BYTES = AW * QT * 8 * 64 * 16;
  constexpr int TILE_BYTES = 2 * AW * VT_BYTES;
  __shared__ __attribute__((aligned(16))) char s_v[TILE_BYTES > FOLD_BYTES ? TILE_BYTES : FOLD_BYTES];
  __shared__ float s_m[AW][QT * 16];
  __shared__ float s_l[AW][QT * 16];

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  // KV head fastest: consecutive workgroup ids go round-robin over the 8 XCDs, so all query
  // blocks and chunks of one KV head share one XCD's L2 and its K/V rows are fetched from HBM once
  const int kvh = blockIdx.x % a.n_kv;
  const int item = blockIdx.x / a.n_kv;
  // Segment 0's fields are asked for together with the segment count: a call with one request (the rule) then
  // waits for one round trip to the plan, not for two in a row.
  int sg_item0 = plan.seg_item0[0], sg_chunks = plan.seg_chunks[0], sg_rows = plan.seg_rows[0], sg_row0 = plan.seg_row0[0];
  int sg_P = plan.seg_P[0], sg_T = plan.seg_T[0], sg_clen = plan.seg_clen[0], sg_req = plan.seg_req[0];
  int sg_first = plan.seg_first[0], sg_unit0 = plan.seg_unit0[0];
  long long sg_base = plan.seg_base[0];
  const int n_seg = plan.n_seg, units_total = plan.units_total;
  int seg = 0;
  while (seg + 1 < n_seg && item >= plan.seg_item0[seg + 1]) ++seg;
  if (seg != 0) {
    sg_item0 = plan.seg_item0[seg]; sg_chunks = plan.seg_chunks[seg]; sg_rows = plan.seg_rows[seg];
    sg_row0 = plan.seg_row0[seg]; sg_P = plan.seg_P[seg]; sg_T = plan.seg_T[seg]; sg_clen = plan.seg_clen[seg];
    sg_req = plan.seg_req[seg]; sg_first = plan.seg_first[seg]; sg_unit0 = plan.seg_unit0[seg];
    sg_base = plan.seg_base[seg];
  }
  const int local = item - sg_item0;
  const int chunks = sg_chunks;
  const int qb = local / chunks, ch = local - qb * chunks;
  const int g = a.n_q / a.n_kv;
  const float inv_g = 1.f / (float)g;              // (qi + 0.5) * inv_g truncates to qi / g for these small integers
  const int seg_rows = sg_rows, row0 = sg_row0;
  const int nqrows = seg_rows * g;                 // query rows of this (request, KV head)
  const int P = sg_P, T = sg_T;
  const int span = P + T;
  const int c0 = ch * sg_clen;
  const int c1 = min(c0 + sg_clen, span);
  // this wave's run of 32-slot tiles inside [c0, c1)
  const int ntiles = (c1 - c0 + 31) >> 5;
  const int w0 = c0 + 32 * ((wave * ntiles) / AW);
  const int w1 = min(c0 + 32 * (((wave + 1) * ntiles) / AW), c1);
  const int l15 = lane & 15, kg = lane >> 4;

  // contiguous cache: the request's range starts at its base slot; paged: logical slots go through
  // the request's page table, one lookup per 32-slot tile (a tile never straddles a page)
  const size_t base_b = PAGED ? 0 : (size_t)sg_base * 256;
  const char* kplane = a.g.kv + ((size_t)(a.layer * 2 + 0) * a.n_kv + kvh) * a.g.plane_bytes + base_b;
  const char* vplane = a.g.kv + ((size_t)(a.layer * 2 + 1) * a.n_kv + kvh) * a.g.plane_bytes + base_b;
  const int* pt = PAGED ? a.g.page_table + (size_t)sg_req * a.g.pt_stride : nullptr;
  const int pg_sh = PAGED ? a.g.pg_shift : 0, pg_mask = (1 << pg_sh) - 1;
  const int page0 = PAGED ? pt[0] : 0;
#define SP_PHYS(slot, pg) (PAGED ? (((slot) < span ? (pg) : page0) << pg_sh | ((slot) < span ? ((slot) & pg_mask) : 0)) \
                                 : ((slot) < span ? (slot) : 0))

  // Loads of one 32-slot tile: K and V as plain 16-byte pieces (row i*4+kg, piece l15).  Slots past
  // the request's data are read from slot 0 (always valid) and masked later.
#define SP_LOAD_TILE(S0)                                                                           \
  {                                                                                                \
    const int pg_ = PAGED ? pt[((S0) < span ? (S0) : 0) >> pg_sh] : 0;                             \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                \
      int slot = (S0) + i * 4 + kg;                                                                \
      slot = SP_PHYS(slot, pg_);                                                                   \
      const u32x4_t* vp_ = reinterpret_cast<const u32x4_t*>(vplane + (size_t)slot * 256 + l15 * 16); \
      vreg[i] = STREAM ? __builtin_nontemporal_load(vp_) : *vp_;                                   \
      const u32x4_t* kp_ = reinterpret_cast<const u32x4_t*>(kplane + (size_t)slot * 256 + l15 * 16); \
      kreg[i >> 2][i & 3] = STREAM ? __builtin_nontemporal_load(kp_) : *kp_;                       \
    }                                                                                              \
  }

  // the first tile's loads go out before anything else that has to wait
  u32x4_t kreg[2][4], vreg[8];
  char* vt = s_v + wave * VT_BYTES;
  char* kt = s_v + (AW + wave) * VT_BYTES;         // this wave's K tile, rows as in the V tile
  SP_LOAD_TILE(w0 < w1 ? w0 : span)

  // ---- query fragments and ancestor masks of this lane's query row per tile ------
  u32x4_t qf[QT][4];
  unsigned long long anc[QT][SP_W];
  const ReqTables* tab = a.tables + sg_req;
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int qi = qb * (QT * 16) + t * 16 + l15;  // index inside (request, KV head): node_local * g + gq
    const bool ok = qi < nqrows;
    const int nl = ok ? (int)(((float)qi + 0.5f) * inv_g) : 0, gq = ok ? qi - nl * g : 0;
    const bf16_t* qp = a.q + ((size_t)(row0 + nl) * a.n_q + (size_t)kvh * g + gq) * DH + kg * 8;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const u32x4_t v = *reinterpret_cast<const u32x4_t*>(qp + s * 32);
      qf[t][s] = ok ? v : (u32x4_t){0u, 0u, 0u, 0u};
    }
    const int node = sg_first + nl;
#pragma unroll
    for (int w = 0; w < SP_W; ++w) {
      const unsigned long long v = tab->anc[node][w];
      anc[t][w] = ok ? v : 0ull;
    }
  }

  f32x4_t o[QT][8];
  float mrun[QT], lrun[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    mrun[t] = -INFINITY; lrun[t] = 0.f;
#pragma unroll
    for (int d = 0; d < 8; ++d) o[t][d] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
  }
  const float sc = 0.08838834764831845f * 1.4426950408889634f;   // 1/sqrt(128) * log2(e)
  // mrun is the running maximum of the raw scores q.k; negm = -mrun*sc (0 while mrun is -inf),
  // so that exp2(fma(s, sc, negm)) is the softmax weight
  float negm[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) negm[t] = 0.f;

  for (int s0 = w0; s0 < w1; s0 += 32) {
    // K and V tiles -> LDS; then the next tile's loads are issued, so that they fly during
    // the score products, the softmax and the PV product (the tile after the last one
    // re-reads slot 0 and is discarded).
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4_t*>(vt + (i * 4 + kg) * VS + l15 * 16) = vreg[i];
    // K rows to the wave's K tile and back as A fragments: row l15 of each 16-slot half, 16 B at d = s*32 + kg*8
#pragma unroll
    for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4_t*>(kt + (i * 4 + kg) * VS + l15 * 16) = kreg[i >> 2][i & 3];
    __builtin_amdgcn_wave_barrier();
    // the tile is in LDS: the next tile's loads go out now and fly during everything below
    {
      const int nxt = (s0 + 32 < w1) ? s0 + 32 : span;     // span: every slot clamps to 0
      SP_LOAD_TILE(nxt)
    }
    f32x4_t sacc[QT][2];
#pragma unroll
    for (int t = 0; t < QT; ++t)
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) sacc[t][t2] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const u32x4_t kf = *reinterpret_cast<const u32x4_t*>(kt + (t2 * 16 + l15) * VS + s * 64 + kg * 16);
#pragma unroll
        for (int t = 0; t < QT; ++t)
          sacc[t][t2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(&kf),
                                                                *reinterpret_cast<const bf16x8_t*>(&qf[t][s]),
                                                                sacc[t][t2], 0, 0, 0);
      }

    const bool tail = s0 + 32 > P || s0 + 32 > w1;   // tile touches the tree region or the run's end
    uint32_t pb[QT][4];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      float sv[8];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int i = 0; i < 4; ++i) sv[t2 * 4 + i] = sacc[t][t2][i];
      if (tail) {
        // bits [n0, n0+64) of the row's 256-bit ancestor mask, n0 = first tree index of the tile
        const int n0 = s0 - P;
        unsigned long long win = 0ull;
#pragma unroll
        for (int w = 0; w < SP_W; ++w) {
          const int sh = w * 64 - n0;
          if (sh > -64 && sh < 64) win |= sh >= 0 ? (anc[t][w] << sh) : (anc[t][w] >> (-sh));
        }
        const int lim = w1 - s0, pfx = P - s0, tl = span - s0;   // offsets below: in run / committed / live
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int off = (j >> 2) * 16 + kg * 4 + (j & 3);
          const bool vis = (off < lim) & ((off < pfx) | ((off < tl) & (bool)((win >> off) & 1ull)));
          sv[j] = vis ? sv[j] : -INFINITY;
        }
      }
      float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
      // The running maximum only has to bound the scores, so it is raised (and the
      // accumulators rescaled) only when some lane of the wave sees a larger score.
      if (__builtin_amdgcn_ballot_w64(mx > mrun[t])) {
        mx = quad_rows_max(mx);
        const float mnew = fmaxf(mrun[t], mx);
        const float alpha = (mnew == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f((mrun[t] - mnew) * sc);  // 0 from -inf
        lrun[t] *= alpha;
#pragma unroll
        for (int d = 0; d < 8; ++d) o[t][d] *= alpha;
        mrun[t] = mnew;
        negm[t] = (mnew == -INFINITY) ? 0.f : -mnew * sc;
      }
      float pv[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) pv[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[j], sc, negm[t]));
      lrun[t] += ((pv[0] + pv[1]) + (pv[2] + pv[3])) + ((pv[4] + pv[5]) + (pv[6] + pv[7]));
#pragma unroll
      for (int j = 0; j < 4; ++j) pb[t][j] = pack_bf16x2(pv[2 * j], pv[2 * j + 1]);
    }

    // O^T += V^T P^T.  Lane (l15, kg) of the d-group G pair reads V[slot(kg,j)][G*32 + 2*l15 .. +1].
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int G = 0; G < 4; ++G) {
      uint32_t w[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int srow = (j >> 2) * 16 + kg * 4 + (j & 3);
        w[j] = *reinterpret_cast<const uint32_t*>(vt + srow * VS + (G * 32 + 2 * l15) * 2);
      }
      u32x4_t alo, ahi;     // low halves: column 2*l15; high halves: column 2*l15+1
      alo.x = __builtin_amdgcn_perm(w[1], w[0], 0x05040100); ahi.x = __builtin_amdgcn_perm(w[1], w[0], 0x07060302);
      alo.y = __builtin_amdgcn_perm(w[3], w[2], 0x05040100); ahi.y = __builtin_amdgcn_perm(w[3], w[2], 0x07060302);
      alo.z = __builtin_amdgcn_perm(w[5], w[4], 0x05040100); ahi.z = __builtin_amdgcn_perm(w[5], w[4], 0x07060302);
      alo.w = __builtin_amdgcn_perm(w[7], w[6], 0x05040100); ahi.w = __builtin_amdgcn_perm(w[7], w[6], 0x07060302);
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        const bf16x8_t pfrag = *reinterpret_cast<const bf16x8_t*>(&pb[t][0]);
        o[t][2 * G] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(&alo), pfrag,
                                                              o[t][2 * G], 0, 0, 0);
        o[t][2 * G + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(&ahi), pfrag,
                                                                  o[t][2 * G + 1], 0, 0, 0);
      }
    }
  }
#undef SP_LOAD_TILE
#undef SP_PHYS

  // ---- fold the eight wave states (fixed order, so results do not depend on timing) ----
  // Every wave rescales its state to the common maximum and leaves it in LDS; after one barrier the block's
  // 4 * QT pieces (query tile t, 32 output columns G) are each summed over the eight waves and written by a
  // wave of their own.
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    lrun[t] = quad_rows_sum(lrun[t]);
    mrun[t] = mrun[t] * sc;              // to the log2 domain (-inf stays -inf)
    if (kg == 0) s_m[wave][t * 16 + l15] = mrun[t];
  }
  __syncthreads();                       // every wave is done with its V tile; maxima are posted
  f32x4_t* fold = reinterpret_cast<f32x4_t*>(s_v);
  float mall[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    float m = -INFINITY;
#pragma unroll
    for (int w = 0; w < AW; ++w) m = fmaxf(m, s_m[w][t * 16 + l15]);
    mall[t] = m;
    const float f = (mrun[t] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mrun[t] - m);
#pragma unroll
    for (int d = 0; d < 8; ++d) fold[((wave * QT + t) * 8 + d) * 64 + lane] = o[t][d] * f;
    if (kg == 0) s_l[wave][t * 16 + l15] = lrun[t] * f;
  }
  __syncthreads();
  if (wave >= 4 * QT) return;
  const int t = wave >> 2, G = wave & 3;            // this wave's piece
  f32x4_t e0 = {0.f, 0.f, 0.f, 0.f}, e1 = {0.f, 0.f, 0.f, 0.f};   // d-tiles 2G and 2G+1
  float lsum = 0.f;
#pragma unroll
  for (int w = 0; w < AW; ++w) {
    e0 += fold[((w * QT + t) * 8 + 2 * G) * 64 + lane];
    e1 += fold[((w * QT + t) * 8 + 2 * G + 1) * 64 + lane];
    lsum += s_l[w][t * 16 + l15];
  }

  // e0[i] / e1[i] are output columns G*32 + 2*(4*kg+i) and +1 of query row t*16 + l15.
  const int qi = qb * (QT * 16) + t * 16 + l15;
  if (qi >= nqrows) return;
  const int nl = (int)(((float)qi + 0.5f) * inv_g), gq = qi - nl * g;
  const int head = kvh * g + gq;
  if (chunks == 1) {
    const float inv = 1.f / lsum;
    bf16_t* po = a.out + ((size_t)(row0 + nl) * a.n_q + head) * DH;
    u32x4_t pk;
    pk.x = pack_bf16x2(e0[0] * inv, e1[0] * inv);
    pk.y = pack_bf16x2(e0[1] * inv, e1[1] * inv);
    pk.z = pack_bf16x2(e0[2] * inv, e1[2] * inv);
    pk.w = pack_bf16x2(e0[3] * inv, e1[3] * inv);
    *reinterpret_cast<u32x4_t*>(po + G * 32 + 8 * kg) = pk;
  } else {
    const size_t unit = (size_t)sg_unit0 + (size_t)ch * seg_rows * a.n_q + (size_t)nl * a.n_q + head;
    float* po = a.part_o + unit * DH;
    f32x4_t lo, hi;
    lo[0] = e0[0]; lo[1] = e1[0]; lo[2] = e0[1]; lo[3] = e1[1];
    hi[0] = e0[2]; hi[1] = e1[2]; hi[2] = e0[3]; hi[3] = e1[3];
    *reinterpret_cast<f32x4_t*>(po + G * 32 + 8 * kg) = lo;
    *reinterpret_cast<f32x4_t*>(po + G * 32 + 8 * kg + 4) = hi;
    if (G == 0 && kg == 0) {
      float* part_ml = a.part_o + (size_t)units_total * DH;
      // the common maximum of query row t*16 + l15 (a wave-uniform choice between the two tiles' registers)
      const float m_t = (t == 0) ? mall[0] : mall[QT - 1];
      part_ml[unit * 2] = m_t; part_ml[unit * 2 + 1] = lsum;
    }
  }
}

// One wave per (row, query head) of the requests that were cut into several chunks: combine the
// chunk partials (log2-domain maxima).  Lane c first takes chunk c's (max, sum) and turns them into
// the chunk's weight; the outputs are then accumulated chunk by chunk, two columns per lane.
__global__ void __launch_bounds__(256) k_attn_merge(AttnArgs a, int M) {
  const AttnPlan& plan = *a.plan;
  int sg_chunks = plan.seg_chunks[0], sg_rows = plan.seg_rows[0], sg_unit0 = plan.seg_unit0[0], sg_row0 = plan.seg_row0[0];
  const int n_seg = plan.n_seg;
  const float* part_ml = a.part_o + (size_t)plan.units_total * DH;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int item = blockIdx.x * 4 + wave;
  if (item >= M * a.n_q) return;
  const int row = item / a.n_q, head = item - row * a.n_q;
  int seg = 0;
  while (seg + 1 < n_seg && row >= plan.seg_row0[seg + 1]) ++seg;
  if (seg != 0) {
    sg_chunks = plan.seg_chunks[seg]; sg_rows = plan.seg_rows[seg]; sg_unit0 = plan.seg_unit0[seg]; sg_row0 = plan.seg_row0[seg];
  }
  const int chunks = sg_chunks, seg_rows = sg_rows;
  if (chunks == 1) return;               // written directly by the attention kernel
  const size_t stride = (size_t)seg_rows * a.n_q;
  const size_t u0 = (size_t)sg_unit0 + (size_t)(row - sg_row0) * a.n_q + head;
  float acc0 = 0.f, acc1 = 0.f, lsum = 0.f, mx = -INFINITY;
  for (int c0 = 0; c0 < chunks; c0 += 64) {        // blocks of 64 chunks (one is the rule)
    const int c = c0 + lane;
    float m = -INFINITY, l = 0.f;
    if (c < chunks) {
      const float2 ml = *reinterpret_cast<const float2*>(part_ml + (u0 + c * stride) * 2);
      m = ml.x; l = ml.y;
    }
    const float bm = wave_max(m);
    const float nmx = fmaxf(mx, bm);
    if (nmx == -INFINITY) continue;
    const float resc = (mx == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mx - nmx);
    acc0 *= resc; acc1 *= resc; lsum *= resc;
    mx = nmx;
    const float wgt = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mx);
    lsum += wave_sum(wgt * l);
    const int nb = min(64, chunks - c0);
    int j = 0;
    // sixteen chunks' partial rows in flight at a time: the loop is a chain of memory round trips otherwise
    for (; j + 16 <= nb; j += 16) {
      float o0[16], o1[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float* po = a.part_o + (u0 + (size_t)(c0 + j + i) * stride) * DH;
        o0[i] = po[lane]; o1[i] = po[64 + lane];
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float w1 = __shfl(wgt, j + i, 64);
        acc0 += w1 * o0[i]; acc1 += w1 * o1[i];
      }
    }
    for (; j + 4 <= nb; j += 4) {
      float w4[4], o0[4], o1[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        w4[i] = __shfl(wgt, j + i, 64);
        const float* po = a.part_o + (u0 + (size_t)(c0 + j + i) * stride) * DH;
        o0[i] = po[lane]; o1[i] = po[64 + lane];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) { acc0 += w4[i] * o0[i]; acc1 += w4[i] * o1[i]; }
    }
    for (; j < nb; ++j) {
      const float w1 = __shfl(wgt, j, 64);
      const float* po = a.part_o + (u0 + (size_t)(c0 + j) * stride) * DH;
      acc0 += w1 * po[lane]; acc1 += w1 * po[64 + lane];
    }
  }
  const float inv = 1.f / lsum;
  bf16_t* po = a.out + ((size_t)row * a.n_q + head) * DH;
  po[lane] = f32_to_bf16(acc0 * inv);
  po[64 + lane] = f32_to_bf16(acc1 * inv);
}

hipError_t sp_launch_attn_bf16(const bf16_t* q, const ReqTables* tables, KvGeom g, int layer, const AttnPlan& plan,
                               const AttnPlan* plan_dev, float* part, bf16_t* out, int M, int n_q, int n_kv,
                               int d_head, hipStream_t st) {
  if (d_head != DH || g.row_bytes != 256) return hipErrorInvalidValue;
  AttnArgs a;
  a.q = q; a.tables = tables; a.g = g; a.layer = layer; a.n_q = n_q; a.n_kv = n_kv;
  a.part_o = part;
  a.out = out;
  a.plan = plan_dev;
  dim3 grid(plan.total_items * n_kv);
  bool stream = true;                     // one block of query rows per request: K/V rows are read once
  for (int i = 0; i < plan.n_seg; ++i) stream = stream && plan.seg_qblocks[i] <= 1;
#define SP_ATTN_GO(QTV, PG, STR) hipLaunchKernelGGL((k_attn_bf16<QTV, PG, STR>), grid, dim3(64 * AW), 0, st, a)
#define SP_ATTN_QT(QTV)                                                              \
  if (g.page_table) { if (stream) SP_ATTN_GO(QTV, true, true); else SP_ATTN_GO(QTV, true, false); }   \
  else { if (stream) SP_ATTN_GO(QTV, false, true); else SP_ATTN_GO(QTV, false, false); }
  switch (plan.qt) {
    case 1: SP_ATTN_QT(1) break;
    case 2: SP_ATTN_QT(2) break;
    default: return hipErrorInvalidValue;
  }
#undef SP_ATTN_QT
#undef SP_ATTN_GO
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !plan.any_split) return e;
  hipLaunchKernelGGL(k_attn_merge, dim3((M * n_q + 3) / 4), dim3(256), 0, st, a, M);
  return hipGetLastError();
}
