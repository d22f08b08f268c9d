// bf16 projections for few rows (M = tree nodes in flight, typically <= 64) on the
// CDNA4 matrix cores.  With so few rows every weight is used once, so the kernel is a
// weight streamer (decode is bound by loading parameters, Sec. 2.2): each wave pulls
// its 16 weight rows straight from HBM into registers in MFMA operand layout (one
// 16-byte load per lane per k-step, PF chunks ahead of the math), while the M x K
// activation panel -- shared by every wave -- is staged once per workgroup through LDS.
// Up to 16 rows a workgroup is four waves over 64 columns (the panel is small, more workgroups
// stream better); from 17 rows on it is eight waves over 128 columns, or over the CU's even share
// of the gate/up columns, one workgroup per CU, because the panel's way from L2 into the CU is
// then what the rows cost.  The weights carry the non-temporal hint.
//
//   out[y][m][n] = sum_{k in slice y} X[m][k] * W[n][k]        (f32 partial sums)
//
// v_mfma_f32_16x16x32_bf16: A = 16 weight rows x 32 k (lane l: row l%16, k (l/16)*8..+8),
// B = 32 k x 16 activation rows (lane l: row l%16, same k), D[4*(l/16)+i][l%16].
#include "sp_launch.h"

// Tunables (defaults chosen by measurement on MI355X).
#ifndef SP_GEMM_KC_PLAIN
#define SP_GEMM_KC_PLAIN 128      // k per staged chunk (smaller LDS panel: three workgroups per CU)
#endif
#ifndef SP_GEMM_KC_GATEUP
#define SP_GEMM_KC_GATEUP 256
#endif
#ifndef SP_GEMM_PF
#define SP_GEMM_PF 2              // weight chunks in flight ahead of the math
#endif
// Workgroup shapes from 17 rows on, each measured against the four-wave 64-column workgroup it replaces (1 = on):
#ifndef SP_GEMM_PLAIN8
#define SP_GEMM_PLAIN8 1          // plain products, 17-64 rows: eight waves over 128 columns, one workgroup per CU
#endif
#ifndef SP_GEMM_PLAIN8_MT8
#define SP_GEMM_PLAIN8_MT8 1      // ... and at 65-128 rows (small matrices; the large ones take two strips per wave)
#endif
#ifndef SP_GEMM_PLAIN6
#define SP_GEMM_PLAIN6 1          // ... six waves over 96 columns where that divides the CUs evenly and 128 do not
#endif
#ifndef SP_GEMM_ARGMAX8
#define SP_GEMM_ARGMAX8 1         // the output head's top-column kernel in the eight-wave shape
#endif
#ifndef SP_GEMM_EVEN7
#define SP_GEMM_EVEN7 1           // gate/up, one workgroup per CU over 96 < d_ff / CUs <= 112 columns (seven waves)
#endif
#ifndef SP_GEMM_EVEN_MT8
#define SP_GEMM_EVEN_MT8 1        // gate/up, one workgroup per CU, also at 65-128 rows
#endif
#ifndef SP_GEMM_PF_EVEN
#define SP_GEMM_PF_EVEN 3         // the eight-wave gate/up kernel has the registers for a third chunk (45.5 -> 44.9 us)
#endif
#ifndef SP_GEMM_PF_EIGHT
#define SP_GEMM_PF_EIGHT SP_GEMM_PF   // the eight-wave plain kernels are faster with two
#endif
#ifndef SP_GEMM_EVEN_MIN_MT
#define SP_GEMM_EVEN_MIN_MT 2     // row tiles from which gate/up takes one workgroup per CU where d_ff allows
#endif
#ifndef SP_GEMM_NCG_PLAIN
#define SP_GEMM_NCG_PLAIN 4       // column groups (of 16 weight rows) per workgroup
#endif
#ifndef SP_GEMM_NCG_GATEUP
#define SP_GEMM_NCG_GATEUP 2
#endif
#ifndef SP_GEMM_ROWSTORE
#define SP_GEMM_ROWSTORE 1        // split-K partial sums written in whole rows through LDS ...
#endif
#ifndef SP_GEMM_ROWSTORE_MIN_MT
#define SP_GEMM_ROWSTORE_MIN_MT 8 // ... from this many row tiles
#endif
#ifndef SP_GEMM_ROT
// Plain products split over k, K up to 8192 (the QKV and O shapes): workgroups walk their k slice from
// different starting chunks.  At 1-16 rows: 6144 x 4096 12.3 -> 10.3 us, 8192 x 8192 25.2 -> 23.2 us,
// 10240 x 8192 33.2 -> 32.2 us, 4096 x 4096 unchanged; at 32 and 64 rows 8192 x 8192 29.2 -> 24.8 and
// 31.0 -> 27.9 us, the other shapes within 1 %; with K = 14336 or 28672 (down) 2-3 % slower at 1-16 rows,
// and nothing gained in gate/up: those keep the plain order.
#define SP_GEMM_ROT 1
#endif
#ifndef SP_GEMM_TARGET_WGS
#define SP_GEMM_TARGET_WGS 768    // one row tile: split K until the grid has about this many workgroups
#endif
#ifndef SP_GEMM_TARGET_WGS_ROWS
#define SP_GEMM_TARGET_WGS_ROWS 512   // more row tiles: at most this many (two per CU)
#endif

// PACKED: the weights were re-laid at load time (sp_pack_weights) into MFMA fragment order --
// per strip of 16 rows, one contiguous 1 KB block per k-step of 32, lane-major -- so that every
// wave load is one contiguous kilobyte instead of sixteen 64-byte pieces.
// ARGMAX (output head of the last stage, Algorithm 1 "verify new token"): instead of the
// products, a workgroup leaves per row the largest of its 16*NCG columns and that column's
// index (the lowest one among equal maxima) as a (float, int) pair at out[(m * tiles + tile) * 2].
// TWO (plain products only): a wave holds two strips of 16 weight rows, 64 rows apart, so that a workgroup
// covers 32*NCG columns: with 128 activation rows the staged panel would otherwise be twice the size of the
// weights it meets, and the reads of the panel out of L2, not HBM, would set the pace.
// EVEN (gate/up): one workgroup per CU covers cpw = d_ff / CUs activation columns, a multiple of 8, in NCG column
// groups of 16 columns and a last one of cpw - 16 * (NCG - 1) -- eight waves as four groups times two k-halves for
// 48 < cpw <= 64, seven waves as seven groups for 96 < cpw <= 112 (the upper lanes of a short last group re-read
// its last row and their results are dropped; 8 rows of the fragment layout are one 128-byte line, so nothing is
// fetched twice).  Every CU then streams the same bytes, which 16-row
// strips in fixed 32-column workgroups cannot do when d_ff / 32 is not a multiple of the CU count (d_ff = 14336:
// 1.75 workgroups per CU), and the panel is staged once per CU instead of once per four waves.
template <int MT, int NCG, bool GATEUP, int KC, int PF, bool PACKED, bool ARGMAX = false, bool TWO = false,
          int NWAVES = 4, bool EVEN = false, bool WNT = true>
__global__ void __launch_bounds__(64 * NWAVES)
k_gemm_bf16(const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, float* __restrict__ out,
            bf16_t* __restrict__ act, int M, int N, int K, int chunks_total, int S, int cpw = 0, int rot = 0) {
  static_assert(!(TWO && (GATEUP || ARGMAX)), "two strips per wave: plain products only");
  static_assert(!EVEN || GATEUP, "even split: gate/up only");
  constexpr int NTH = 64 * NWAVES;
  constexpr int NKH = NWAVES / NCG;       // waves sharing a column group split each chunk's k-steps
  constexpr int KSTEPS = (KC / 32) / NKH;
  constexpr int NW = (GATEUP || TWO) ? 2 : 1;
  constexpr int ROWS = MT * 16;
  constexpr int XS = KC * 2 + 16;         // LDS row stride in bytes (conflict-free 16-byte reads)
  constexpr int UPR = KC / 8;             // 16-byte units per X row chunk
  constexpr int RPP = NTH / UPR;          // rows per staging pass
  constexpr int PASSES = (ROWS + RPP - 1) / RPP;   // the last pass may cover fewer rows (48 rows, 32 per pass)
  constexpr bool RAGGED_PASS = ROWS % RPP != 0;
  constexpr int NB = PF + 1;              // weight register buffers
  __shared__ __attribute__((aligned(16))) char lds[2][ROWS * XS];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int cg = wave % NCG, kh = wave / NCG;
  const int r = lane & 15, kg = lane >> 4;
  const int n0 = EVEN ? blockIdx.x * cpw + cg * 16 : blockIdx.x * (16 * NCG * (TWO ? 2 : 1)) + cg * 16;
  const int vr = EVEN ? min(16, cpw - cg * 16) : 16;     // valid columns of this wave's group (8 or 16)
  const int pair_off = TWO ? 16 * NCG : N;   // rows between a wave's two strips (gate/up: the up rows follow the N gate rows)
  const int m_base = blockIdx.z * ROWS;
  const int c_begin = (int)(((long long)blockIdx.y * chunks_total) / S);
  const int c_end = (int)(((long long)(blockIdx.y + 1) * chunks_total) / S);

  // EVEN: a group starts at a multiple of 8, so its 16 rows may lie in two fragment blocks: per-lane row addresses
  const int wr0 = n0 + min(r, vr - 1), wr1 = pair_off + wr0;
  const bf16_t* w0 =
      EVEN ? (PACKED ? W + ((size_t)(wr0 >> 4) * (K / 32) + kh * KSTEPS) * 512 + (kg * 16 + (wr0 & 15)) * 8
                     : W + (size_t)wr0 * K + kg * 8 + kh * (KSTEPS * 32))
           : (PACKED ? W + ((size_t)(n0 / 16) * (K / 32) + kh * KSTEPS) * 512 + lane * 8
                     : W + (size_t)(n0 + r) * K + kg * 8 + kh * (KSTEPS * 32));
  const bf16_t* w1 =                                                                                // second strip
      EVEN ? (PACKED ? W + ((size_t)(wr1 >> 4) * (K / 32) + kh * KSTEPS) * 512 + (kg * 16 + (wr1 & 15)) * 8
                     : W + (size_t)wr1 * K + kg * 8 + kh * (KSTEPS * 32))
           : (PACKED ? W + ((size_t)((pair_off + n0) / 16) * (K / 32) + kh * KSTEPS) * 512 + lane * 8
                     : W + (size_t)(pair_off + n0 + r) * K + kg * 8 + kh * (KSTEPS * 32));
#define SP_WOFF(C, s) (PACKED ? ((size_t)(C) * (KC / 32) + (s)) * 512 : (size_t)(C)*KC + (s) * 32)
  // rot: workgroups start at different chunks of their k slice and wrap around, so that the workgroups of one
  // slice, whose weight rows lie a fixed distance apart, are not all at the same offset of their rows at the
  // same moment (the start moves with id / 8; id, id / 2, id / 4 and id / 16 measured worse).  The sum over k
  // is then taken in a different, still fixed, order per workgroup.
  const int c_n = c_end - c_begin;
  const int c_rot = rot && c_n > 1 ? (int)((blockIdx.x >> 3) % (unsigned)c_n) : 0;
#define SP_PC(C) ((C) + c_rot < c_end ? (C) + c_rot : (C) + c_rot - c_n)
  const int xu = tid % UPR, xr = tid / UPR;
  // rows past M are read from the last valid row and multiply into output rows that are never stored
  const int m_last = M - 1;

  u32x4_t wb[NB][NW][KSTEPS];
  u32x4_t xnxt[PASSES];
  f32x4_t acc[NW][MT];
#pragma unroll
  for (int a = 0; a < NW; ++a)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[a][mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

#define SP_LOAD_X(C)                                                                                   \
  _Pragma("unroll") for (int p = 0; p < PASSES; ++p) {                                                  \
    const int m = min(m_base + p * RPP + xr, m_last);                                                   \
    xnxt[p] = *reinterpret_cast<const u32x4_t*>(X + (size_t)m * K + (size_t)SP_PC(C) * KC + xu * 8);     \
  }
#define SP_STORE_X(BUF)                                                                                 \
  _Pragma("unroll") for (int p = 0; p < PASSES; ++p)                                                    \
      if (!RAGGED_PASS || p * RPP + xr < ROWS)                                                          \
        *reinterpret_cast<u32x4_t*>(&lds[BUF][(p * RPP + xr) * XS + xu * 16]) = xnxt[p];
  // Every weight is read once per launch: the loads carry the non-temporal hint (WNT), so the stream does not
  // push the activation panel (which every workgroup re-reads) out of L2 nor fill the Infinity Cache
  // (gate/up at 8 rows: 43.4 -> 38.8 us, at 64 rows: 50.7 -> 49.5 us).  The exception is a matrix the caller
  // wants to find in the Infinity Cache again at the next step: ordinary loads.
#define SP_LOAD_W(B, C)                                                                                 \
  _Pragma("unroll") for (int s = 0; s < KSTEPS; ++s) {                                                  \
    const int pc_ = SP_PC(C);                                                                           \
    wb[B][0][s] = WNT ? __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(w0 + SP_WOFF(pc_, s))) \
                      : *reinterpret_cast<const u32x4_t*>(w0 + SP_WOFF(pc_, s));                         \
    if (NW == 2)                                                                                        \
      wb[B][NW - 1][s] = WNT ? __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(w1 + SP_WOFF(pc_, s))) \
                             : *reinterpret_cast<const u32x4_t*>(w1 + SP_WOFF(pc_, s));                  \
  }
  // One chunk C out of weight buffer B.  The activation panel of chunk C+1 was loaded to
  // registers one chunk earlier and goes to the other LDS buffer first; then the loads of
  // panel C+2 and of weight chunk C+PF are issued, and chunk C is multiplied.  A wave only
  // ever waits for loads that have had a whole chunk of math to arrive, and never for the
  // youngest weight loads (waits retire loads in issue order).
#define SP_CHUNK(B, C)                                                                                  \
  {                                                                                                     \
    const int c_ = (C);                                                                                 \
    const int buf = (c_ - c_begin) & 1;                                                                 \
    if (c_ + 1 < c_end) { SP_STORE_X(buf ^ 1) }                                                         \
    if (c_ + 2 < c_end) { SP_LOAD_X(c_ + 2) }                                                           \
    if (c_ + PF < c_end) { SP_LOAD_W((B + PF) % NB, c_ + PF) }                                          \
    _Pragma("unroll") for (int s = 0; s < KSTEPS; ++s) {                                                \
      _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) {                                               \
        const bf16x8_t b = *reinterpret_cast<const bf16x8_t*>(                                          \
            &lds[buf][(mt * 16 + r) * XS + ((kh * KSTEPS + s) * 32 + kg * 8) * 2]);                     \
        _Pragma("unroll") for (int a = 0; a < NW; ++a) acc[a][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16( \
            *reinterpret_cast<const bf16x8_t*>(&wb[B][a][s]), b, acc[a][mt], 0, 0, 0);                  \
      }                                                                                                 \
    }                                                                                                   \
    __syncthreads();                                                                                    \
  }

  if (c_begin < c_end) {
    SP_LOAD_X(c_begin)
    SP_LOAD_W(0, c_begin)
    if (PF >= 2 && c_begin + 1 < c_end) { SP_LOAD_W(1 % NB, c_begin + 1) }
    if (PF >= 3 && c_begin + 2 < c_end) { SP_LOAD_W(2 % NB, c_begin + 2) }
    SP_STORE_X(0)
    if (c_begin + 1 < c_end) { SP_LOAD_X(c_begin + 1) }
  }
  __syncthreads();
  for (int c = c_begin; c < c_end; c += NB) {
    SP_CHUNK(0, c)
    if (NB >= 2 && c + 1 < c_end) SP_CHUNK(1 % NB, c + 1)
    if (NB >= 3 && c + 2 < c_end) SP_CHUNK(2 % NB, c + 2)
    if (NB >= 4 && c + 3 < c_end) SP_CHUNK(3 % NB, c + 3)
  }
  static_assert(PF >= 1 && PF <= 3, "weight chunks in flight");
#undef SP_CHUNK
#undef SP_LOAD_W
#undef SP_STORE_X
#undef SP_LOAD_X
#undef SP_PC
#undef SP_WOFF

  if (NKH == 2) {       // fold the two k-halves of a column group together through LDS
    float* red = reinterpret_cast<float*>(&lds[0][0]);
    if (kh == 1) {
#pragma unroll
      for (int a = 0; a < NW; ++a)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          *reinterpret_cast<f32x4_t*>(red + (((cg * NW + a) * MT + mt) * 64 + lane) * 4) = acc[a][mt];
    }
    __syncthreads();
    if (kh == 1) return;
#pragma unroll
    for (int a = 0; a < NW; ++a)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        acc[a][mt] += *reinterpret_cast<const f32x4_t*>(red + (((cg * NW + a) * MT + mt) * 64 + lane) * 4);
  }

  // lane holds, for activation row m = mt*16 + l%16, output columns n0 + 4*(l/16) + 0..3
  const int ncol = n0 + 4 * kg;
  if (EVEN && 4 * kg >= vr) return;       // columns past a short last group
  if (ARGMAX) {
    static_assert(!ARGMAX || (NKH == 1 && !GATEUP), "one wave per column group");
    float* s_val = reinterpret_cast<float*>(&lds[0][0]);          // [NCG][ROWS]; the panels are no longer read
    int* s_idx = reinterpret_cast<int*>(s_val + NCG * ROWS);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float bv = acc[0][mt][0];
      int bi = ncol;
#pragma unroll
      for (int i = 1; i < 4; ++i)
        if (acc[0][mt][i] > bv) { bv = acc[0][mt][i]; bi = ncol + i; }
#pragma unroll
      for (int off = 16; off <= 32; off <<= 1) {                  // the four lanes that hold the row
        const float ov = __shfl_xor(bv, off, 64);
        const int oi = __shfl_xor(bi, off, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
      }
      if (kg == 0) { s_val[cg * ROWS + mt * 16 + r] = bv; s_idx[cg * ROWS + mt * 16 + r] = bi; }
    }
    __syncthreads();
    const int m = m_base + tid;
    if (tid < ROWS && m < M) {
      float bv = s_val[tid];
      int bi = s_idx[tid];
#pragma unroll
      for (int c = 1; c < NCG; ++c)                               // ascending columns: ties keep the lower one
        if (s_val[c * ROWS + tid] > bv) { bv = s_val[c * ROWS + tid]; bi = s_idx[c * ROWS + tid]; }
      float* o = out + ((size_t)m * gridDim.x + blockIdx.x) * 2;
      o[0] = bv;
      reinterpret_cast<int*>(o)[1] = bi;
    }
    return;
  }
  if (SP_GEMM_ROWSTORE && !GATEUP && MT >= SP_GEMM_ROWSTORE_MIN_MT) {
    // Partial sums leave in whole rows of the workgroup's columns: the waves' 16-column pieces are put together in
    // LDS (the panels are no longer read: every wave has passed the barrier that ends its last chunk), and a store
    // instruction then writes 1 KB of consecutive addresses instead of 64 bytes in each of 16 rows.
    static_assert(NKH == 1 || GATEUP, "plain products: one wave per column group");
    constexpr int WCOLS = 16 * NCG * (TWO ? 2 : 1);
    constexpr int LSF = WCOLS + 4;                        // floats per LDS row
    static_assert(ROWS * LSF * 4 <= (int)sizeof(lds), "the row tile fits the panels' LDS");
    float* tile = reinterpret_cast<float*>(&lds[0][0]);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int a = 0; a < NW; ++a)
        *reinterpret_cast<f32x4_t*>(tile + (mt * 16 + r) * LSF + a * (16 * NCG) + cg * 16 + 4 * kg) = acc[a][mt];
    __syncthreads();
    constexpr int UPRW = WCOLS / 4;                       // 16-byte units per row
    const int col0 = blockIdx.x * WCOLS;
    for (int idx = tid; idx < ROWS * UPRW; idx += NTH) {
      const int row = idx / UPRW, u = idx - row * UPRW;
      const int m = m_base + row;
      if (m < M)
        *reinterpret_cast<f32x4_t*>(out + ((size_t)blockIdx.y * M + m) * N + col0 + u * 4) =
            *reinterpret_cast<const f32x4_t*>(tile + row * LSF + u * 4);
    }
    return;
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = m_base + mt * 16 + r;
    if (m >= M) continue;
    if (GATEUP) {
      float o[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float gte = acc[0][mt][i], up = acc[NW - 1][mt][i];
        o[i] = gte / (1.f + __expf(-gte)) * up;
      }
      uint2 pk;
      pk.x = pack_bf16x2(o[0], o[1]);
      pk.y = pack_bf16x2(o[2], o[3]);
      *reinterpret_cast<uint2*>(act + (size_t)m * N + ncol) = pk;
    } else {
      float* o = out + ((size_t)blockIdx.y * M + m) * N + ncol;
      *reinterpret_cast<f32x4_t*>(o) = acc[0][mt];
      if (TWO) *reinterpret_cast<f32x4_t*>(o + pair_off) = acc[NW - 1][mt];
    }
  }
}

// ---- launchers -------------------------------------------------------------------
// Up to 64 rows run as one block of MT = ceil(M/16) tiles; more rows run in blocks of 128 (MT = 8,
// always with the 128-wide chunk so that the two LDS panels fit), each block streaming the weights once.
// More than 64 rows (MT = 8): workgroups of twice the columns -- two strips per wave for the plain products,
// four column groups instead of two for gate/up -- so that panel and weights stay one to one.
// staggered starting chunks: plain products that are split over k, K up to 8192 (see SP_GEMM_ROT)
static inline int rot_for(int S, int K) { return (SP_GEMM_ROT && S > 1 && K <= 8192) ? 1 : 0; }

template <int NCG, bool GATEUP, int KCV, bool PACKED, bool ARGMAX = false>
static hipError_t launch_mt(int MT, dim3 grid, hipStream_t st, const bf16_t* X, const bf16_t* W, float* out,
                            bf16_t* act, int M, int N, int K, int S, bool two = false) {
#define SP_GO(MTV, KCX)                                                                                        \
  hipLaunchKernelGGL((k_gemm_bf16<MTV, NCG, GATEUP, KCX, SP_GEMM_PF, PACKED, ARGMAX>), grid, dim3(256), 0, st, X, \
                     W, out, act, M, N, K, K / KCX, S, 0, (!GATEUP && !ARGMAX) ? rot_for(S, K) : 0)
  if (!ARGMAX && MT == 4 && GATEUP && NCG == 4) {      // the 64 + 64 column gate/up workgroup at 49-64 rows
    hipLaunchKernelGGL((k_gemm_bf16<4, 4, true, 128, SP_GEMM_PF, PACKED, false>), grid, dim3(256), 0, st, X, W, out, act, M, N, K, K / 128, S);
    return hipGetLastError();
  }
  switch (MT) {
    case 1: SP_GO(1, KCV); break;
    case 2: SP_GO(2, KCV); break;
    case 3: SP_GO(3, KCV); break;
    case 4: SP_GO(4, KCV); break;
    default:
      if (ARGMAX) SP_GO(8, 128);
      else if (GATEUP && NCG == 4)
        hipLaunchKernelGGL((k_gemm_bf16<8, 4, true, 128, SP_GEMM_PF, PACKED, false>), grid, dim3(256), 0, st, X, W, out, act,
                           M, N, K, K / 128, S);
      else if (GATEUP || !two) SP_GO(8, 128);
      else
        hipLaunchKernelGGL((k_gemm_bf16<8, 4, false, 128, SP_GEMM_PF, PACKED, false, true>), grid, dim3(256), 0, st, X, W,
                           out, act, M, N, K, K / 128, S, 0, rot_for(S, K));
      break;
  }
#undef SP_GO
  return hipGetLastError();
}
// columns one workgroup covers
static inline int tile_cols(int MT, bool gateup) { return 16 * (gateup ? SP_GEMM_NCG_GATEUP : SP_GEMM_NCG_PLAIN); }

static inline void row_blocks(int M, int* MT, int* mblocks) {
  if (M <= 64) { *MT = (M + 15) / 16; *mblocks = 1; }
  else { *MT = 8; *mblocks = (M + 127) / 128; }
}

hipError_t sp_launch_gemm_bf16(const bf16_t* X, const bf16_t* W, bool packed, float* out, int M, int N, int K,
                               int max_split, size_t part_capacity_floats, int* S_out, hipStream_t st, bool resident) {
  int MT, mblocks;
  row_blocks(M, &MT, &mblocks);
  // 128-row blocks: two strips per wave (128 columns per workgroup) halve the panel traffic out of L2 (the
  // 128 x K panel is read once per column tile: N/128 instead of N/64 times) but double the split count that
  // fills the chip, i.e. the partial sums that go to memory and back.  The panel saving is N/128 * M*K*2 bytes
  // of L2 reads, the price 65536/N * M*N*4 bytes of memory traffic: worth it for the large matrices (70B
  // shape: 5.38 -> 4.78 ms per 128-node step), not for the 8B shape (65-128 rows: +3 to +6 %).
  const bool two = MT == 8 && N % 128 == 0 && (double)N * (double)K >= 64.0 * 1048576.0;
  // 17-64 rows: workgroups of eight waves over 128 columns, one per CU -- the same waves per CU as two
  // four-wave workgroups of 64 columns, but the panel slice is staged once for all eight
  const bool eight = SP_GEMM_PLAIN8 && N % 128 == 0 && ((MT >= 2 && MT <= 4) || (SP_GEMM_PLAIN8_MT8 && MT == 8 && !two && mblocks == 1));
  // ... or six waves over 96 columns where that divides the CUs evenly and 128 columns do not (N = 6144 on 256 CUs:
  // 64 tiles x 4 slices of equal length instead of 48 x 5 of 6 or 7 chunks)
  const bool six = SP_GEMM_PLAIN6 && eight && MT <= 4 && N % 96 == 0 && (SP_GEMM_TARGET_WGS_ROWS / 2) % (N / 128) != 0 &&
                   (SP_GEMM_TARGET_WGS_ROWS / 2) % (N / 96) == 0;
  const int TILE = six ? 96 : (two || eight) ? 128 : 16 * SP_GEMM_NCG_PLAIN;
  if (M < 1 || N % TILE || K % SP_GEMM_KC_PLAIN || K % 128) return hipErrorInvalidValue;
  const int chunks = K / (MT == 8 ? 128 : SP_GEMM_KC_PLAIN);
  const int tiles = N / TILE;
  // Enough workgroups to keep every CU streaming, within the partial-sum buffer.
  // With one row tile the partial sums are small and three workgroups per CU stream best.  With more
  // rows every slice costs M*N*4 bytes written here and read again by the kernel that folds them, which
  // outweighs the finer split: at most two workgroups per CU (measured on the whole 64-row step:
  // 0.608 ms against 0.617 ms; a count between two and three per CU, which leaves the CUs unevenly
  // loaded, 0.638 ms; two waves per column group with half the slices again: 0.612 ms).
  int S = MT == 1 ? (SP_GEMM_TARGET_WGS + tiles * mblocks - 1) / (tiles * mblocks)
                  : (eight ? SP_GEMM_TARGET_WGS_ROWS / 2 : SP_GEMM_TARGET_WGS_ROWS) / (tiles * mblocks);
  if (S > max_split) S = max_split;
  if (S > chunks) S = chunks;
  while (S > 1 && (size_t)S * M * N > part_capacity_floats) --S;
  if (S < 1) S = 1;
  if ((size_t)S * M * N > part_capacity_floats) return hipErrorInvalidValue;
  *S_out = S;
  const dim3 grid(tiles, S, mblocks);
  if (six) {
#define SP_GO6(MTV, PK)                                                                                          \
  hipLaunchKernelGGL((k_gemm_bf16<MTV, 6, false, SP_GEMM_KC_PLAIN, SP_GEMM_PF, PK, false, false, 6>), grid, dim3(384), 0, \
                     st, X, W, out, nullptr, M, N, K, K / SP_GEMM_KC_PLAIN, S, 0, rot_for(S, K))
    if (packed) { if (MT == 2) SP_GO6(2, true); else if (MT == 3) SP_GO6(3, true); else SP_GO6(4, true); }
    else { if (MT == 2) SP_GO6(2, false); else if (MT == 3) SP_GO6(3, false); else SP_GO6(4, false); }
#undef SP_GO6
    return hipGetLastError();
  }
  if (eight) {
#define SP_GO8(MTV, PK)                                                                                          \
  if (resident)                                                                                                  \
    hipLaunchKernelGGL((k_gemm_bf16<MTV, 8, false, SP_GEMM_KC_PLAIN, SP_GEMM_PF_EIGHT, PK, false, false, 8, false, false>), \
                       grid, dim3(512), 0, st, X, W, out, nullptr, M, N, K, K / SP_GEMM_KC_PLAIN, S, 0, rot_for(S, K)); \
  else                                                                                                           \
  hipLaunchKernelGGL((k_gemm_bf16<MTV, 8, false, SP_GEMM_KC_PLAIN, SP_GEMM_PF_EIGHT, PK, false, false, 8>), grid, dim3(512), 0, \
                     st, X, W, out, nullptr, M, N, K, K / SP_GEMM_KC_PLAIN, S, 0, rot_for(S, K))
    if (packed) { if (MT == 2) SP_GO8(2, true); else if (MT == 3) SP_GO8(3, true); else if (MT == 4) SP_GO8(4, true); else SP_GO8(8, true); }
    else { if (MT == 2) SP_GO8(2, false); else if (MT == 3) SP_GO8(3, false); else if (MT == 4) SP_GO8(4, false); else SP_GO8(8, false); }
#undef SP_GO8
    return hipGetLastError();
  }
  if (resident && MT == 1) {     // one row tile of a matrix that is to stay in the Infinity Cache: ordinary weight loads
    if (packed)
      hipLaunchKernelGGL((k_gemm_bf16<1, SP_GEMM_NCG_PLAIN, false, SP_GEMM_KC_PLAIN, SP_GEMM_PF, true, false, false, 4, false, false>),
                         grid, dim3(256), 0, st, X, W, out, nullptr, M, N, K, K / SP_GEMM_KC_PLAIN, S, 0, rot_for(S, K));
    else
      hipLaunchKernelGGL((k_gemm_bf16<1, SP_GEMM_NCG_PLAIN, false, SP_GEMM_KC_PLAIN, SP_GEMM_PF, false, false, false, 4, false, false>),
                         grid, dim3(256), 0, st, X, W, out, nullptr, M, N, K, K / SP_GEMM_KC_PLAIN, S, 0, rot_for(S, K));
    return hipGetLastError();
  }
  if (packed) return launch_mt<SP_GEMM_NCG_PLAIN, false, SP_GEMM_KC_PLAIN, true>(MT, grid, st, X, W, out, nullptr, M, N, K, S, two);
  return launch_mt<SP_GEMM_NCG_PLAIN, false, SP_GEMM_KC_PLAIN, false>(MT, grid, st, X, W, out, nullptr, M, N, K, S, two);
}

template <bool PACKED>
static hipError_t launch_even(int MT, int n_wg, hipStream_t st, const bf16_t* X, const bf16_t* W, bf16_t* act, int M,
                              int F, int K, int cpw) {
#define SP_GO(MTV)                                                                                              \
  hipLaunchKernelGGL((k_gemm_bf16<MTV, 4, true, SP_GEMM_KC_GATEUP, SP_GEMM_PF_EVEN, PACKED, false, false, 8, true>),   \
                     dim3(n_wg), dim3(512), 0, st, X, W, nullptr, act, M, F, K, K / SP_GEMM_KC_GATEUP, 1, cpw)
  switch (MT) {
    case 2: SP_GO(2); break;
    case 3: SP_GO(3); break;
    case 4: SP_GO(4); break;
    default:      // 65-128 rows: the 128-k chunk, so that the two 128-row panels fit
      hipLaunchKernelGGL((k_gemm_bf16<8, 4, true, 128, SP_GEMM_PF_EVEN, PACKED, false, false, 8, true>), dim3(n_wg), dim3(512), 0,
                         st, X, W, nullptr, act, M, F, K, K / 128, 1, cpw);
      break;
  }
#undef SP_GO
  return hipGetLastError();
}
// the same for 96 < cpw <= 112 (the 70B shape's d_ff = 28672 on 256 CUs): seven column groups, one wave each
template <bool PACKED>
static hipError_t launch_even7(int MT, int n_wg, hipStream_t st, const bf16_t* X, const bf16_t* W, bf16_t* act, int M,
                               int F, int K, int cpw) {
  // three weight chunks in flight up to 64 rows (148 -> 145 us per launch), two with 128 (three: 171 -> 179 us)
#define SP_GO(MTV, PFV)                                                                                         \
  hipLaunchKernelGGL((k_gemm_bf16<MTV, 7, true, 128, PFV, PACKED, false, false, 7, true>), dim3(n_wg), dim3(448), 0, st, X, \
                     W, nullptr, act, M, F, K, K / 128, 1, cpw)
  switch (MT) {
    case 2: SP_GO(2, 3); break;
    case 3: SP_GO(3, 3); break;
    case 4: SP_GO(4, 3); break;
    default: SP_GO(8, 2); break;
  }
#undef SP_GO
  return hipGetLastError();
}

hipError_t sp_launch_gemm_gateup_bf16(const bf16_t* X, const bf16_t* W, bool packed, bf16_t* act, int M, int F,
                                      int K, int n_cu, hipStream_t st) {
  int MT, mblocks;
  row_blocks(M, &MT, &mblocks);
  if (M < 1 || F % 64 || K % SP_GEMM_KC_GATEUP || K % 128) return hipErrorInvalidValue;
  // 17-64 rows and a d_ff that gives every CU the same 56 or 64 columns: one eight-wave workgroup per CU
  if (MT >= SP_GEMM_EVEN_MIN_MT && (MT <= 4 || (SP_GEMM_EVEN_MT8 && mblocks == 1)) && n_cu > 0 && F % n_cu == 0 && (F / n_cu) % 8 == 0 && F / n_cu > 48 &&
      F / n_cu <= 64 && SP_GEMM_KC_GATEUP == 256) {
    return packed ? launch_even<true>(MT, n_cu, st, X, W, act, M, F, K, F / n_cu)
                  : launch_even<false>(MT, n_cu, st, X, W, act, M, F, K, F / n_cu);
  }
  if (SP_GEMM_EVEN7 && MT >= 2 && mblocks == 1 && n_cu > 0 && F % n_cu == 0 && (F / n_cu) % 8 == 0 && F / n_cu > 96 &&
      F / n_cu <= 112) {
    return packed ? launch_even7<true>(MT, n_cu, st, X, W, act, M, F, K, F / n_cu)
                  : launch_even7<false>(MT, n_cu, st, X, W, act, M, F, K, F / n_cu);
  }
  // From 49 rows on: 64 gate + 64 up columns per workgroup (four column groups, 128-k chunks) where that
  // still gives every CU a workgroup, so that the staged panel is at most as large as the weights it meets
  // (70B shape: gate/up 193.6 -> 179.3 us at 64 rows, 252 -> 212 us at 128 rows); else 32 + 32 columns.  With
  // d_ff = 14336 the wider workgroups number 224 and run level with the 448 narrow ones (53.2 against 53.9 us).
  if ((MT == 8 || MT == 4) && F / 64 * mblocks >= 256) {
    const dim3 grid(F / 64, 1, mblocks);
    if (packed) return launch_mt<4, true, SP_GEMM_KC_GATEUP, true>(MT, grid, st, X, W, nullptr, act, M, F, K, 1);
    return launch_mt<4, true, SP_GEMM_KC_GATEUP, false>(MT, grid, st, X, W, nullptr, act, M, F, K, 1);
  }
  const int TILE = tile_cols(MT, true);
  const dim3 grid(F / TILE, 1, mblocks);
  if (packed) return launch_mt<SP_GEMM_NCG_GATEUP, true, SP_GEMM_KC_GATEUP, true>(MT, grid, st, X, W, nullptr, act, M, F, K, 1);
  return launch_mt<SP_GEMM_NCG_GATEUP, true, SP_GEMM_KC_GATEUP, false>(MT, grid, st, X, W, nullptr, act, M, F, K, 1);
}

// Output head: per row the top column of every 64-column tile, as (value, index) pairs
// pairs[(m * tiles + tile) * 2]; *tiles_out = V / 64.  One pass over the vocabulary matrix.
hipError_t sp_launch_gemm_argmax_bf16(const bf16_t* X, const bf16_t* W, bool packed, float* pairs, int M, int V, int K,
                                      size_t pair_capacity_floats, int* tiles_out, hipStream_t st) {
  static_assert(SP_GEMM_NCG_PLAIN == 4, "the top-column epilogue needs one wave per column group");
  int MT, mblocks;
  row_blocks(M, &MT, &mblocks);
  // 17-64 rows: eight waves over 128 columns share one staged panel, as in the plain projections
  const bool eight = SP_GEMM_ARGMAX8 && MT >= 2 && MT <= 4 && V % 128 == 0 && SP_GEMM_KC_PLAIN == 128;
  const int TILE = eight ? 128 : 16 * SP_GEMM_NCG_PLAIN;
  if (M < 1 || V % TILE || K % SP_GEMM_KC_PLAIN || K % 128) return hipErrorInvalidValue;
  const int tiles = V / TILE;
  if ((size_t)M * tiles * 2 > pair_capacity_floats) return hipErrorInvalidValue;
  *tiles_out = tiles;
  const dim3 grid(tiles, 1, mblocks);
  if (eight) {
#define SP_GOA(MTV, PK)                                                                                        \
  hipLaunchKernelGGL((k_gemm_bf16<MTV, 8, false, 128, SP_GEMM_PF, PK, true, false, 8>), grid, dim3(512), 0, st, X, W, \
                     pairs, nullptr, M, V, K, K / 128, 1, 0)
    if (packed) { if (MT == 2) SP_GOA(2, true); else if (MT == 3) SP_GOA(3, true); else SP_GOA(4, true); }
    else { if (MT == 2) SP_GOA(2, false); else if (MT == 3) SP_GOA(3, false); else SP_GOA(4, false); }
#undef SP_GOA
    return hipGetLastError();
  }
  if (packed) return launch_mt<SP_GEMM_NCG_PLAIN, false, SP_GEMM_KC_PLAIN, true, true>(MT, grid, st, X, W, pairs, nullptr, M, V, K, 1);
  return launch_mt<SP_GEMM_NCG_PLAIN, false, SP_GEMM_KC_PLAIN, false, true>(MT, grid, st, X, W, pairs, nullptr, M, V, K, 1);
}

// Re-lays a [N][K] row-major bf16 matrix into MFMA fragment order: 16-byte unit u of the output
// holds W[strip*16 + u%16][kstep*32 + ((u/16)%4)*8 .. +8] with u/64 = strip*(K/32) + kstep.
__global__ void k_pack_weights(const u32x4_t* __restrict__ in, u32x4_t* __restrict__ out, int N, int K) {
  const size_t units = (size_t)N * K / 8;
  for (size_t u = (size_t)blockIdx.x * blockDim.x + threadIdx.x; u < units; u += (size_t)gridDim.x * blockDim.x) {
    const size_t blk = u >> 6;
    const int lane = (int)(u & 63);
    const size_t strip = blk / (K / 32), ks = blk - strip * (K / 32);
    const size_t n = strip * 16 + (lane & 15), k = ks * 32 + (lane >> 4) * 8;
    out[u] = in[(n * K + k) / 8];
  }
}

hipError_t sp_launch_pack_weights(const void* in, void* out, int N, int K, hipStream_t st) {
  if (N % 16 || K % 32 || in == out) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_pack_weights, dim3(4096), dim3(256), 0, st, (const u32x4_t*)in, (u32x4_t*)out, N, K);
  return hipGetLastError();
}
