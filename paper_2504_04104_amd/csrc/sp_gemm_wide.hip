// bf16 projections for many rows (M > 128: a cold ragged batch forwards several hundred tree
// nodes at once, Sec. 4 "Implementation" / Sec. 4.4).  Here the matrix cores, not the weight
// stream, set the pace, so each wave keeps SPW strips of 16 weight rows in registers and every
// activation fragment it reads from LDS feeds SPW MFMAs.  A workgroup covers up to 16*MT rows x
// 64*SPW output columns.  Full row blocks come first in launch order, and those of one column
// tile get consecutive ids modulo 8: they run at the same time on the same XCD and share the
// tile's weights through its L2.  The last, partial row block of every tile comes after all
// full ones and runs a body compiled for its own height, so the short workgroups fill the CUs
// that the full ones leave over.
//
//   out[y][m][n] = sum_{k in slice y} X[m][k] * W[n][k]        (f32 partial sums)
//   gate/up:      act[m][f] = silu(X Wg^T) * (X Wu^T)          (each wave pairs gate and up strips)
#include "sp_launch.h"

#ifndef WKC
#define WKC 64                  // k per staged chunk
#endif
#define WXS (WKC * 2 + 16)      // LDS row stride of the activation panel in bytes

// Loads run NB-1 chunks ahead of the math in NB weight register sets, with NB LDS panels.  The
// memory counter retires loads in issue order, so activations and weights of one chunk are
// issued together and at matching distances: waiting for the activations that go to LDS next
// never forces a younger weight load.  Chunk indices past the end are clamped (a few redundant
// loads at the tail keep every chunk one straight-line block, which lets the LDS reads be
// scheduled among the MFMAs).
template <int SPW, int MT, bool GATEUP, bool PACKED>
__device__ __forceinline__ void wide_body(const bf16_t* __restrict__ X, const bf16_t* __restrict__ W,
                                          float* __restrict__ out, bf16_t* __restrict__ act, int M, int N, int K,
                                          int tile, int m_base, int c_begin, int c_end, char* lds_raw) {
  constexpr int WROWS = MT * 16;
  constexpr int NB = MT > 8 ? 3 : 4;               // weight register sets and LDS panels
  constexpr int NBX = MT > 8 ? 2 : 4;              // activation register sets
  constexpr int KSTEPS = WKC / 32;
  constexpr int ITEMS = KSTEPS * MT;               // (k step, row tile) pairs of a chunk
  constexpr int BQ = 4;                            // activation fragments read ahead of their MFMAs
  constexpr int UPR = WKC / 8, RPP = 256 / UPR, PASSES = WROWS / RPP;
  constexpr int GS = GATEUP ? SPW / 2 : SPW;       // strips per wave and matrix half
  char (*lds)[WROWS * WXS] = reinterpret_cast<char (*)[WROWS * WXS]>(lds_raw);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // known uniform: addresses split into scalar + lane part
  const int r = lane & 15, kg = lane >> 4;
  const int c_last = c_end - 1;
  // first weight row of strip a of this wave; for gate/up, strips GS.. are the up rows of the same columns
  const int n0 = tile * (64 * GS) + wave * (16 * GS);

  // weights: uniform strip origin + per-lane offset (elements)
  const bf16_t* ws[SPW];
#pragma unroll
  for (int a = 0; a < SPW; ++a) {
    const int row0 = (GATEUP && a >= GS) ? N + n0 + (a - GS) * 16 : n0 + a * 16;
    ws[a] = PACKED ? W + (size_t)(row0 / 16) * (K / 32) * 512 : W + (size_t)row0 * K;
  }
  const unsigned wl = PACKED ? lane * 8 : r * K + kg * 8;
#define SP_WOFF(C, s) (PACKED ? ((size_t)(C) * (WKC / 32) + (s)) * 512 : (size_t)(C)*WKC + (s) * 32)
  // activations: per-thread row offset (elements; rows past the end repeat the last row) + uniform chunk origin
  const int xu = tid % UPR, xr = tid / UPR;
  unsigned xo[PASSES];
#pragma unroll
  for (int p = 0; p < PASSES; ++p) xo[p] = (unsigned)min(m_base + p * RPP + xr, M - 1) * K + xu * 8;
  const unsigned bl = r * WXS + kg * 16;            // fragment read: row (tile*16 + l%16), k group l/16

  u32x4_t wb[NB][SPW][KSTEPS];
  u32x4_t xb[NBX][PASSES];
  f32x4_t acc[SPW][MT];
#pragma unroll
  for (int a = 0; a < SPW; ++a)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[a][mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

#define SP_LOAD_X(B, C)                                                                                 \
  {                                                                                                     \
    const bf16_t* xs = X + (size_t)min((C), c_last) * WKC;                                              \
    _Pragma("unroll") for (int p = 0; p < PASSES; ++p)                                                  \
        xb[B][p] = *reinterpret_cast<const u32x4_t*>(xs + xo[p]);                                       \
  }
#define SP_STORE_X(B, BUF)                                                                              \
  _Pragma("unroll") for (int p = 0; p < PASSES; ++p)                                                    \
      *reinterpret_cast<u32x4_t*>(&lds[BUF][(p * RPP + xr) * WXS + xu * 16]) = xb[B][p];
#define SP_LOAD_W(B, C)                                                                                 \
  {                                                                                                     \
    const int cw = min((C), c_last);                                                                    \
    _Pragma("unroll") for (int a = 0; a < SPW; ++a)                                                     \
        _Pragma("unroll") for (int s = 0; s < KSTEPS; ++s)                                              \
            wb[B][a][s] = *reinterpret_cast<const u32x4_t*>(ws[a] + SP_WOFF(cw, s) + wl);               \
  }
  // item j of a chunk: k step j / MT, row tile j % MT
#define SP_LDS_B(BUF, j)                                                                                \
  (*reinterpret_cast<const bf16x8_t*>(&lds[BUF][((j) % MT) * 16 * WXS + ((j) / MT) * 64 + bl]))
  // Chunk C, weights in register set B, activations in LDS panel B.  The activations of chunk
  // C+2 go from their register set BX to their panel; that set then takes chunk C+2+NBX and
  // weight set B-1 the weights of chunk C+NB-1.  The last BQ fragment reads already address the
  // next panel, which has been complete since the previous barrier, so the barrier at the end of
  // the chunk is not followed by an exposed LDS round trip.
#define SP_CHUNK(B, BX, C)                                                                              \
  {                                                                                                     \
    const int c_ = (C);                                                                                 \
    SP_STORE_X(BX, ((B) + 2) % NB)                                                                      \
    SP_LOAD_X(BX, c_ + 2 + NBX)                                                                         \
    SP_LOAD_W(((B) + NB - 1) % NB, c_ + NB - 1)                                                         \
    _Pragma("unroll") for (int j = 0; j < ITEMS; ++j) {                                                 \
      const bf16x8_t b = bq[j % BQ];                                                                    \
      if (j + BQ < ITEMS) bq[j % BQ] = SP_LDS_B(B, j + BQ);                                             \
      else bq[j % BQ] = SP_LDS_B(((B) + 1) % NB, j + BQ - ITEMS);                                       \
      _Pragma("unroll") for (int a = 0; a < SPW; ++a) acc[a][j % MT] = __builtin_amdgcn_mfma_f32_16x16x32_bf16( \
          *reinterpret_cast<const bf16x8_t*>(&wb[B][a][j / MT]), b, acc[a][j % MT], 0, 0, 0);           \
    }                                                                                                   \
    /* issue order: panel stores, then per fragment SPW MFMAs, a global load, the next fragment read */ \
    __builtin_amdgcn_sched_group_barrier(0x200, PASSES, 0);                                             \
    _Pragma("unroll") for (int j = 0; j < ITEMS; ++j) {                                                 \
      __builtin_amdgcn_sched_group_barrier(0x008, SPW, 0);                                              \
      if (j < PASSES + SPW * KSTEPS) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                 \
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                \
    }                                                                                                   \
    __syncthreads();                                                                                    \
  }

  // prologue: chunks 0 and 1 to their panels, the next NBX activation chunks and the first NB-1
  // weight chunks in flight
#pragma unroll
  for (int i = 0; i < NBX; ++i) SP_LOAD_X(i, c_begin + i)
#pragma unroll
  for (int i = 0; i + 1 < NB; ++i) SP_LOAD_W(i, c_begin + i)
  SP_STORE_X(0, 0)
  SP_STORE_X(1, 1)
  SP_LOAD_X(0, c_begin + NBX)
  SP_LOAD_X(1, c_begin + NBX + 1)
  __syncthreads();
  bf16x8_t bq[BQ];
#pragma unroll
  for (int j = 0; j < BQ; ++j) bq[j] = SP_LDS_B(0, j);
  // unrolled over the common period of the weight and activation set indices
  constexpr int PERIOD = NB == NBX ? NB : NB * NBX;
  for (int c = c_begin; c < c_end; c += PERIOD) {
    SP_CHUNK(0, 2 % NBX, c)
    if (c + 1 < c_end) SP_CHUNK(1 % NB, 3 % NBX, c + 1)
    if (c + 2 < c_end) SP_CHUNK(2 % NB, 4 % NBX, c + 2)
    if (c + 3 < c_end) SP_CHUNK(3 % NB, 5 % NBX, c + 3)
    if (PERIOD > 4) {
      if (c + 4 < c_end) SP_CHUNK(4 % NB, 6 % NBX, c + 4)
      if (c + 5 < c_end) SP_CHUNK(5 % NB, 7 % NBX, c + 5)
    }
  }
#undef SP_CHUNK
#undef SP_LDS_B
#undef SP_LOAD_W
#undef SP_STORE_X
#undef SP_LOAD_X
#undef SP_WOFF

  // lane holds, for activation row m = mt*16 + l%16, output columns (strip base) + 4*(l/16) + 0..3
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = m_base + mt * 16 + r;
    if (m >= M) continue;
    if (GATEUP) {
#pragma unroll
      for (int a = 0; a < GS; ++a) {
        float o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float gte = acc[a][mt][i], up = acc[GS + a][mt][i];
          o[i] = gte / (1.f + __expf(-gte)) * up;
        }
        uint2 pk;
        pk.x = pack_bf16x2(o[0], o[1]);
        pk.y = pack_bf16x2(o[2], o[3]);
        *reinterpret_cast<uint2*>(act + (size_t)m * N + n0 + a * 16 + 4 * kg) = pk;
      }
    } else {
#pragma unroll
      for (int a = 0; a < SPW; ++a)
        *reinterpret_cast<f32x4_t*>(out + ((size_t)blockIdx.y * M + m) * N + n0 + a * 16 + 4 * kg) = acc[a][mt];
    }
  }
}

#ifndef SP_WIDE_OCC8
#define SP_WIDE_OCC8 1
#endif
template <int SPW, int MTMAX, bool GATEUP, bool PACKED>
__global__ void __launch_bounds__(256, MTMAX > 8 ? 1 : SP_WIDE_OCC8)
k_gemm_wide(const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, float* __restrict__ out,
            bf16_t* __restrict__ act, int M, int N, int K, int n_tiles, int S) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];      // activation panels
  constexpr int WROWS = MTMAX * 16;
  const int n_full = M / WROWS;                     // full row blocks of every column tile
  const int tiles8 = (n_tiles + 7) & ~7;
  const int lin = blockIdx.x;
  int tile, mblk;
  if (lin < tiles8 * n_full) {
    const int xcd = lin & 7, j = lin >> 3;
    tile = (j / n_full) * 8 + xcd;
    mblk = j % n_full;
  } else {
    tile = lin - tiles8 * n_full;
    mblk = n_full;
  }
  if (tile >= n_tiles) return;                      // whole workgroup (the grid is padded to a multiple of 8)
  const int m_base = mblk * WROWS;
  const int chunks_total = K / WKC;
  const int c_begin = (int)(((long long)blockIdx.y * chunks_total) / S);
  const int c_end = (int)(((long long)(blockIdx.y + 1) * chunks_total) / S);
  if (c_begin >= c_end) return;                     // whole workgroup (S never exceeds the chunk count)
  const int rows = M - m_base;                      // uniform over the workgroup
  if (MTMAX > 12 && rows > 192) wide_body<SPW, MTMAX, GATEUP, PACKED>(X, W, out, act, M, N, K, tile, m_base, c_begin, c_end, lds_raw);
  else if (MTMAX > 8 && rows > 128) wide_body<SPW, 12, GATEUP, PACKED>(X, W, out, act, M, N, K, tile, m_base, c_begin, c_end, lds_raw);
  else if (rows > 64) wide_body<SPW, 8, GATEUP, PACKED>(X, W, out, act, M, N, K, tile, m_base, c_begin, c_end, lds_raw);
  else wide_body<SPW, 4, GATEUP, PACKED>(X, W, out, act, M, N, K, tile, m_base, c_begin, c_end, lds_raw);
}

// Launch with the activation panels as dynamic LDS (more than the 64 KB a kernel may declare
// statically).
template <int SPW, int MT, bool GATEUP, bool PACKED>
static hipError_t launch_wide(dim3 grid, hipStream_t st, const bf16_t* X, const bf16_t* W, float* out, bf16_t* act,
                              int M, int N, int K, int n_tiles, int S) {
  constexpr int LDS_BYTES = (MT > 8 ? 3 : 4) * MT * 16 * WXS;    // NB panels of the tallest body
  static bool ready = false;
  if (!ready) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_wide<SPW, MT, GATEUP, PACKED>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (e != hipSuccess) return e;
    ready = true;
  }
  hipLaunchKernelGGL((k_gemm_wide<SPW, MT, GATEUP, PACKED>), grid, dim3(256), LDS_BYTES, st, X, W, out, act, M, N, K,
                     n_tiles, S);
  return hipGetLastError();
}

// rows per workgroup: 256 once there are enough rows to fill them, else 128
#ifndef SP_WIDE_ROWS
#define SP_WIDE_ROWS(M) ((M) > 384 ? 256 : 128)
#endif
static inline int wide_rows(int M) { return SP_WIDE_ROWS(M); }

hipError_t sp_launch_gemm_wide(const bf16_t* X, const bf16_t* W, bool packed, float* out, int M, int N, int K,
                               int n_cu, size_t part_capacity_floats, int* S_out, hipStream_t st) {
  constexpr int SPW = 4;
  if (M < 1 || N % (64 * SPW) || K % WKC) return hipErrorInvalidValue;
  const int WROWS = wide_rows(M);
  const int n_tiles = N / (64 * SPW), m_blocks = (M + WROWS - 1) / WROWS;
  const int chunks = K / WKC;
  int S = n_cu / (n_tiles * m_blocks);              // split K until about every CU has a workgroup
  if (S < 1) S = 1;
  if (S > 8) S = 8;
  if (S > chunks) S = chunks;
  while (S > 1 && (size_t)S * M * N > part_capacity_floats) --S;
  if ((size_t)S * M * N > part_capacity_floats) return hipErrorInvalidValue;
  *S_out = S;
  const int tiles8 = (n_tiles + 7) / 8 * 8;
  const dim3 grid(tiles8 * m_blocks, S);
  if (WROWS == 256)
    return packed ? launch_wide<SPW, 16, false, true>(grid, st, X, W, out, nullptr, M, N, K, n_tiles, S)
                  : launch_wide<SPW, 16, false, false>(grid, st, X, W, out, nullptr, M, N, K, n_tiles, S);
  return packed ? launch_wide<SPW, 8, false, true>(grid, st, X, W, out, nullptr, M, N, K, n_tiles, S)
                : launch_wide<SPW, 8, false, false>(grid, st, X, W, out, nullptr, M, N, K, n_tiles, S);
}

hipError_t sp_launch_gemm_wide_gateup(const bf16_t* X, const bf16_t* W, bool packed, bf16_t* act, int M, int F, int K,
                                      hipStream_t st) {
  constexpr int SPW = 4;                            // two gate strips and two up strips per wave
  constexpr int TW = 64 * (SPW / 2);                // activation columns per workgroup
  if (M < 1 || F % TW || K % WKC) return hipErrorInvalidValue;
  const int WROWS = wide_rows(M);
  const int n_tiles = F / TW, m_blocks = (M + WROWS - 1) / WROWS;
  const int tiles8 = (n_tiles + 7) / 8 * 8;
  const dim3 grid(tiles8 * m_blocks, 1);
  if (WROWS == 256)
    return packed ? launch_wide<SPW, 16, true, true>(grid, st, X, W, nullptr, act, M, F, K, n_tiles, 1)
                  : launch_wide<SPW, 16, true, false>(grid, st, X, W, nullptr, act, M, F, K, n_tiles, 1);
  return packed ? launch_wide<SPW, 8, true, true>(grid, st, X, W, nullptr, act, M, F, K, n_tiles, 1)
                : launch_wide<SPW, 8, true, false>(grid, st, X, W, nullptr, act, M, F, K, n_tiles, 1);
}
