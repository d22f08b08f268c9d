// bf16 projections for many rows (M > 128: a cold ragged batch forwards several hundred tree
// nodes at once, Sec. 4 "Implementation" / Sec. 4.4).  Here the matrix cores, not the weight
// stream, set the pace, so each wave keeps SPW strips of 16 weight rows in registers and every
// activation fragment it reads from LDS feeds SPW MFMAs.  A workgroup covers 128 rows x 64*SPW
// output columns; the row blocks of one column tile are given consecutive ids modulo 8, so they
// run on the same XCD and all but the first find the weights in that XCD's L2.
//
//   out[y][m][n] = sum_{k in slice y} X[m][k] * W[n][k]        (f32 partial sums)
//   gate/up:      act[m][f] = silu(X Wg^T) * (X Wu^T)          (each wave pairs gate and up strips)
#include "sp_launch.h"

#define WKC 64                  // k per staged chunk
#define WXS (WKC * 2 + 16)      // LDS row stride of the activation panel in bytes
#define WROWS 128               // rows per block
#ifndef SP_WIDE_PF
#define SP_WIDE_PF 3            // weight chunks in flight ahead of the math (each is SPW*2 registers of 16 B)
#endif

template <int SPW, bool GATEUP, bool PACKED>
__global__ void __launch_bounds__(256)
k_gemm_wide(const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, float* __restrict__ out,
            bf16_t* __restrict__ act, int M, int N, int K, int n_tiles, int m_blocks, int S) {
  constexpr int MT = WROWS / 16;
  constexpr int KSTEPS = WKC / 32;
  constexpr int UPR = WKC / 8, RPP = 256 / UPR, PASSES = WROWS / RPP;
  constexpr int GS = GATEUP ? SPW / 2 : SPW;       // strips per wave and matrix half
  __shared__ __attribute__((aligned(16))) char lds[2][WROWS * WXS];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, kg = lane >> 4;
  // (column tile, row block) of this workgroup: row blocks of a tile share an XCD (ids equal modulo 8)
  const int lin = blockIdx.x;
  const int xcd = lin & 7, j = lin >> 3;
  const int tile = (j / m_blocks) * 8 + xcd, mblk = j % m_blocks;
  if (tile >= n_tiles) return;                      // whole workgroup (grid is padded to a multiple of 8)
  const int m_base = mblk * WROWS;
  const int chunks_total = K / WKC;
  const int c_begin = (int)(((long long)blockIdx.y * chunks_total) / S);
  const int c_end = (int)(((long long)(blockIdx.y + 1) * chunks_total) / S);
  // first weight row of strip a of this wave; for gate/up, strips GS.. are the up rows of the same columns
  const int n0 = tile * (64 * GS) + wave * (16 * GS);

  const bf16_t* wp[SPW];
#pragma unroll
  for (int a = 0; a < SPW; ++a) {
    const int row0 = (GATEUP && a >= GS) ? N + n0 + (a - GS) * 16 : n0 + a * 16;
    wp[a] = PACKED ? W + (size_t)(row0 / 16) * (K / 32) * 512 + lane * 8 : W + (size_t)(row0 + r) * K + kg * 8;
  }
#define SP_WOFF(C, s) (PACKED ? ((size_t)(C) * (WKC / 32) + (s)) * 512 : (size_t)(C)*WKC + (s) * 32)
  const int xu = tid % UPR, xr = tid / UPR;
  const int m_last = M - 1;

  constexpr int PF = SP_WIDE_PF, NB = PF + 1;
  u32x4_t wb[NB][SPW][KSTEPS];
  u32x4_t xnxt[PASSES];
  f32x4_t acc[SPW][MT];
#pragma unroll
  for (int a = 0; a < SPW; ++a)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[a][mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

#define SP_LOAD_X(C)                                                                                    \
  _Pragma("unroll") for (int p = 0; p < PASSES; ++p) {                                                  \
    const int m = min(m_base + p * RPP + xr, m_last);                                                   \
    xnxt[p] = *reinterpret_cast<const u32x4_t*>(X + (size_t)m * K + (size_t)(C)*WKC + xu * 8);          \
  }
#define SP_STORE_X(BUF)                                                                                 \
  _Pragma("unroll") for (int p = 0; p < PASSES; ++p)                                                    \
      *reinterpret_cast<u32x4_t*>(&lds[BUF][(p * RPP + xr) * WXS + xu * 16]) = xnxt[p];
#define SP_LOAD_W(B, C)                                                                                 \
  _Pragma("unroll") for (int a = 0; a < SPW; ++a)                                                       \
      _Pragma("unroll") for (int s = 0; s < KSTEPS; ++s)                                                \
          wb[B][a][s] = *reinterpret_cast<const u32x4_t*>(wp[a] + SP_WOFF(C, s));
#define SP_CHUNK(B, C)                                                                                  \
  {                                                                                                     \
    const int c_ = (C);                                                                                 \
    const int buf = (c_ - c_begin) & 1;                                                                 \
    if (c_ + 1 < c_end) { SP_STORE_X(buf ^ 1) }                                                         \
    if (c_ + 2 < c_end) { SP_LOAD_X(c_ + 2) }                                                           \
    if (c_ + PF < c_end) { SP_LOAD_W(((B) + PF) % NB, c_ + PF) }                                        \
    _Pragma("unroll") for (int s = 0; s < KSTEPS; ++s) {                                                \
      _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) {                                               \
        const bf16x8_t b = *reinterpret_cast<const bf16x8_t*>(                                          \
            &lds[buf][(mt * 16 + r) * WXS + (s * 32 + kg * 8) * 2]);                                    \
        _Pragma("unroll") for (int a = 0; a < SPW; ++a) acc[a][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16( \
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
#undef SP_CHUNK
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

hipError_t sp_launch_gemm_wide(const bf16_t* X, const bf16_t* W, bool packed, float* out, int M, int N, int K,
                               int n_cu, size_t part_capacity_floats, int* S_out, hipStream_t st) {
  constexpr int SPW = 4;
  if (M < 1 || N % (64 * SPW) || K % WKC) return hipErrorInvalidValue;
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
  if (packed)
    hipLaunchKernelGGL((k_gemm_wide<SPW, false, true>), grid, dim3(256), 0, st, X, W, out, nullptr, M, N, K, n_tiles,
                       m_blocks, S);
  else
    hipLaunchKernelGGL((k_gemm_wide<SPW, false, false>), grid, dim3(256), 0, st, X, W, out, nullptr, M, N, K, n_tiles,
                       m_blocks, S);
  return hipGetLastError();
}

hipError_t sp_launch_gemm_wide_gateup(const bf16_t* X, const bf16_t* W, bool packed, bf16_t* act, int M, int F, int K,
                                      hipStream_t st) {
  constexpr int SPW = 4;                            // two gate strips and two up strips per wave
  constexpr int TW = 64 * (SPW / 2);                // activation columns per workgroup
  if (M < 1 || F % TW || K % WKC) return hipErrorInvalidValue;
  const int n_tiles = F / TW, m_blocks = (M + WROWS - 1) / WROWS;
  const int tiles8 = (n_tiles + 7) / 8 * 8;
  const dim3 grid(tiles8 * m_blocks, 1);
  if (packed)
    hipLaunchKernelGGL((k_gemm_wide<SPW, true, true>), grid, dim3(256), 0, st, X, W, nullptr, act, M, F, K, n_tiles,
                       m_blocks, 1);
  else
    hipLaunchKernelGGL((k_gemm_wide<SPW, true, false>), grid, dim3(256), 0, st, X, W, nullptr, act, M, F, K, n_tiles,
                       m_blocks, 1);
  return hipGetLastError();
}
