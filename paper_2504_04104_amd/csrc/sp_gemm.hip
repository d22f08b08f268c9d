// bf16 projections for few rows (M = tree nodes in flight, typically <= 64) on the
// CDNA4 matrix cores.  With so few rows every weight is used once, so the kernel is a
// weight streamer (decode is bound by loading parameters, Sec. 2.2): each wave pulls
// its 16 weight rows straight from HBM into registers in MFMA operand layout (one
// 16-byte load per lane per k-step, two chunks deep), while the M x K activation
// panel -- shared by every wave -- is staged once per workgroup through LDS.
//
//   out[y][m][n] = sum_{k in slice y} X[m][k] * W[n][k]        (f32 partial sums)
//
// v_mfma_f32_16x16x32_bf16: A = 16 weight rows x 32 k (lane l: row l%16, k (l/16)*8..+8),
// B = 32 k x 16 activation rows (lane l: row l%16, same k), D[4*(l/16)+i][l%16].
#include "sp_launch.h"

#define KC 256                 // k per staged chunk
#define XS 528                 // LDS row stride in bytes: KC*2 + 16 (conflict-free 16-byte reads)

template <int MT, int NCG, bool GATEUP>
__global__ void __launch_bounds__(256)
k_gemm_bf16(const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, float* __restrict__ out,
            bf16_t* __restrict__ act, int M, int N, int K, int chunks_total, int S) {
  constexpr int NKH = 4 / NCG;          // waves sharing a column group split each chunk's k-steps
  constexpr int KSTEPS = 8 / NKH;
  constexpr int NW = GATEUP ? 2 : 1;
  constexpr int ROWS = MT * 16;
  __shared__ __attribute__((aligned(16))) char lds[2][ROWS * XS];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int cg = wave % NCG, kh = wave / NCG;
  const int r = lane & 15, kg = lane >> 4;
  const int n0 = blockIdx.x * (16 * NCG) + cg * 16;
  const int m_base = blockIdx.z * 64;
  const int c_begin = (int)(((long long)blockIdx.y * chunks_total) / S);
  const int c_end = (int)(((long long)(blockIdx.y + 1) * chunks_total) / S);

  const bf16_t* w0 = W + (size_t)(n0 + r) * K + kg * 8 + kh * (KSTEPS * 32);
  const bf16_t* w1 = W + (size_t)(N + n0 + r) * K + kg * 8 + kh * (KSTEPS * 32);   // up rows (GATEUP)
  const int xu = tid & 31, xr = tid >> 5;       // 16-byte unit and row (8 rows per pass) of the X stager

  uint4 wcur[NW][KSTEPS], wnxt[NW][KSTEPS];
  uint4 xnxt[2 * MT];
  f32x4_t acc[NW][MT];
#pragma unroll
  for (int a = 0; a < NW; ++a)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[a][mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

  auto load_x = [&](int c) {
#pragma unroll
    for (int p = 0; p < 2 * MT; ++p) {
      const int m = m_base + p * 8 + xr;
      xnxt[p] = (m < M) ? *reinterpret_cast<const uint4*>(X + (size_t)m * K + (size_t)c * KC + xu * 8)
                        : make_uint4(0u, 0u, 0u, 0u);
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int p = 0; p < 2 * MT; ++p)
      *reinterpret_cast<uint4*>(&lds[buf][(p * 8 + xr) * XS + xu * 16]) = xnxt[p];
  };
  auto load_w = [&](uint4 (&dst)[NW][KSTEPS], int c) {
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
      dst[0][s] = *reinterpret_cast<const uint4*>(w0 + (size_t)c * KC + s * 32);
      if (GATEUP) dst[NW - 1][s] = *reinterpret_cast<const uint4*>(w1 + (size_t)c * KC + s * 32);
    }
  };

  if (c_begin < c_end) {
    load_x(c_begin);
    load_w(wcur, c_begin);
    store_x(0);
  }
  __syncthreads();
  for (int c = c_begin; c < c_end; ++c) {
    const int buf = (c - c_begin) & 1;
    const bool more = c + 1 < c_end;
    if (more) { load_x(c + 1); load_w(wnxt, c + 1); }   // X first: its wait must not drain the weight loads
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const bf16x8_t b = *reinterpret_cast<const bf16x8_t*>(
            &lds[buf][(mt * 16 + r) * XS + ((kh * KSTEPS + s) * 32 + kg * 8) * 2]);
#pragma unroll
        for (int a = 0; a < NW; ++a)
          acc[a][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(&wcur[a][s]), b,
                                                               acc[a][mt], 0, 0, 0);
      }
    }
    if (more) store_x(buf ^ 1);
    __syncthreads();
    if (more) {
#pragma unroll
      for (int a = 0; a < NW; ++a)
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) wcur[a][s] = wnxt[a][s];
    }
  }

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
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = m_base + mt * 16 + r;
    if (m >= M) continue;
    if (GATEUP) {
      uint16_t o[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float gte = acc[0][mt][i], up = acc[NW - 1][mt][i];
        o[i] = f32_to_bf16(gte / (1.f + __expf(-gte)) * up);
      }
      uint2 pk;
      pk.x = (uint32_t)o[0] | ((uint32_t)o[1] << 16);
      pk.y = (uint32_t)o[2] | ((uint32_t)o[3] << 16);
      *reinterpret_cast<uint2*>(act + (size_t)m * N + ncol) = pk;
    } else {
      *reinterpret_cast<f32x4_t*>(out + ((size_t)blockIdx.y * M + m) * N + ncol) = acc[0][mt];
    }
  }
}

// ---- launchers -------------------------------------------------------------------
template <int NCG, bool GATEUP>
static hipError_t launch_mt(int MT, dim3 grid, hipStream_t st, const bf16_t* X, const bf16_t* W, float* out,
                            bf16_t* act, int M, int N, int K, int chunks, int S) {
  switch (MT) {
    case 1: hipLaunchKernelGGL((k_gemm_bf16<1, NCG, GATEUP>), grid, dim3(256), 0, st, X, W, out, act, M, N, K, chunks, S); break;
    case 2: hipLaunchKernelGGL((k_gemm_bf16<2, NCG, GATEUP>), grid, dim3(256), 0, st, X, W, out, act, M, N, K, chunks, S); break;
    case 3: hipLaunchKernelGGL((k_gemm_bf16<3, NCG, GATEUP>), grid, dim3(256), 0, st, X, W, out, act, M, N, K, chunks, S); break;
    default: hipLaunchKernelGGL((k_gemm_bf16<4, NCG, GATEUP>), grid, dim3(256), 0, st, X, W, out, act, M, N, K, chunks, S); break;
  }
  return hipGetLastError();
}

hipError_t sp_launch_gemm_bf16(const bf16_t* X, const bf16_t* W, float* out, int M, int N, int K, int max_split,
                               size_t part_capacity_floats, int* S_out, hipStream_t st) {
  if (M < 1 || N % 64 || K % KC) return hipErrorInvalidValue;
  const int chunks = K / KC;
  const int mblocks = (M + 63) / 64;
  const int MT = M >= 64 ? 4 : (M + 15) / 16;
  const int tiles = N / 64;
  // enough workgroups to keep every CU streaming, within the partial-sum buffer
  int S = (768 + tiles * mblocks - 1) / (tiles * mblocks);
  if (S > max_split) S = max_split;
  if (S > chunks) S = chunks;
  while (S > 1 && (size_t)S * M * N > part_capacity_floats) --S;
  if (S < 1) S = 1;
  if ((size_t)S * M * N > part_capacity_floats) return hipErrorInvalidValue;
  *S_out = S;
  return launch_mt<4, false>(MT, dim3(tiles, S, mblocks), st, X, W, out, nullptr, M, N, K, chunks, S);
}

hipError_t sp_launch_gemm_gateup_bf16(const bf16_t* X, const bf16_t* W, bf16_t* act, int M, int F, int K,
                                      hipStream_t st) {
  if (M < 1 || F % 32 || K % KC) return hipErrorInvalidValue;
  const int mblocks = (M + 63) / 64;
  const int MT = M >= 64 ? 4 : (M + 15) / 16;
  return launch_mt<2, true>(MT, dim3(F / 32, 1, mblocks), st, X, W, nullptr, act, M, F, K, K / KC, 1);
}
