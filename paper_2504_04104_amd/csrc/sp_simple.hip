// Plain kernels for any dtype: a dot-product GEMM and a one-wave-per-(row, head)
// tree attention.  They carry the float32 configuration and serve as the slow
// path selected by SP_FLAG_SIMPLE_KERNELS; the bf16 MFMA kernels replace them on
// the hot path.
#include "sp_launch.h"

// out[m][n] = sum_k X[m][k] W[n][k].  A wave owns one n and eight rows m at a time;
// lanes stride over k.
template <typename T>
__global__ void __launch_bounds__(256) k_gemm_simple(const T* X, const T* W, float* out, int M, int N, int K) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + wave;
  const int m0 = blockIdx.y * 8;
  if (n >= N) return;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const T* w = W + (size_t)n * K;
  for (int k = lane; k < K; k += 64) {
    const float wv = Elt<T>::ld(w + k);
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (m0 + i < M) acc[i] += wv * Elt<T>::ld(X + (size_t)(m0 + i) * K + k);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float v = wave_sum(acc[i]);
    if (lane == 0 && m0 + i < M) out[(size_t)(m0 + i) * N + n] = v;
  }
}

// Tree attention (Sec. 2.1 attention; Sec. 2.2 / 3.3.2 tree mask).  One wave per
// (row, query head).  Lanes stride over the visible cache slots -- the committed
// context, then the tree nodes whose bit is set in the row's ancestor mask -- each
// lane keeping an online softmax of its own; the 64 partial states are merged at
// the end.
template <typename T, int DH>
__global__ void __launch_bounds__(256) k_attn_simple(const T* q, const RowInfo* rows, const ReqTables* tables,
                                                      KvGeom g, int layer, T* out, int M, int n_q, int n_kv) {
  __shared__ float s_q[4][DH];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int item = blockIdx.x * 4 + wave;            // row * n_q + head
  const bool valid = item < M * n_q;
  const int row = valid ? item / n_q : 0, head = valid ? item - row * n_q : 0;
  const int kvh = head / (n_q / n_kv);
  const RowInfo ri = rows[row];
  for (int t = lane; t < DH; t += 64) s_q[wave][t] = Elt<T>::ld(q + ((size_t)row * n_q + head) * DH + t);
  __syncthreads();
  if (!valid) return;
  unsigned long long anc[SP_W];
#pragma unroll
  for (int w = 0; w < SP_W; ++w) anc[w] = tables[ri.req].anc[ri.node][w];
  const char* kplane = g.kv + ((size_t)(layer * 2 + 0) * n_kv + kvh) * g.plane_bytes + (size_t)ri.base * g.row_bytes;
  const char* vplane = g.kv + ((size_t)(layer * 2 + 1) * n_kv + kvh) * g.plane_bytes + (size_t)ri.base * g.row_bytes;
  const float scale = rsqrtf((float)DH);
  float mx = -INFINITY, l = 0.f;
  float o[DH];
#pragma unroll
  for (int t = 0; t < DH; ++t) o[t] = 0.f;
  const int total = ri.P + ri.T;
  for (int s = lane; s < total; s += 64) {
    if (s >= ri.P) {
      const int j = s - ri.P;
      if (!((anc[j >> 6] >> (j & 63)) & 1ull)) continue;
    }
    // kplane / vplane start at the request's base slot; a paged request has base 0
    const size_t ps = g.page_table ? sp_phys_slot(g, ri.req, 0, s) : (size_t)s;
    const T* k = reinterpret_cast<const T*>(kplane + ps * g.row_bytes);
    const T* v = reinterpret_cast<const T*>(vplane + ps * g.row_bytes);
    float sc = 0.f;
#pragma unroll 8
    for (int t = 0; t < DH; ++t) sc += s_q[wave][t] * Elt<T>::ld(k + t);
    sc *= scale;
    const float mn = fmaxf(mx, sc);
    const float corr = __expf(mx - mn), p = __expf(sc - mn);
    l = l * corr + p;
#pragma unroll
    for (int t = 0; t < DH; ++t) o[t] = o[t] * corr + p * Elt<T>::ld(v + t);
    mx = mn;
  }
  const float gm = wave_max(mx);
  const float f = (mx == -INFINITY) ? 0.f : __expf(mx - gm);
  const float gl = wave_sum(l * f);
  const float inv = 1.f / gl;
  T* orow = out + ((size_t)row * n_q + head) * DH;
#pragma unroll
  for (int t = 0; t < DH; ++t) {
    const float v = wave_sum(o[t] * f) * inv;
    if (lane == (t & 63)) Elt<T>::st(orow + t, v);
  }
}

hipError_t sp_launch_gemm_simple(int dtype, const void* X, const void* W, float* out, int M, int N, int K,
                                 hipStream_t st) {
  dim3 grid((N + 3) / 4, (M + 7) / 8);
  if (dtype == 0)
    hipLaunchKernelGGL(k_gemm_simple<float>, grid, dim3(256), 0, st, (const float*)X, (const float*)W, out, M, N, K);
  else
    hipLaunchKernelGGL(k_gemm_simple<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)X, (const bf16_t*)W, out, M, N, K);
  return hipGetLastError();
}

hipError_t sp_launch_attn_simple(int dtype, const void* q, const RowInfo* rows, const ReqTables* tables, KvGeom g,
                                 int layer, void* out, int M, int n_q, int n_kv, int d_head, hipStream_t st) {
  dim3 grid((M * n_q + 3) / 4);
#define SP_ATTN_CASE(TT, DH)                                                                                       \
  hipLaunchKernelGGL((k_attn_simple<TT, DH>), grid, dim3(256), 0, st, (const TT*)q, rows, tables, g, layer, (TT*)out, \
                     M, n_q, n_kv)
  if (dtype == 0 && d_head == 64) SP_ATTN_CASE(float, 64);
  else if (dtype == 0 && d_head == 128) SP_ATTN_CASE(float, 128);
  else if (dtype == 1 && d_head == 64) SP_ATTN_CASE(bf16_t, 64);
  else if (dtype == 1 && d_head == 128) SP_ATTN_CASE(bf16_t, 128);
  else return hipErrorInvalidValue;
#undef SP_ATTN_CASE
  return hipGetLastError();
}
