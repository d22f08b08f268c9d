// Row-wise pieces of the decoder layer (Llama family: Sec. 2.1, Sec. 4 "Testbed"):
// row descriptors and rotary tables, residual add + RMSNorm, RoPE + KV append,
// SiLU*mul, and the final write-out.  The projections leave their results as
// float32 partial sums [S][M][N]; the kernels here fold the S slices in.
#include "sp_launch.h"

// -----------------------------------------------------------------------------
// One thread per (row, pair t).  Position of a node = prefix length + depth: each
// tree level is one future position (Sec. 3.2).  The angle is formed in double so
// that positions of tens of thousands keep full float accuracy in cos and sin.
__global__ void k_prep_rows(FwdBatch b, const ReqMeta* meta, const ReqTables* tables, RowInfo* rows, float* cs,
                            int d_head, float theta) {
  const int half = d_head >> 1;
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int row = idx / half, tt = idx - row * half;
  if (row >= b.n_rows) return;
  int seg = 0;
  while (seg + 1 < b.n_req && row >= b.row0[seg + 1]) ++seg;
  const int req = b.req[seg];
  const int node = b.first[seg] + (row - b.row0[seg]);
  const ReqMeta m = meta[req];
  const int pos = m.P + tables[req].depth[node];
  if (tt == 0) {
    RowInfo ri;
    ri.base = m.base; ri.req = req; ri.node = node; ri.pos = pos; ri.P = m.P; ri.T = m.T; ri.seg = seg;
    rows[row] = ri;
  }
  const double inv_freq = exp2(-(2.0 * (double)tt / (double)d_head) * log2((double)theta));
  const double ang = (double)pos * inv_freq;
  cs[(size_t)row * d_head + tt] = (float)cos(ang);
  cs[(size_t)row * d_head + half + tt] = (float)sin(ang);
}

template <typename T>
__global__ void k_load_rows(const T* x, float* h, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    h[i] = Elt<T>::ld(x + i);
}

__device__ __forceinline__ float block_sum(float v, float* s_red) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane == 0) s_red[wave] = v;
  __syncthreads();
  float tot = 0.f;
  const int nw = blockDim.x >> 6;
  for (int w = 0; w < nw; ++w) tot += s_red[w];
  __syncthreads();
  return tot;
}

// One workgroup (1024 threads) per row, four columns per thread and pass:
// h[row] += sum_s part[s][row]; xn[row] = h * rsqrt(mean(h^2)+eps) * gain.
template <typename T>
__global__ void __launch_bounds__(1024) k_add_norm(float* h, const float* part, int S, size_t part_stride,
                                                    const T* gain, T* xn, int d, float eps) {
  __shared__ float s_red[16];
  const int row = blockIdx.x;
  float* hr = h + (size_t)row * d;
  float ss = 0.f;
  for (int c = threadIdx.x * 4; c < d; c += blockDim.x * 4) {
    f32x4_t v = *reinterpret_cast<const f32x4_t*>(hr + c);
    if (part) {
      f32x4_t a = {0.f, 0.f, 0.f, 0.f};
      for (int s = 0; s < S; ++s)
        a += *reinterpret_cast<const f32x4_t*>(part + (size_t)s * part_stride + (size_t)row * d + c);
      v += a;
      *reinterpret_cast<f32x4_t*>(hr + c) = v;
    }
    ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
  const float tot = block_sum(ss, s_red);
  const float scale = rsqrtf(tot / (float)d + eps);
  for (int c = threadIdx.x * 4; c < d; c += blockDim.x * 4) {
    const f32x4_t v = *reinterpret_cast<const f32x4_t*>(hr + c);
#pragma unroll
    for (int i = 0; i < 4; ++i) Elt<T>::st(xn + (size_t)row * d + c + i, v[i] * scale * Elt<T>::ld(gain + c + i));
  }
}

// One workgroup per (row, head) over the projection's columns: n_q query heads, n_kv key
// heads, n_kv value heads.  Query and key heads are rotated (half-split pairing: t with
// t + d_head/2); value heads are copied.  Keys and values go to the node's cache slot.
template <typename T>
__global__ void __launch_bounds__(64) k_rope_kv(const float* part, int S, size_t part_stride, const RowInfo* rows,
                                                 const float* cs, T* qbuf, KvGeom g, int layer, int n_q, int n_kv,
                                                 int d_head) {
  const int row = blockIdx.x, head = blockIdx.y;
  const int half = d_head >> 1;
  const int N = (n_q + 2 * n_kv) * d_head;
  const RowInfo ri = rows[row];
  const size_t slot = (size_t)(ri.base + ri.P + ri.node);
  const float* pr = part + (size_t)row * N + (size_t)head * d_head;
  if (head < n_q + n_kv) {
    const float* c = cs + (size_t)row * d_head;
    T* dst = head < n_q
                 ? qbuf + ((size_t)row * n_q + head) * d_head
                 : reinterpret_cast<T*>(g.kv + ((size_t)(layer * 2 + 0) * n_kv + (head - n_q)) * g.plane_bytes +
                                        slot * g.row_bytes);
    for (int t = threadIdx.x; t < half; t += blockDim.x) {
      float a = 0.f, bb = 0.f;
      for (int s = 0; s < S; ++s) {
        a += pr[(size_t)s * part_stride + t];
        bb += pr[(size_t)s * part_stride + half + t];
      }
      const float co = c[t], si = c[half + t];
      Elt<T>::st(dst + t, a * co - bb * si);
      Elt<T>::st(dst + half + t, bb * co + a * si);
    }
  } else {
    T* dst = reinterpret_cast<T*>(g.kv + ((size_t)(layer * 2 + 1) * n_kv + (head - n_q - n_kv)) * g.plane_bytes +
                                  slot * g.row_bytes);
    for (int t = threadIdx.x; t < d_head; t += blockDim.x) {
      float a = 0.f;
      for (int s = 0; s < S; ++s) a += pr[(size_t)s * part_stride + t];
      Elt<T>::st(dst + t, a);
    }
  }
}

template <typename T>
__global__ void k_silu_mul(const float* gu, T* act, int M, int F) {
  const size_t n = (size_t)M * F;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const size_t m = i / F, f = i - m * F;
    const float gte = gu[m * 2 * F + f], up = gu[m * 2 * F + F + f];
    Elt<T>::st(act + i, gte / (1.f + __expf(-gte)) * up);
  }
}

template <typename T>
__global__ void k_finish(const float* h, const float* part, int S, size_t part_stride, T* out, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    float v = h[i];
    for (int s = 0; s < S; ++s) v += part[(size_t)s * part_stride + i];
    Elt<T>::st(out + i, v);
  }
}

// ---- launchers -------------------------------------------------------------------
static inline int grid_for(size_t n, int block, int cap = 4096) {
  size_t g = (n + block - 1) / block;
  if (g < 1) g = 1;
  if (g > (size_t)cap) g = cap;
  return (int)g;
}

hipError_t sp_launch_prep_rows(const FwdBatch& b, const ReqMeta* meta, const ReqTables* tables, RowInfo* rows,
                               float* cs, int d_head, float theta, hipStream_t st) {
  const int n = b.n_rows * (d_head / 2);
  hipLaunchKernelGGL(k_prep_rows, dim3((n + 255) / 256), dim3(256), 0, st, b, meta, tables, rows, cs, d_head, theta);
  return hipGetLastError();
}

hipError_t sp_launch_load_rows(int dtype, const void* x, float* h, size_t n, hipStream_t st) {
  if (dtype == 0) hipLaunchKernelGGL(k_load_rows<float>, dim3(grid_for(n, 256)), dim3(256), 0, st, (const float*)x, h, n);
  else hipLaunchKernelGGL(k_load_rows<bf16_t>, dim3(grid_for(n, 256)), dim3(256), 0, st, (const bf16_t*)x, h, n);
  return hipGetLastError();
}

hipError_t sp_launch_add_norm(int dtype, float* h, const float* part, int S, size_t part_stride, const void* gain,
                              void* xn, int M, int d, float eps, hipStream_t st) {
  if (dtype == 0)
    hipLaunchKernelGGL(k_add_norm<float>, dim3(M), dim3(1024), 0, st, h, part, S, part_stride, (const float*)gain,
                       (float*)xn, d, eps);
  else
    hipLaunchKernelGGL(k_add_norm<bf16_t>, dim3(M), dim3(1024), 0, st, h, part, S, part_stride, (const bf16_t*)gain,
                       (bf16_t*)xn, d, eps);
  return hipGetLastError();
}

hipError_t sp_launch_rope_kv(int dtype, const float* part, int S, size_t part_stride, const RowInfo* rows,
                             const float* cs, void* qbuf, KvGeom g, int layer, int M, int n_q, int n_kv, int d_head,
                             hipStream_t st) {
  if (dtype == 0)
    hipLaunchKernelGGL(k_rope_kv<float>, dim3(M, n_q + 2 * n_kv), dim3(64), 0, st, part, S, part_stride, rows, cs, (float*)qbuf, g,
                       layer, n_q, n_kv, d_head);
  else
    hipLaunchKernelGGL(k_rope_kv<bf16_t>, dim3(M, n_q + 2 * n_kv), dim3(64), 0, st, part, S, part_stride, rows, cs, (bf16_t*)qbuf,
                       g, layer, n_q, n_kv, d_head);
  return hipGetLastError();
}

hipError_t sp_launch_silu_mul(int dtype, const float* gu, void* act, int M, int F, hipStream_t st) {
  const size_t n = (size_t)M * F;
  if (dtype == 0) hipLaunchKernelGGL(k_silu_mul<float>, dim3(grid_for(n, 256)), dim3(256), 0, st, gu, (float*)act, M, F);
  else hipLaunchKernelGGL(k_silu_mul<bf16_t>, dim3(grid_for(n, 256)), dim3(256), 0, st, gu, (bf16_t*)act, M, F);
  return hipGetLastError();
}

hipError_t sp_launch_finish(int dtype, const float* h, const float* part, int S, size_t part_stride, void* out,
                            int M, int d, hipStream_t st) {
  const size_t n = (size_t)M * d;
  if (dtype == 0)
    hipLaunchKernelGGL(k_finish<float>, dim3(grid_for(n, 256)), dim3(256), 0, st, h, part, S, part_stride,
                       (float*)out, n);
  else
    hipLaunchKernelGGL(k_finish<bf16_t>, dim3(grid_for(n, 256)), dim3(256), 0, st, h, part, S, part_stride,
                       (bf16_t*)out, n);
  return hipGetLastError();
}
