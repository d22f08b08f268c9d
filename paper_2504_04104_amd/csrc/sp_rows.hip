// Row-wise pieces of the decoder layer (Llama family: Sec. 2.1, Sec. 4 "Testbed"):
// row descriptors and rotary tables, residual add + RMSNorm, RoPE + KV append,
// SiLU*mul, and the final write-out.  The projections leave their results as
// float32 partial sums [S][M][N]; the kernels here fold the S slices in.
#include "sp_launch.h"

// Four consecutive elements of the storage type to and from float.
template <typename T> struct Vec4;
template <> struct Vec4<float> {
  static __device__ __forceinline__ f32x4_t ld(const float* p) { return *reinterpret_cast<const f32x4_t*>(p); }
  static __device__ __forceinline__ void st(float* p, f32x4_t v) { *reinterpret_cast<f32x4_t*>(p) = v; }
};
template <> struct Vec4<bf16_t> {
  static __device__ __forceinline__ f32x4_t ld(const bf16_t* p) {
    const uint2 u = *reinterpret_cast<const uint2*>(p);
    return (f32x4_t){bf16_lo(u.x), bf16_hi(u.x), bf16_lo(u.y), bf16_hi(u.y)};
  }
  static __device__ __forceinline__ void st(bf16_t* p, f32x4_t v) {
    uint2 u;
    u.x = pack_bf16x2(v[0], v[1]);
    u.y = pack_bf16x2(v[2], v[3]);
    *reinterpret_cast<uint2*>(p) = u;
  }
};

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

// Folds S partial slices into four columns: all loads are issued before the first add.
__device__ __forceinline__ f32x4_t fold4(const float* p, int S, size_t stride) {
  f32x4_t a = {0.f, 0.f, 0.f, 0.f};
  int s = 0;
  for (; s + 4 <= S; s += 4) {
    const f32x4_t v0 = *reinterpret_cast<const f32x4_t*>(p + (size_t)s * stride);
    const f32x4_t v1 = *reinterpret_cast<const f32x4_t*>(p + (size_t)(s + 1) * stride);
    const f32x4_t v2 = *reinterpret_cast<const f32x4_t*>(p + (size_t)(s + 2) * stride);
    const f32x4_t v3 = *reinterpret_cast<const f32x4_t*>(p + (size_t)(s + 3) * stride);
    a += (v0 + v1) + (v2 + v3);
  }
  for (; s < S; ++s) a += *reinterpret_cast<const f32x4_t*>(p + (size_t)s * stride);
  return a;
}

// One workgroup (1024 threads) per row, four columns per thread and pass.
//   FIRST: the row enters the stage: h[row] = x[row]; the row's descriptor and its rotary
//          table are written as well.  Position of a node = prefix length + depth: each tree
//          level is one future position (Sec. 3.2).  The angle is formed in double so that
//          positions of tens of thousands keep full float accuracy in cos and sin.
//   else:  h[row] += sum_s part[s][row].
// Then xn[row] = h * rsqrt(mean(h^2)+eps) * gain.  The first two passes stay in registers.
struct NoPlan { int unused; };
template <bool FIRST> struct PlanArg { typedef NoPlan type; };
template <> struct PlanArg<true> { typedef AttnPlan type; };

template <typename T, bool FIRST>
__global__ void __launch_bounds__(1024) k_add_norm(float* h, const float* part, int S, size_t part_stride,
                                                    const T* gain, T* xn, int d, float eps, const T* x,
                                                    typename PlanArg<FIRST>::type b, AttnPlan* plan_dev,
                                                    const ReqMeta* meta, const ReqTables* tables, RowInfo* rows,
                                                    float* cs, int d_head, float theta) {
  __shared__ float s_red[16];
  const int row = blockIdx.x;
  if constexpr (FIRST) {
    // the call's plan goes to device memory for the kernels that follow
    if (plan_dev && row == 0) {
      const uint32_t* src = reinterpret_cast<const uint32_t*>(&b);
      uint32_t* dst = reinterpret_cast<uint32_t*>(plan_dev);
      for (int i = threadIdx.x; i < (int)(sizeof(AttnPlan) / 4); i += blockDim.x) dst[i] = src[i];
    }
    const int half = d_head >> 1;
    if ((int)threadIdx.x < half) {
      const int tt = threadIdx.x;
      int seg = 0;
      while (seg + 1 < b.n_seg && row >= b.seg_row0[seg + 1]) ++seg;
      const int req = b.seg_req[seg];
      const int node = b.seg_first[seg] + (row - b.seg_row0[seg]);
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
  }
  float* hr = h + (size_t)row * d;
  const int c0 = threadIdx.x * 4, step = blockDim.x * 4;
  f32x4_t keep[2];
  float ss = 0.f;
#define SP_ROW_VALUE(c, v)                                                             \
  if (FIRST) {                                                                         \
    v = Vec4<T>::ld(x + (size_t)row * d + (c));                                        \
    *reinterpret_cast<f32x4_t*>(hr + (c)) = v;                                         \
  } else {                                                                             \
    v = *reinterpret_cast<const f32x4_t*>(hr + (c));                                   \
    v += fold4(part + (size_t)row * d + (c), S, part_stride);                          \
    *reinterpret_cast<f32x4_t*>(hr + (c)) = v;                                         \
  }                                                                                    \
  ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int c = c0 + p * step;
    if (c < d) { f32x4_t v; SP_ROW_VALUE(c, v) keep[p] = v; }
  }
  for (int c = c0 + 2 * step; c < d; c += step) { f32x4_t v; SP_ROW_VALUE(c, v) }
#undef SP_ROW_VALUE
  const float tot = block_sum(ss, s_red);
  const float scale = rsqrtf(tot / (float)d + eps);
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int c = c0 + p * step;
    if (c < d) Vec4<T>::st(xn + (size_t)row * d + c, keep[p] * scale * Vec4<T>::ld(gain + c));
  }
  for (int c = c0 + 2 * step; c < d; c += step)
    Vec4<T>::st(xn + (size_t)row * d + c, *reinterpret_cast<const f32x4_t*>(hr + c) * scale * Vec4<T>::ld(gain + c));
}

// Threads work in groups of d_head/8, one group per (row, head) over the projection's
// columns: n_q query heads, n_kv key heads, n_kv value heads; a thread owns four pairs
// (t, t + d_head/2).  Query and key heads are rotated (half-split pairing); value heads are
// copied.  Keys and values go to the node's cache slot.
template <typename T>
__global__ void __launch_bounds__(256) k_rope_kv(const float* part, int S, size_t part_stride, const RowInfo* rows,
                                                  const float* cs, T* qbuf, KvGeom g, int layer, int n_q, int n_kv,
                                                  int d_head) {
  const int half = d_head >> 1, tph = half >> 2;
  const int row = blockIdx.x;
  const int head = blockIdx.y * (256 / tph) + threadIdx.x / tph;
  if (head >= n_q + 2 * n_kv) return;
  const int t = (threadIdx.x % tph) * 4;
  const int N = (n_q + 2 * n_kv) * d_head;
  const RowInfo ri = rows[row];
  const size_t slot = sp_phys_slot(g, ri.req, ri.base, ri.P + ri.node);
  const float* pr = part + (size_t)row * N + (size_t)head * d_head;
  const f32x4_t a = fold4(pr + t, S, part_stride), bb = fold4(pr + half + t, S, part_stride);
  if (head < n_q + n_kv) {
    const float* c = cs + (size_t)row * d_head;
    const f32x4_t co = *reinterpret_cast<const f32x4_t*>(c + t), si = *reinterpret_cast<const f32x4_t*>(c + half + t);
    T* dst = head < n_q
                 ? qbuf + ((size_t)row * n_q + head) * d_head
                 : reinterpret_cast<T*>(g.kv + ((size_t)(layer * 2 + 0) * n_kv + (head - n_q)) * g.plane_bytes +
                                        slot * g.row_bytes);
    Vec4<T>::st(dst + t, a * co - bb * si);
    Vec4<T>::st(dst + half + t, bb * co + a * si);
  } else {
    T* dst = reinterpret_cast<T*>(g.kv + ((size_t)(layer * 2 + 1) * n_kv + (head - n_q - n_kv)) * g.plane_bytes +
                                  slot * g.row_bytes);
    Vec4<T>::st(dst + t, a);
    Vec4<T>::st(dst + half + t, bb);
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
  for (size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; i < n; i += (size_t)gridDim.x * blockDim.x * 4)
    Vec4<T>::st(out + i, *reinterpret_cast<const f32x4_t*>(h + i) + fold4(part + i, S, part_stride));
}

// Top-1 token of each row (Sec. 3.4) from either the per-tile (value, index) pairs the
// output-head kernel left (PAIRS) or plain logits [rows][n_items]; the lowest index among
// equal maxima.  Also stores it as the node's prediction in the request's tables.
template <bool PAIRS>
__global__ void __launch_bounds__(256) k_argmax_rows(const float* part, int n_items, FwdBatch b, ReqTables* tables,
                                                      int* pred_out, float* max_out) {
  __shared__ float s_v[4];
  __shared__ int s_i[4];
  const int row = blockIdx.x;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  for (int t = threadIdx.x; t < n_items; t += blockDim.x) {
    float v;
    int i;
    if (PAIRS) {
      const float* p = part + ((size_t)row * n_items + t) * 2;
      v = p[0];
      i = reinterpret_cast<const int*>(p)[1];
    } else {
      v = part[(size_t)row * n_items + t];
      i = t;
    }
    if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(bv, off, 64);
    const int oi = __shfl_xor(bi, off, 64);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane == 0) { s_v[wave] = bv; s_i[wave] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < 4; ++w)
      if (s_v[w] > bv || (s_v[w] == bv && s_i[w] < bi)) { bv = s_v[w]; bi = s_i[w]; }
    if (pred_out) pred_out[row] = bi;
    if (max_out) max_out[row] = bv;
    int seg = 0;
    while (seg + 1 < b.n_req && row >= b.row0[seg + 1]) ++seg;
    tables[b.req[seg]].pred[b.first[seg] + (row - b.row0[seg])] = bi;
  }
}

// ---- launchers -------------------------------------------------------------------
static inline int grid_for(size_t n, int block, int cap = 4096) {
  size_t g = (n + block - 1) / block;
  if (g < 1) g = 1;
  if (g > (size_t)cap) g = cap;
  return (int)g;
}

hipError_t sp_launch_enter_norm(int dtype, const void* x, const AttnPlan& plan, AttnPlan* plan_dev,
                                const ReqMeta* meta, const ReqTables* tables, RowInfo* rows, float* cs, int d_head,
                                float theta, float* h, const void* gain, void* xn, int M, int d, float eps,
                                hipStream_t st) {
  static_assert(sizeof(AttnPlan) % 4 == 0 && sizeof(AttnPlan) < 3900, "the plan travels as a kernel argument");
  if (dtype == 0)
    hipLaunchKernelGGL((k_add_norm<float, true>), dim3(M), dim3(1024), 0, st, h, nullptr, 0, 0, (const float*)gain,
                       (float*)xn, d, eps, (const float*)x, plan, plan_dev, meta, tables, rows, cs, d_head, theta);
  else
    hipLaunchKernelGGL((k_add_norm<bf16_t, true>), dim3(M), dim3(1024), 0, st, h, nullptr, 0, 0,
                       (const bf16_t*)gain, (bf16_t*)xn, d, eps, (const bf16_t*)x, plan, plan_dev, meta, tables, rows,
                       cs, d_head, theta);
  return hipGetLastError();
}

hipError_t sp_launch_add_norm(int dtype, float* h, const float* part, int S, size_t part_stride, const void* gain,
                              void* xn, int M, int d, float eps, hipStream_t st) {
  const NoPlan none{0};
  if (dtype == 0)
    hipLaunchKernelGGL((k_add_norm<float, false>), dim3(M), dim3(1024), 0, st, h, part, S, part_stride,
                       (const float*)gain, (float*)xn, d, eps, nullptr, none, nullptr, nullptr, nullptr, nullptr,
                       nullptr, 0, 0.f);
  else
    hipLaunchKernelGGL((k_add_norm<bf16_t, false>), dim3(M), dim3(1024), 0, st, h, part, S, part_stride,
                       (const bf16_t*)gain, (bf16_t*)xn, d, eps, nullptr, none, nullptr, nullptr, nullptr, nullptr,
                       nullptr, 0, 0.f);
  return hipGetLastError();
}

hipError_t sp_launch_argmax_rows(bool pairs, const float* part, int n_items, const FwdBatch& b, ReqTables* tables,
                                 int* pred_out, float* max_out, hipStream_t st) {
  if (pairs) hipLaunchKernelGGL(k_argmax_rows<true>, dim3(b.n_rows), dim3(256), 0, st, part, n_items, b, tables, pred_out, max_out);
  else hipLaunchKernelGGL(k_argmax_rows<false>, dim3(b.n_rows), dim3(256), 0, st, part, n_items, b, tables, pred_out, max_out);
  return hipGetLastError();
}

hipError_t sp_launch_rope_kv(int dtype, const float* part, int S, size_t part_stride, const RowInfo* rows,
                             const float* cs, void* qbuf, KvGeom g, int layer, int M, int n_q, int n_kv, int d_head,
                             hipStream_t st) {
  const int heads_per_block = 256 / (d_head / 8);
  const dim3 grid(M, (n_q + 2 * n_kv + heads_per_block - 1) / heads_per_block);
  if (dtype == 0)
    hipLaunchKernelGGL(k_rope_kv<float>, grid, dim3(256), 0, st, part, S, part_stride, rows, cs, (float*)qbuf, g,
                       layer, n_q, n_kv, d_head);
  else
    hipLaunchKernelGGL(k_rope_kv<bf16_t>, grid, dim3(256), 0, st, part, S, part_stride, rows, cs, (bf16_t*)qbuf,
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
    hipLaunchKernelGGL(k_finish<float>, dim3(grid_for(n / 4, 256)), dim3(256), 0, st, h, part, S, part_stride,
                       (float*)out, n);
  else
    hipLaunchKernelGGL(k_finish<bf16_t>, dim3(grid_for(n / 4, 256)), dim3(256), 0, st, h, part, S, part_stride,
                       (bf16_t*)out, n);
  return hipGetLastError();
}
