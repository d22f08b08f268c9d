// Lossy verification at the last stage (Sec. 3.4, "Lossless and Lossy Acceleration"):
//   (1) relaxed: of the root's children, the one whose token the large model finds most
//       probable -- some child is always verified, the pipeline never stalls;
//   (2) top-p:   children whose token lies in the large model's top-p set (tokens in descending
//       probability, the shortest prefix whose mass reaches p) are acceptable; the one with the
//       highest draft probability wins; none acceptable = a miss as in the lossless case.
// Equal probabilities are ordered by ascending token id, equal candidates by ascending node.
//
// Input: one row of logits per request (the root's output through the final norm and the
// vocabulary matrix).  A token t is in the top-p set iff the mass of the tokens in front of it,
//   before(t) = sum over { v : l_v > l_t  or  (l_v == l_t and v < t) } of softmax(l)_v,
// is below p.  k_lossy_slices cuts the vocabulary into slices of SLICE tokens, one workgroup
// each: slice maximum and its first index, sum of exp(l - slice max), and, one thread per
// candidate, the slice's share of before(token of the candidate).  k_lossy_decide rescales and
// adds the slices in order (so the result does not depend on timing) and decides.
#include "sp_launch.h"

#define SLICE 2048

template <typename T>
__global__ void __launch_bounds__(1024) k_row_norm(const T* __restrict__ x, const T* __restrict__ gain,
                                                    T* __restrict__ xn, int d, float eps) {
  __shared__ float s_red[16];
  const int row = blockIdx.x;
  const T* xr = x + (size_t)row * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += 1024) { const float v = Elt<T>::ld(xr + c); ss += v * v; }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) tot += s_red[w];
  const float rs = rsqrtf(tot / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += 1024)
    Elt<T>::st(xn + (size_t)row * d + c, Elt<T>::ld(xr + c) * rs * Elt<T>::ld(gain + c));
}

// The root's children in node order: s_node[0..nc), their tokens in s_tok.  Called by all 256 threads.
__device__ __forceinline__ int root_children(const ReqTables& t, int T, int* s_node, int* s_tok, int* s_wcount) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const bool is = tid < T && t.parent[tid] == -1;
  const unsigned long long bal = __ballot(is);
  if (lane == 0) s_wcount[wave] = __popcll(bal);
  __syncthreads();
  int before = 0;
  for (int w = 0; w < wave; ++w) before += s_wcount[w];
  if (is) {
    const int pos = before + __popcll(bal & ((1ull << lane) - 1ull));
    s_node[pos] = tid;
    s_tok[pos] = t.token[tid];
  }
  const int nc = s_wcount[0] + s_wcount[1] + s_wcount[2] + s_wcount[3];
  __syncthreads();
  return nc;
}

struct LossyBatch {
  int n, mode, V, n_slices;
  float top_p;
  int req[SP_BATCH];
};

// stats[item][slice] = (slice max, sum of exp(l - max), first index of the max as int bits, 0);
// before[item][slice][j] = sum over the slice's tokens in front of candidate j's token of exp(l - slice max).
__global__ void __launch_bounds__(256) k_lossy_slices(const ReqMeta* meta, const ReqTables* tables,
                                                       const float* __restrict__ logits, LossyBatch b, float* stats,
                                                       float* before) {
  __shared__ __attribute__((aligned(16))) float s_l[SLICE];
  __shared__ __attribute__((aligned(16))) float s_e[SLICE + 256];   // + the partial sums of the candidate pass
  __shared__ int s_node[SP_T], s_tok[SP_T], s_wcount[4];
  __shared__ float s_rv[4];
  __shared__ int s_ri[4];
  const int item = blockIdx.y, slice = blockIdx.x;
  const int req = b.req[item];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float* L = logits + (size_t)item * b.V;
  const int v0 = slice * SLICE, len = min(SLICE, b.V - v0);
  const int nc = root_children(tables[req], meta[req].T, s_node, s_tok, s_wcount);

  float bv = -INFINITY;
  int bi = 0x7fffffff;
  {
    float lv[SLICE / 256];                             // all loads first: one memory round trip, not eight
#pragma unroll
    for (int u = 0; u < SLICE / 256; ++u) lv[u] = (tid + u * 256 < len) ? L[v0 + tid + u * 256] : -INFINITY;
#pragma unroll
    for (int u = 0; u < SLICE / 256; ++u) {
      const int i = tid + u * 256;
      if (i < len) {
        s_l[i] = lv[u];
        if (lv[u] > bv) { bv = lv[u]; bi = v0 + i; }   // ascending i: the first of equal maxima stays
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(bv, off, 64);
    const int oi = __shfl_xor(bi, off, 64);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
  }
  if (lane == 0) { s_rv[wave] = bv; s_ri[wave] = bi; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < 4; ++w)
    if (s_rv[w] > bv || (s_rv[w] == bv && s_ri[w] < bi)) { bv = s_rv[w]; bi = s_ri[w]; }
  __syncthreads();
  float z = 0.f;
  for (int i = tid; i < len; i += 256) {
    const float e = expf(s_l[i] - bv);
    s_e[i] = e;
    z += e;
  }
  z = wave_sum(z);
  if (lane == 0) s_rv[wave] = z;
  __syncthreads();
  if (tid == 0) {
    float* st = stats + ((size_t)item * b.n_slices + slice) * 4;
    st[0] = bv;
    st[1] = (s_rv[0] + s_rv[1]) + (s_rv[2] + s_rv[3]);
    reinterpret_cast<int*>(st)[2] = bi;
    st[3] = 0.f;
  }
  // Candidate against every token of the slice.  Up to 64 candidates: lane = candidate, and the four
  // waves take a quarter of the slice each; up to 128: two halves; else one wave per 64 candidates.
  // All lanes of a wave read the same LDS words (a broadcast), four tokens per read.  The parts are
  // added in order afterwards, so the sum does not depend on timing.
  __syncthreads();
  const int groups = nc <= 64 ? 1 : (nc <= 128 ? 2 : 4), parts = 4 / groups;
  const int cand = (wave / parts) * 64 + lane, part = wave % parts;
  float* s_part = s_e + SLICE;                       // [4][64] partial sums, behind the exponentials
  {
    float acc = 0.f;
    const int tk = cand < nc ? s_tok[cand] : -1;
    if (tk >= 0 && tk < b.V) {
      const float thr = L[tk];
      const int rel = tk - v0;                       // tokens of the slice with index < rel come first among equals
      const int per = ((len + parts - 1) / parts + 3) & ~3;
      const int i0 = part * per, i1 = min(i0 + per, len);
      int i = i0;
      for (; i + 4 <= i1; i += 4) {
        const f32x4_t l4 = *reinterpret_cast<const f32x4_t*>(&s_l[i]);
        const f32x4_t e4 = *reinterpret_cast<const f32x4_t*>(&s_e[i]);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc += (l4[u] > thr || (l4[u] == thr && i + u < rel)) ? e4[u] : 0.f;
      }
      for (; i < i1; ++i) acc += (s_l[i] > thr || (s_l[i] == thr && i < rel)) ? s_e[i] : 0.f;
    }
    s_part[wave * 64 + lane] = acc;
  }
  __syncthreads();
  if (tid < nc) {
    const int g0 = (tid >> 6) * parts;               // first wave of the candidate's group
    float acc = 0.f;
    for (int q = 0; q < parts; ++q) acc += s_part[(g0 + q) * 64 + (tid & 63)];
    before[((size_t)item * b.n_slices + slice) * SP_T + tid] = acc;
  }
}

// out[2*item] = verified node or -1, out[2*item+1] = the model's top-1 token, which also becomes the
// root's stored prediction (what a miss falls back to).
__global__ void __launch_bounds__(256) k_lossy_decide(ReqMeta* meta, const ReqTables* tables,
                                                       const float* __restrict__ logits, LossyBatch b,
                                                       const float* stats, const float* before, int* out) {
  __shared__ int s_node[SP_T], s_tok[SP_T], s_wcount[4];
  __shared__ float s_key[SP_T];          // relaxed: the candidate's logit; top-p: its draft probability
  __shared__ unsigned char s_ok[SP_T];
  const int item = blockIdx.x, req = b.req[item], tid = threadIdx.x;
  const ReqTables& t = tables[req];
  const float* L = logits + (size_t)item * b.V;
  const int nc = root_children(t, meta[req].T, s_node, s_tok, s_wcount);
  const float* st = stats + (size_t)item * b.n_slices * 4;
  // slice maxima -> the row's maximum and its first index; then each slice's factor exp(max_s - max)
  __shared__ float s_sc[256], s_z[256];
  __shared__ int s_top1;
  __shared__ float s_m;
  {
    // thread s takes slices s, s+256, ...; then the 256 candidates are folded in order by thread 0
    float mv = -INFINITY;
    int mi = 0x7fffffff;
    for (int s0 = tid; s0 < b.n_slices; s0 += 256) {
      const float v = st[s0 * 4];
      const int i = reinterpret_cast<const int*>(st)[s0 * 4 + 2];
      if (v > mv || (v == mv && i < mi)) { mv = v; mi = i; }
    }
    s_sc[tid] = mv;
    reinterpret_cast<int*>(s_z)[tid] = mi;
    __syncthreads();
    if (tid == 0) {
      float m = -INFINITY;
      int top1 = 0x7fffffff;
      const int lim = min(256, b.n_slices);
      for (int q = 0; q < lim; ++q) {
        const float v = s_sc[q];
        const int i = reinterpret_cast<const int*>(s_z)[q];
        if (v > m || (v == m && i < top1)) { m = v; top1 = i; }
      }
      s_m = m; s_top1 = top1;
    }
  }
  __syncthreads();
  const float m = s_m;
  const int top1 = s_top1;
  float Z = 0.f, bf = 0.f;
  const bool mine = tid < nc;
  const int tk = mine ? s_tok[tid] : -1;
  const bool valid = tk >= 0 && tk < b.V;
  for (int s0 = 0; s0 < b.n_slices; s0 += 256) {     // blocks of 256 slices (one is the rule)
    const int ns = min(256, b.n_slices - s0);
    __syncthreads();
    if (tid < ns) {
      s_sc[tid] = expf(st[(s0 + tid) * 4] - m);
      s_z[tid] = st[(s0 + tid) * 4 + 1];
    }
    __syncthreads();
    if (mine && b.mode == 2) {
      const float* bp = before + ((size_t)item * b.n_slices + s0) * SP_T + tid;
      int q = 0;
      for (; q + 8 <= ns; q += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = bp[(size_t)(q + u) * SP_T];
#pragma unroll
        for (int u = 0; u < 8; ++u) { Z += s_z[q + u] * s_sc[q + u]; bf += v[u] * s_sc[q + u]; }
      }
      for (; q < ns; ++q) { Z += s_z[q] * s_sc[q]; bf += bp[(size_t)q * SP_T] * s_sc[q]; }
    }
  }
  if (mine) {
    if (b.mode == 1) {
      s_ok[tid] = valid;
      s_key[tid] = valid ? L[tk] : -INFINITY;
    } else {
      s_ok[tid] = valid && bf < b.top_p * Z;
      s_key[tid] = t.prob[s_node[tid]];
    }
  }
  __syncthreads();
  if (tid == 0) {
    int best = -1;
    float bk = -INFINITY;
    for (int j = 0; j < nc; ++j)
      if (s_ok[j] && (best < 0 || s_key[j] > bk)) { best = s_node[j]; bk = s_key[j]; }
    out[2 * item] = best;
    out[2 * item + 1] = top1;
    meta[req].root_pred = top1;
  }
}

// ---------------------------------------------------------------------------------------------
// Stochastic verification (Sec. 4.3, "Stochastic Decoding"): the token after the root is drawn from
// the large model's distribution at temperature T, among the candidates collected in descending
// probability until their probabilities sum to top_p or top_k of them have been taken (equal
// probabilities by ascending token id); the draw is the inverse CDF of the candidates' renormalised
// probabilities at a uniform number the caller supplies.  The drawn token takes the place of the
// top-1 token: it becomes the root's prediction, and the verified node is the first root child that
// carries it (-1: a stall).
// One workgroup of 1024 threads per request: row maximum, normaliser over the whole vocabulary, the
// top_k-th largest logit by a radix select over the order-preserving bit pattern (four passes of 8
// bits, one histogram per wave), an index-ordered gather of the logits above it and of the first
// ones equal to it, a sort by counting, and the running sums by one thread.
struct SampleBatch {
  int n, V, top_k;
  float inv_T, top_p;
  int req[SP_BATCH];
  float u[SP_BATCH];
};

__device__ __forceinline__ uint32_t order_key(float f) {           // ascending like the floats themselves
  const uint32_t b = __float_as_uint(f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Eight loads of W floats per thread, all issued before the first use: one workgroup reads the whole row, so
// with a load per iteration a pass would be a chain of V / 1024 memory latencies.  W = 4 needs V % 4 == 0
// (then an index below V is followed by three more).  Index of element (u, c): base + (u * 1024 + tid) * W + c.
template <int W>
__device__ __forceinline__ void sample_load(const float* __restrict__ L, int V, int base, int tid, float (&v)[8][W]) {
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int i = base + (u * 1024 + tid) * W;
    if constexpr (W == 4) {
      const float4 t = i < V ? *reinterpret_cast<const float4*>(L + i) : make_float4(0.f, 0.f, 0.f, 0.f);
      v[u][0] = t.x; v[u][1] = t.y; v[u][2] = t.z; v[u][3] = t.w;
    } else {
      v[u][0] = i < V ? L[i] : 0.f;
    }
  }
}

#define SP_SAMPLE_CAND 2048   // candidates the short path can hold

// One workgroup per request.  The K = top_k largest logits are found without ordering the row: every thread
// keeps the maximum of the elements it reads, a wave takes the ceil(K / 16) largest of its 64 thread maxima,
// and the smallest of those 16 * ceil(K / 16) >= K distinct elements is a lower bound t0 of the K-th largest
// logit.  A second pass collects the elements >= t0 (a few hundred on a spread-out row) and their places follow
// from counting.  Rows that defeat the bound (long runs of equal logits, vocabularies under a few thousand)
// take a radix selection over the whole row instead.
template <int W>
__global__ void __launch_bounds__(1024) k_sample_decide(ReqMeta* meta, const ReqTables* tables,
                                                         const float* __restrict__ logits, SampleBatch b, int* out) {
  __shared__ float s_f[16], s_g[16];
  __shared__ unsigned s_hist[16][256];
  __shared__ unsigned s_scan[16];
  __shared__ unsigned s_pick[2];                  // digit chosen by a pass, and how many of the top_k are still to find below it
  __shared__ uint32_t s_key[SP_SAMPLE_MAX_K], s_skey[SP_SAMPLE_MAX_K];
  __shared__ int s_idx[SP_SAMPLE_MAX_K], s_sidx[SP_SAMPLE_MAX_K];
  __shared__ uint32_t s_ckey[SP_SAMPLE_CAND];
  __shared__ int s_cidx[SP_SAMPLE_CAND];
  __shared__ unsigned s_ncand;
  __shared__ int s_tok, s_best;
  const int item = blockIdx.x, req = b.req[item];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float* L = logits + (size_t)item * b.V;
  const int V = b.V, K = min(b.top_k, V);

  // first pass: thread maxima, from them the row maximum and the bound t0
  float tm = -INFINITY;
  for (int base = 0; base < V; base += 8 * 1024 * W) {
    float v[8][W];
    sample_load<W>(L, V, base, tid, v);
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (base + (u * 1024 + tid) * W < V) {
#pragma unroll
        for (int c = 0; c < W; ++c) tm = fmaxf(tm, v[u][c]);
      }
  }
  {
    const float wmx = wave_max(tm);
    float cur = tm, kept = wmx;
    const int rounds = (K + 15) >> 4;
    for (int r = 0; r < rounds; ++r) {           // the wave's r-th largest thread maximum, one thread retired per round
      kept = wave_max(cur);
      const unsigned long long holders = __ballot(cur == kept);
      if (holders == 0ull) { kept = -INFINITY; break; }          // only NaNs left
      if (lane == (int)__builtin_ctzll(holders)) cur = -INFINITY;
    }
    if (lane == 0) { s_f[wave] = wmx; s_g[wave] = kept; }
    if (tid == 0) s_ncand = 0u;
  }
  __syncthreads();
  float mx = s_f[0], t0 = s_g[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) { mx = fmaxf(mx, s_f[w]); t0 = fminf(t0, s_g[w]); }
  __syncthreads();

  // second pass: the normaliser of softmax(l / T) over the whole vocabulary, added in a fixed order, and the candidates
  float z = 0.f;
  for (int base = 0; base < V; base += 8 * 1024 * W) {
    float v[8][W];
    sample_load<W>(L, V, base, tid, v);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = base + (u * 1024 + tid) * W;
      if (i < V) {
#pragma unroll
        for (int c = 0; c < W; ++c) {
          z += expf((v[u][c] - mx) * b.inv_T);
          if (v[u][c] >= t0) {
            const unsigned p = atomicAdd(&s_ncand, 1u);
            if (p < SP_SAMPLE_CAND) { s_ckey[p] = order_key(v[u][c]); s_cidx[p] = i + c; }
          }
        }
      }
    }
  }
  z = wave_sum(z);
  if (lane == 0) s_f[wave] = z;
  __syncthreads();
  float Z = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) Z += s_f[w];
  const int n_cand = (int)s_ncand;

  if (n_cand <= SP_SAMPLE_CAND) {
    // descending probability, equal ones by ascending token id: a candidate's place is the number that beat it
    for (int i = tid; i < n_cand; i += 1024) {
      const uint32_t k = s_ckey[i];
      const int ix = s_cidx[i];
      int rank = 0;
      for (int j = 0; j < n_cand; ++j) rank += (s_ckey[j] > k) || (s_ckey[j] == k && s_cidx[j] < ix);
      if (rank < K) { s_skey[rank] = k; s_sidx[rank] = ix; }
    }
  } else {
    // the K-th largest key: fix its bytes from the top, counting the keys that share the bytes fixed so far
    uint32_t prefix = 0u, mask = 0u;
    unsigned need = (unsigned)K;
    for (int shift = 24; shift >= 0; shift -= 8) {
      for (int i = tid; i < 16 * 256; i += 1024) (&s_hist[0][0])[i] = 0u;
      __syncthreads();
      for (int base = 0; base < V; base += 8 * 1024 * W) {
        float v[8][W];
        sample_load<W>(L, V, base, tid, v);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if (base + (u * 1024 + tid) * W < V) {
#pragma unroll
            for (int c = 0; c < W; ++c) {
              const uint32_t k = order_key(v[u][c]);
              if ((k & mask) == prefix) atomicAdd(&s_hist[wave][(k >> shift) & 255u], 1u);
            }
          }
        }
      }
      __syncthreads();
      if (tid < 256) {
        unsigned c = 0u;
#pragma unroll
        for (int w = 0; w < 16; ++w) c += s_hist[w][tid];
        s_hist[0][tid] = c;
      }
      __syncthreads();
      if (tid == 0) {
        unsigned above = 0u;
        int bin = 255;
        for (; bin > 0; --bin) {
          if (above + s_hist[0][bin] >= need) break;
          above += s_hist[0][bin];
        }
        s_pick[0] = (unsigned)bin;
        s_pick[1] = need - above;
      }
      __syncthreads();
      prefix |= s_pick[0] << shift;
      mask |= 255u << shift;
      need = s_pick[1];
      __syncthreads();
    }
    const uint32_t kth = prefix;                    // `need` of the keys equal to it belong to the top K: those with the lowest index
    const int n_gt = K - (int)need;

    // gather in index order: wave w owns the indices [w * seg, (w + 1) * seg) and reads them 64 at a time, so a
    // candidate's place is the count of the waves in front, of the rows in front and of the lower lanes of its row
    const int seg = (((V + 15) >> 4) + 63) & ~63;
    const int w0 = min(wave * seg, V), w1 = min(w0 + seg, V);
    unsigned c_gt = 0u, c_eq = 0u;                  // wave-uniform
    for (int r0 = w0; r0 < w1; r0 += 16 * 64) {
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) { const int i = r0 + u * 64 + lane; v[u] = i < w1 ? L[i] : 0.f; }
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const bool in = r0 + u * 64 + lane < w1;
        const uint32_t k = order_key(v[u]);
        c_gt += (unsigned)__popcll(__ballot(in && k > kth));
        c_eq += (unsigned)__popcll(__ballot(in && k == kth));
      }
    }
    if (lane == 0) s_scan[wave] = (c_gt << 16) | min(c_eq, 0xffffu);   // more equal keys than that: only the first `need` matter
    __syncthreads();
    unsigned base = 0u;
    for (int w = 0; w < wave; ++w) {                 // saturating in the low half: the sum is only compared with `need`
      const unsigned sw = s_scan[w];
      base = ((base >> 16) + (sw >> 16)) << 16 | min((base & 0xffffu) + (sw & 0xffffu), 0xffffu);
    }
    int p_gt = (int)(base >> 16), p_eq = (int)(base & 0xffffu);
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int r0 = w0; r0 < w1; r0 += 16 * 64) {
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) { const int i = r0 + u * 64 + lane; v[u] = i < w1 ? L[i] : 0.f; }
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int i = r0 + u * 64 + lane;
        const bool in = i < w1;
        const uint32_t k = order_key(v[u]);
        const unsigned long long m_gt = __ballot(in && k > kth), m_eq = __ballot(in && k == kth);
        if (in && k > kth) { const int p = p_gt + __popcll(m_gt & below); s_key[p] = k; s_idx[p] = i; }
        if (in && k == kth) {
          const int p = p_eq + __popcll(m_eq & below);
          if (p < (int)need) { s_key[n_gt + p] = k; s_idx[n_gt + p] = i; }
        }
        p_gt += __popcll(m_gt);
        p_eq = min(p_eq + __popcll(m_eq), 0xffff);
      }
    }
    __syncthreads();
    if (tid < K) {
      const uint32_t k = s_key[tid];
      const int ix = s_idx[tid];
      int rank = 0;
      for (int j = 0; j < K; ++j) rank += (s_key[j] > k) || (s_key[j] == k && s_idx[j] < ix);
      s_skey[rank] = k;
      s_sidx[rank] = ix;
    }
  }
  if (tid == 0) s_best = 0x7fffffff;
  __syncthreads();
  float* cum = reinterpret_cast<float*>(&s_hist[1][0]);           // K floats, free by now
  if (tid < K) cum[tid] = expf((key_value(s_skey[tid]) - mx) * b.inv_T) / Z;
  __syncthreads();
  if (tid == 0) {
    // running sums until top_p is reached (or the K candidates are used up); then the inverse CDF at u
    float run = 0.f;
    int m = 0;
    for (; m < K;) {
      run += cum[m];
      cum[m] = run;
      ++m;
      if (run >= b.top_p) break;
    }
    const float x = b.u[item] * run;
    int j = 0;
    while (j + 1 < m && !(x < cum[j])) ++j;
    s_tok = s_sidx[j];
  }
  __syncthreads();
  const int tok = s_tok;
  const ReqTables& t = tables[req];
  if (tid < meta[req].T && t.parent[tid] == -1 && t.token[tid] == tok) atomicMin(&s_best, tid);
  __syncthreads();
  if (tid == 0) {
    out[2 * item] = s_best == 0x7fffffff ? -1 : s_best;
    out[2 * item + 1] = tok;
    meta[req].root_pred = tok;
  }
}

hipError_t sp_launch_verify_sample(ReqMeta* meta, const ReqTables* tables, const float* logits, int n, const int* reqs,
                                   int V, float temperature, float top_p, int top_k, const float* u, int* out,
                                   hipStream_t st) {
  SampleBatch b;
  b.n = n; b.V = V; b.top_k = top_k; b.inv_T = 1.f / temperature; b.top_p = top_p;
  for (int i = 0; i < n; ++i) { b.req[i] = reqs[i]; b.u[i] = u[i]; }
  if (V % 4 == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0)
    hipLaunchKernelGGL(k_sample_decide<4>, dim3(n), dim3(1024), 0, st, meta, tables, logits, b, out);
  else
    hipLaunchKernelGGL(k_sample_decide<1>, dim3(n), dim3(1024), 0, st, meta, tables, logits, b, out);
  return hipGetLastError();
}

hipError_t sp_launch_row_norm(int dtype, const void* x, const void* gain, void* xn, int M, int d, float eps,
                              hipStream_t st) {
  if (dtype == 0)
    hipLaunchKernelGGL(k_row_norm<float>, dim3(M), dim3(1024), 0, st, (const float*)x, (const float*)gain, (float*)xn, d, eps);
  else
    hipLaunchKernelGGL(k_row_norm<bf16_t>, dim3(M), dim3(1024), 0, st, (const bf16_t*)x, (const bf16_t*)gain, (bf16_t*)xn, d, eps);
  return hipGetLastError();
}

size_t sp_lossy_scratch_floats(int n, int V) {
  const size_t slices = (size_t)(V + SLICE - 1) / SLICE;
  return (size_t)n * slices * (4 + SP_T);
}

hipError_t sp_launch_verify_lossy(ReqMeta* meta, const ReqTables* tables, const float* logits, int n, const int* reqs,
                                  int V, int mode, float top_p, float* scratch, int* out, hipStream_t st) {
  LossyBatch b;
  b.n = n; b.mode = mode; b.V = V; b.n_slices = (V + SLICE - 1) / SLICE; b.top_p = top_p;
  for (int i = 0; i < n; ++i) b.req[i] = reqs[i];
  float* stats = scratch;
  float* before = scratch + (size_t)n * b.n_slices * 4;
  hipLaunchKernelGGL(k_lossy_slices, dim3(b.n_slices, n), dim3(256), 0, st, meta, tables, logits, b, stats, before);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_lossy_decide, dim3(n), dim3(256), 0, st, meta, tables, logits, b, stats, before, out);
  return hipGetLastError();
}
