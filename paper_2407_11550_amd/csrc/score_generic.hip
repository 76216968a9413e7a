// Observation-window scoring (Alg. 2 lines 1-5, group mean of Section 3.5) with plain fp32 FMA
// arithmetic: one thread per prefix key.  This path serves fp32 inputs and every shape the
// MFMA path does not take; it also hosts the two small kernels both paths share (the
// combination of partial softmax statistics, and the max-pool).
//
// The softmax of Alg. 2 l.3 needs each window row's denominator before rows can be added up,
// so the keys are swept twice: once for per-row (max, sum of exp) and once for the normalised
// weights.  Both sweeps compute a logit with the same instruction sequence, so it is the same
// number in both.
#include <math.h>

#include "common.h"

namespace adakv {

namespace {

constexpr int ROW_TILE = 16;   // window rows staged in LDS at a time

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int PER16 = 4;
  static __device__ __forceinline__ void unpack(const uint4 &v, float *o) {
    o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y);
    o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
  }
};
struct bf16_t { unsigned short bits; };
template <> struct Elem<bf16_t> {
  static constexpr int PER16 = 8;
  static __device__ __forceinline__ void unpack(const uint4 &v, float *o) {
    const unsigned a[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = __uint_as_float(a[i] << 16);
      o[2 * i + 1] = __uint_as_float(a[i] & 0xFFFF0000u);
    }
  }
};

struct f16_t { unsigned short bits; };
template <> struct Elem<f16_t> {
  static constexpr int PER16 = 8;
  static __device__ __forceinline__ void unpack(const uint4 &v, float *o) {
    const unsigned a[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = (float)__builtin_bit_cast(_Float16, (unsigned short)(a[i] & 0xFFFFu));
      o[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (unsigned short)(a[i] >> 16));
    }
  }
};

template <typename T, int D>
__device__ __forceinline__ void load_row(const T *p, float *o) {
  constexpr int P = Elem<T>::PER16;
  const uint4 *v = reinterpret_cast<const uint4 *>(p);
#pragma unroll
  for (int i = 0; i < D / P; ++i) Elem<T>::unpack(v[i], o + i * P);
}

// Stage rows [r0, r0 + ROW_TILE) of one KV head's g*w window queries as fp32 in LDS.
template <typename T, int D>
__device__ __forceinline__ void stage_q(const T *qhead, int r0, int R, float (*qs)[D]) {
  for (int i = threadIdx.x; i < ROW_TILE * D; i += 256) {
    const int r = i / D, e = i % D;
    float v = 0.0f;
    if (r0 + r < R) {
      float tmp[Elem<T>::PER16];
      const T *src = qhead + (size_t)(r0 + r) * D + (e / Elem<T>::PER16) * Elem<T>::PER16;
      Elem<T>::unpack(*reinterpret_cast<const uint4 *>(src), tmp);
      v = tmp[e % Elem<T>::PER16];
    }
    qs[r][e] = v;
  }
}

template <int D>
__device__ __forceinline__ float logit(const float *qrow, const float *k, float scale) {
  float acc = 0.0f;
#pragma unroll
  for (int e = 0; e < D; ++e) acc = fmaf(qrow[e], k[e], acc);
  return acc * scale;
}

// Sweep 1: partial (max, sum exp(s - max)) of every window row over this block's 256 keys.
template <typename T, int D>
__global__ __launch_bounds__(256) void stats_generic_kernel(
    SeqTab st, ChunkTab ct, Dims dm, const T *__restrict__ q, const T *__restrict__ K,
    float2 *__restrict__ part) {
  __shared__ float qs[ROW_TILE][D];
  __shared__ float sm[4][ROW_TILE], sl[4][ROW_TILE];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int b = find_seq(ct, st.batch, blockIdx.x);
  const int chunk = blockIdx.x - ct.off[b];
  const int c = blockIdx.y;
  const int n = st.n[b];
  const int R = dm.g * dm.w, RQ = dm.h_q * dm.w;
  const int j = chunk * GEN_CHUNK + tid;
  const bool valid = j < n;
  float k[D];
  if (valid) {
    load_row<T, D>(K + (st.tok_off[b] + j) * dm.k_stride_tok + c * dm.k_stride_head, k);
  } else {
#pragma unroll
    for (int e = 0; e < D; ++e) k[e] = 0.0f;
  }
  const T *qhead = q + ((size_t)b * RQ + (size_t)c * R) * D;
  for (int r0 = 0; r0 < R; r0 += ROW_TILE) {
    __syncthreads();
    stage_q<T, D>(qhead, r0, R, qs);
    __syncthreads();
    const int rt = min(ROW_TILE, R - r0);
    for (int r = 0; r < rt; ++r) {
      const float s = valid ? logit<D>(qs[r], k, dm.scale) : -INFINITY;
      float m = s;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
      float l = (valid && m > -INFINITY) ? expf(s - m) : 0.0f;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off);
      if (lane == 0) { sm[wv][r] = m; sl[wv][r] = l; }
    }
    __syncthreads();
    if (tid < rt) {
      float M = fmaxf(fmaxf(sm[0][tid], sm[1][tid]), fmaxf(sm[2][tid], sm[3][tid]));
      float L = 0.0f;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (sm[i][tid] > -INFINITY) L += sl[i][tid] * expf(sm[i][tid] - M);
      const size_t o = (size_t)blockIdx.x * RQ + (size_t)c * R + r0 + tid;
      part[o] = make_float2(M, L);
    }
  }
}

// Sweep 2: normalised weights summed over the g*w rows of the head, divided by g*w.
template <typename T, int D>
__global__ __launch_bounds__(256) void raw_generic_kernel(
    SeqTab st, ChunkTab ct, Dims dm, const T *__restrict__ q, const T *__restrict__ K,
    const float *__restrict__ lse, float *__restrict__ raw) {
  __shared__ float qs[ROW_TILE][D];
  __shared__ float sl[ROW_TILE];
  const int tid = threadIdx.x;
  const int b = find_seq(ct, st.batch, blockIdx.x);
  const int chunk = blockIdx.x - ct.off[b];
  const int c = blockIdx.y;
  const int n = st.n[b];
  const int R = dm.g * dm.w, RQ = dm.h_q * dm.w;
  const int j = chunk * GEN_CHUNK + tid;
  const bool valid = j < n;
  float k[D];
  if (valid) {
    load_row<T, D>(K + (st.tok_off[b] + j) * dm.k_stride_tok + c * dm.k_stride_head, k);
  } else {
#pragma unroll
    for (int e = 0; e < D; ++e) k[e] = 0.0f;
  }
  const T *qhead = q + ((size_t)b * RQ + (size_t)c * R) * D;
  float acc = 0.0f;
  for (int r0 = 0; r0 < R; r0 += ROW_TILE) {
    __syncthreads();
    stage_q<T, D>(qhead, r0, R, qs);
    if (tid < ROW_TILE) sl[tid] = (r0 + tid < R) ? lse[(size_t)b * RQ + (size_t)c * R + r0 + tid] : 0.0f;
    __syncthreads();
    const int rt = min(ROW_TILE, R - r0);
    for (int r = 0; r < rt; ++r) acc += expf(logit<D>(qs[r], k, dm.scale) - sl[r]);
  }
  if (valid) raw[st.score_off[b] + (size_t)c * n + j] = acc * (1.0f / (float)R);
}

// The other order of Alg. 2 l.4 (as printed there): every window row is max-pooled along the keys
// first, then the g*w rows of the head are averaged.  A block scores 256 consecutive keys and owns
// the middle 256 - 2*radius of them, so that every owned key finds its pool window in LDS; keys
// outside the sequence count as weight 0, which a max over non-negative weights never picks.
template <typename T, int D>
__global__ __launch_bounds__(256) void pooled_generic_kernel(
    SeqTab st, ChunkTab ct, Dims dm, const T *__restrict__ q, const T *__restrict__ K,
    const float *__restrict__ lse, float *__restrict__ scores) {
  __shared__ float qs[ROW_TILE][D];
  __shared__ float sl[ROW_TILE];
  __shared__ float ps[ROW_TILE][256];
  const int tid = threadIdx.x;
  const int b = find_seq(ct, st.batch, blockIdx.x);
  const int chunk = blockIdx.x - ct.off[b];
  const int c = blockIdx.y;
  const int n = st.n[b];
  const int R = dm.g * dm.w, RQ = dm.h_q * dm.w;
  const int r = dm.pool_k / 2, own = 256 - 2 * r;      // the launcher guarantees own >= 1
  const int j = chunk * own - r + tid;                 // the key this thread scores
  const bool valid = j >= 0 && j < n;
  const bool owner = tid >= r && tid < 256 - r && j < n;
  float k[D];
  if (valid) {
    load_row<T, D>(K + (st.tok_off[b] + j) * dm.k_stride_tok + c * dm.k_stride_head, k);
  } else {
#pragma unroll
    for (int e = 0; e < D; ++e) k[e] = 0.0f;
  }
  const T *qhead = q + ((size_t)b * RQ + (size_t)c * R) * D;
  float acc = 0.0f;
  for (int r0 = 0; r0 < R; r0 += ROW_TILE) {
    __syncthreads();                                   // the previous tile's ps and qs are done with
    stage_q<T, D>(qhead, r0, R, qs);
    if (tid < ROW_TILE) sl[tid] = (r0 + tid < R) ? lse[(size_t)b * RQ + (size_t)c * R + r0 + tid] : 0.0f;
    __syncthreads();
    const int rt = min(ROW_TILE, R - r0);
    for (int rr = 0; rr < rt; ++rr)
      ps[rr][tid] = valid ? expf(logit<D>(qs[rr], k, dm.scale) - sl[rr]) : 0.0f;
    __syncthreads();
    if (owner) {
      for (int rr = 0; rr < rt; ++rr) {
        float m = ps[rr][tid - r];
        for (int t = tid - r + 1; t <= tid + r; ++t) m = fmaxf(m, ps[rr][t]);
        acc += m;
      }
    }
  }
  if (owner) scores[st.score_off[b] + (size_t)c * n + j] = acc * (1.0f / (float)R);
}

}  // namespace

// lse[b][row] = log of the sum over the sequence's chunks of l * exp(m).  One wavefront per row:
// the lanes stride over the chunks (independent loads), then the 64 partial (max, sum) pairs are
// merged with shuffles.
__global__ __launch_bounds__(256) void lse_combine_kernel(SeqTab st, ChunkTab ct, int RQ,
                                                          const float2 *__restrict__ part,
                                                          float *__restrict__ lse) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int b = blockIdx.y;
  if (row >= RQ) return;
  float M = -INFINITY, L = 0.0f;
  for (int k = ct.off[b] + lane; k < ct.off[b + 1]; k += 64) {
    const float2 ml = part[(size_t)k * RQ + row];
    const float m = ml.x, l = ml.y;
    const float nm = fmaxf(M, m);
    if (nm > -INFINITY) L = L * expf(M - nm) + l * expf(m - nm);
    M = nm;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float m2 = __shfl_xor(M, off), l2 = __shfl_xor(L, off);
    const float nm = fmaxf(M, m2);
    if (nm > -INFINITY) L = L * expf(M - nm) + l2 * expf(m2 - nm);
    M = nm;
  }
  if (lane == 0) lse[(size_t)b * RQ + row] = M + logf(L);
}

// scores[j] = max of raw over [j - k/2, j + k/2] clipped to the head's row (stride 1, same length).
__global__ __launch_bounds__(256) void pool_kernel(SeqTab st, ChunkTab ct, int pool_k,
                                                   const float *__restrict__ raw,
                                                   float *__restrict__ scores) {
  const int b = find_seq(ct, st.batch, blockIdx.x);
  const int chunk = blockIdx.x - ct.off[b];
  const int c = blockIdx.y;
  const int n = st.n[b];
  const int j = chunk * GEN_CHUNK + threadIdx.x;
  if (j >= n) return;
  const size_t base = st.score_off[b] + (size_t)c * n;
  const int r = pool_k / 2;
  const int lo = max(0, j - r), hi = min(n - 1, j + r);
  float m = raw[base + lo];
  for (int jj = lo + 1; jj <= hi; ++jj) m = fmaxf(m, raw[base + jj]);
  scores[base + j] = m;
}

ScorePlan plan_score(const SeqTab &st, const Dims &dm, int dtype, bool on_mfma) {
  ScorePlan p;
  // partial statistics: one (max, sum) pair per window row and chunk of keys; the plain-FMA
  // kernels cut a sequence into GEN_CHUNK keys, the matrix-core kernels into longer chunks
  const bool mfma = on_mfma;
  (void)dtype;
  p.part_chunk = mfma ? choose_mfma_variant(st, dm).chunk : GEN_CHUNK;
  const size_t chunks = make_chunks(st, p.part_chunk).off[st.batch];
  const size_t RQ = (size_t)dm.h_q * dm.w;
  size_t o = 0;
  p.part = o; o += align_up(chunks * RQ * 8, 256);
  p.lse = o; o += align_up((size_t)st.batch * RQ * 4, 256);
  p.raw = o; o += align_up((size_t)st.score_off[st.batch] * 4, 256);
  p.total = o;
  return p;
}

void launch_lse_combine(const SeqTab &st, const ChunkTab &ct, int RQ, const float2 *part,
                        float *lse, hipStream_t s) {
  ADAKV_LAUNCH("score_lse_combine", lse_combine_kernel, dim3((RQ + 3) / 4, st.batch),
               dim3(256), s, st, ct, RQ, part, lse);
}

void launch_pool(const SeqTab &st, const Dims &dm, const float *raw, float *scores,
                 hipStream_t s) {
  const ChunkTab ct = make_chunks(st, GEN_CHUNK);
  ADAKV_LAUNCH("score_pool", pool_kernel, dim3(ct.off[st.batch], dm.h_kv), dim3(256), s, st, ct,
               dm.pool_k, raw, scores);
}

template <typename T, int D>
static void run_generic(const SeqTab &st, const Dims &dm, const void *q, const void *K,
                        const float *row_lse, float *scores, char *ws, const ScorePlan &pl,
                        bool pool_first, hipStream_t s) {
  const ChunkTab ct = make_chunks(st, GEN_CHUNK);
  dim3 grid(ct.off[st.batch], dm.h_kv), block(256);
  float2 *part = (float2 *)(ws + pl.part);
  float *lse = (float *)(ws + pl.lse), *raw = (float *)(ws + pl.raw);
  const float *use_lse = row_lse;
  if (!row_lse) {
    ADAKV_LAUNCH("score_stats_fma", (stats_generic_kernel<T, D>), grid, block, s, st, ct, dm,
                 (const T *)q, (const T *)K, part);
    launch_lse_combine(st, ct, dm.h_q * dm.w, part, lse, s);
    use_lse = lse;
  }
  if (pool_first) {
    const ChunkTab co = make_chunks(st, 256 - 2 * (dm.pool_k / 2));
    ADAKV_LAUNCH("score_pooled_fma", (pooled_generic_kernel<T, D>), dim3(co.off[st.batch], dm.h_kv),
                 block, s, st, co, dm, (const T *)q, (const T *)K, use_lse, scores);
    return;
  }
  ADAKV_LAUNCH("score_weights_fma", (raw_generic_kernel<T, D>), grid, block, s, st, ct, dm,
               (const T *)q, (const T *)K, use_lse, raw);
  launch_pool(st, dm, raw, scores, s);
}

hipError_t launch_score_generic(const SeqTab &st, const Dims &dm, int dtype, const void *q,
                                const void *K, const float *row_lse, float *scores, char *ws,
                                const ScorePlan &pl, bool pool_first, hipStream_t s) {
  if (dtype == ADAKV_FP32) {
    if (dm.d == 64) run_generic<float, 64>(st, dm, q, K, row_lse, scores, ws, pl, pool_first, s);
    else run_generic<float, 128>(st, dm, q, K, row_lse, scores, ws, pl, pool_first, s);
  } else if (dtype == ADAKV_FP16) {
    if (dm.d == 64) run_generic<f16_t, 64>(st, dm, q, K, row_lse, scores, ws, pl, pool_first, s);
    else run_generic<f16_t, 128>(st, dm, q, K, row_lse, scores, ws, pl, pool_first, s);
  } else {
    if (dm.d == 64) run_generic<bf16_t, 64>(st, dm, q, K, row_lse, scores, ws, pl, pool_first, s);
    else run_generic<bf16_t, 128>(st, dm, q, K, row_lse, scores, ws, pl, pool_first, s);
  }
  return hipGetLastError();
}

}  // namespace adakv
