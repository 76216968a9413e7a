// Top-k by radix select, used twice:
//   * layer scope  (Algorithm 1 inside Alg. 2 l.7): the B' largest of a sequence's h*n scores,
//     counted per head, then the safeguard of Alg. 2 l.8 in integer arithmetic;
//   * head scope   (Alg. 2 l.9): the B_c largest of one head's n scores, emitted as ascending
//     positions followed by the window positions.
// Ties are decided by position (lower flat index first) through counts and prefix sums; the
// order in which atomics land never reaches a result, so every output is deterministic.
//
// A score becomes a 32-bit key whose unsigned order is the float order.  Three passes over the
// scores take the key's bits 31..21, 20..10, 9..0; each pass histograms the digit of the
// elements that still match the digits chosen so far, and the last block to finish a segment
// picks the digit that holds the k-th largest element.
#include "common.h"

namespace adakv {

namespace {

struct TopkWs {             // byte offsets inside the workspace
  size_t hist;              // u32 [3][batch*h][RADIX_BINS]
  size_t ticket;            // u32 [3][batch*h]
  size_t gt;                // i32 [batch*h]   elements strictly above the threshold, per head
  size_t zero_end;          // everything before this is cleared by the init kernel
  size_t prefix;            // u32 [batch*h]   digits chosen so far (scope segment index)
  size_t krem;              // i32 [batch*h]   rank of the threshold among matching elements
  size_t thr;               // u32 [batch*h]   final threshold key per head (head scope)
  size_t ties;              // i32 [batch*h]   how many threshold-valued elements to take
  size_t chunk_cnt;         // i32 [chunks][h][2]
  size_t total;
};

TopkWs plan(const SeqTab &st, const Dims &dm) {
  TopkWs p;
  const size_t nseg = (size_t)st.batch * dm.h_kv;
  size_t o = 0;
  p.hist = o; o += 3 * nseg * RADIX_BINS * 4;
  p.ticket = o; o += align_up(3 * nseg * 4, 256);
  p.gt = o; o += align_up(nseg * 4, 256);
  p.zero_end = o;
  p.prefix = o; o += align_up(nseg * 4, 256);
  p.krem = o; o += align_up(nseg * 4, 256);
  p.thr = o; o += align_up(nseg * 4, 256);
  p.ties = o; o += align_up(nseg * 4, 256);
  p.chunk_cnt = o;
  o += align_up((size_t)make_chunks(st, SEL_CHUNK).off[st.batch] * dm.h_kv * 2 * 4, 256);
  p.total = o;
  return p;
}

__device__ __forceinline__ unsigned key_of(float x) {
  // +0.0f turns -0 into +0.  Non-negative floats order like their bit patterns; the general
  // transform keeps the order for negative inputs too.
  unsigned u = __float_as_uint(x + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int P> __device__ __forceinline__ bool matches(unsigned key, unsigned prefix) {
  if (P == 0) return true;
  if (P == 1) return (key >> 21) == (prefix >> 21);
  return (key >> 10) == (prefix >> 10);
}
template <int P> __device__ __forceinline__ unsigned digit_of(unsigned key) {
  if (P == 0) return key >> 21;
  if (P == 1) return (key >> 10) & 2047u;
  return key & 1023u;
}
template <int P> __device__ __forceinline__ unsigned with_digit(unsigned prefix, unsigned dgt) {
  if (P == 0) return dgt << 21;
  if (P == 1) return (prefix & 0xFFE00000u) | (dgt << 10);
  return (prefix & 0xFFFFFC00u) | dgt;
}

__device__ __forceinline__ unsigned ld_u32(const unsigned *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_i32(const int *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(256) void topk_init_kernel(SeqTab st, int h, bool layer_scope,
                                                        const int *__restrict__ budgets,
                                                        unsigned *__restrict__ zero_begin,
                                                        size_t zero_words,
                                                        unsigned *__restrict__ prefix,
                                                        int *__restrict__ krem) {
  const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (size_t i = i0; i < zero_words; i += (size_t)gridDim.x * blockDim.x) zero_begin[i] = 0u;
  const int nseg = layer_scope ? st.batch : st.batch * h;
  if (i0 < (size_t)nseg) {
    prefix[i0] = 0u;
    krem[i0] = layer_scope ? st.Bp[i0] : budgets[i0];
  }
}

// One pass of the radix select.  grid.x runs over the SEL_CHUNK-sized chunks of all sequences,
// grid.y over heads.  LAYER: the k-th largest is sought over all heads of a sequence.
template <int P, bool LAYER>
__global__ __launch_bounds__(256) void topk_pass_kernel(
    SeqTab st, ChunkTab ct, int h, int w, int alpha_fix, const float *__restrict__ scores,
    unsigned *__restrict__ hist, unsigned *__restrict__ ticket, int *__restrict__ gt,
    unsigned *__restrict__ prefix_g, int *__restrict__ krem_g, unsigned *__restrict__ thr_g,
    int *__restrict__ ties_g, int *__restrict__ budgets, int *__restrict__ cu) {
  constexpr int NB = (P == 2) ? 1024 : RADIX_BINS;
  __shared__ unsigned lh[RADIX_BINS];
  __shared__ unsigned sh_scan[256];
  __shared__ int sh_gt[64];
  __shared__ unsigned sh_misc[4];
  const int tid = threadIdx.x;
  const int b = find_seq(ct, st.batch, blockIdx.x);
  const int chunk = blockIdx.x - ct.off[b];
  const int c = blockIdx.y;
  const int n = st.n[b];
  const int nsegs = st.batch * h;
  const int seg_head = b * h + c;
  const int S = LAYER ? b : seg_head;
  const unsigned prefix = prefix_g[S];
  const int krem = krem_g[S];

  for (int i = tid; i < NB; i += 256) lh[i] = 0u;
  __syncthreads();
  if (krem > 0) {
    const float *row = scores + st.score_off[b] + (size_t)c * n;
    const int j0 = chunk * SEL_CHUNK;
    const int j1 = min(n, j0 + SEL_CHUNK);
    for (int j = j0 + tid; j < j1; j += 256) {
      const unsigned key = key_of(row[j]);
      if (matches<P>(key, prefix)) atomicAdd(&lh[digit_of<P>(key)], 1u);
    }
  }
  __syncthreads();
  // Publish the block's counts and take a ticket WITHOUT a device-scope fence (on this part a
  // release fence writes the whole L2 back, which costs more than the pass itself).  Everything
  // other blocks read is written by device-scope atomics, which execute at the point of
  // coherence; a returning atomic has been performed there once its value is back, so waiting
  // for the returned values orders the counts in front of the ticket.
  unsigned *gh = hist + ((size_t)P * nsegs + seg_head) * RADIX_BINS;
  unsigned seen = 0u;
  for (int i = tid; i < NB; i += 256) {
    const unsigned v = lh[i];
    if (v) seen |= __hip_atomic_fetch_add(&gh[i], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  asm volatile("" ::"v"(seen));          // the returned values are needed here: waits for them
  __syncthreads();
  if (tid == 0) {
    const unsigned nblk = (unsigned)(ct.off[b + 1] - ct.off[b]) * (LAYER ? (unsigned)h : 1u);
    const unsigned t = __hip_atomic_fetch_add(&ticket[(size_t)P * nsegs + S], 1u, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
    sh_misc[0] = (t == nblk - 1u) ? 1u : 0u;
  }
  __syncthreads();
  if (sh_misc[0] == 0u) return;

  // ---- last block of this segment: choose the digit that holds the krem-th largest --------
  const int c0 = LAYER ? 0 : c, c1 = LAYER ? h : c + 1;
  constexpr int PER = NB / 256;                        // consecutive bins per thread
  unsigned mine[PER];
  unsigned my_sum = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) mine[i] = 0u;
  if (krem > 0) {
    for (int cc = c0; cc < c1; ++cc) {
      const unsigned *hh = hist + ((size_t)P * nsegs + b * h + cc) * RADIX_BINS + tid * PER;
#pragma unroll
      for (int i = 0; i < PER; ++i) mine[i] += ld_u32(hh + i);
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) my_sum += mine[i];
  }
  // inclusive suffix sum over threads: sh_scan[t] = sum of my_sum over threads >= t
  sh_scan[tid] = my_sum;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {
    const unsigned add = (tid + off < 256) ? sh_scan[tid + off] : 0u;
    __syncthreads();
    sh_scan[tid] += add;
    __syncthreads();
  }
  if (tid < 64) sh_gt[tid] = 0;
  if (tid == 0) { sh_misc[1] = 0xFFFFFFFFu; sh_misc[2] = 0u; sh_misc[3] = 0u; }
  __syncthreads();
  const unsigned above = sh_scan[tid] - my_sum;        // elements in bins owned by higher threads
  if (krem > 0 && above < (unsigned)krem && (unsigned)krem <= above + my_sum) {
    unsigned acc = above;
    int dsel = 0;
#pragma unroll
    for (int i = PER - 1; i >= 0; --i) {
      if (acc < (unsigned)krem && (unsigned)krem <= acc + mine[i]) { dsel = i; break; }
      acc += mine[i];
    }
    sh_misc[1] = (unsigned)(tid * PER + dsel);         // chosen digit
    sh_misc[2] = (unsigned)krem - acc;                 // rank inside that digit's bin (>= 1)
  }
  __syncthreads();
  // (the clamp only matters for inputs outside the contract, e.g. NaN scores: it keeps every
  // later read inside the histogram)
  const unsigned dsel = min(sh_misc[1], (unsigned)(NB - 1));
  const unsigned new_prefix = (krem > 0) ? with_digit<P>(prefix, dsel) : 0xFFFFFFFFu;
  const int new_krem = (krem > 0) ? (int)sh_misc[2] : 0;
  // per head: how many elements sit in bins above the chosen digit
  if (krem > 0) {
    for (int cc = c0; cc < c1; ++cc) {
      const unsigned *hh = hist + ((size_t)P * nsegs + b * h + cc) * RADIX_BINS + tid * PER;
      int cnt = 0;
#pragma unroll
      for (int i = 0; i < PER; ++i)
        if ((unsigned)(tid * PER + i) > dsel) cnt += (int)ld_u32(hh + i);
      if (cnt) atomicAdd(&sh_gt[cc - c0], cnt);
    }
  }
  __syncthreads();
  if (tid < c1 - c0) {
    const int hidx = b * h + c0 + tid;
    const int v = ld_i32(&gt[hidx]) + sh_gt[tid];
    gt[hidx] = v;
    sh_gt[tid] = v;
  }
  if (tid == 0) {
    prefix_g[S] = new_prefix;
    krem_g[S] = new_krem;
  }
  if (P != 2) return;
  __syncthreads();
  if (tid != 0) return;
  if (!LAYER) {
    thr_g[seg_head] = new_prefix;
    ties_g[seg_head] = new_krem;
    return;
  }
  // ---- Algorithm 1 counts f_c, then the safeguard (Alg. 2 l.8) in exact integers ----------
  const long long Bp = st.Bp[b];
  long long ties_left = new_krem;                      // threshold-valued elements still to take
  const long long one = 65536, a = alpha_fix, den = one * h;
  long long rem[64];
  int base[64];
  long long given = 0;
  for (int cc = 0; cc < h; ++cc) {
    long long eq = 0;
    if (krem > 0)
      eq = ld_u32(hist + ((size_t)2 * nsegs + b * h + cc) * RADIX_BINS + dsel);
    const long long take = eq < ties_left ? eq : ties_left;
    ties_left -= take;
    const long long f = (long long)sh_gt[cc] + take;
    const long long num = (one - a) * h * f + a * Bp;
    base[cc] = (int)(num / den);
    rem[cc] = num % den;
    given += base[cc];
  }
  int left = (int)(Bp - given);                        // 0 <= left < h
  while (left > 0) {
    int best = 0;
    for (int cc = 1; cc < h; ++cc)
      if (rem[cc] > rem[best]) best = cc;              // strict: ties stay with the lower head
    base[best] += 1;
    rem[best] = -1;
    --left;
  }
  int run = st.out_off[b];
  if (b == 0) cu[0] = 0;
  for (int cc = 0; cc < h; ++cc) {
    budgets[b * h + cc] = base[cc];
    run += base[cc] + w;
    cu[b * h + cc + 1] = run;
  }
}

// Exclusive prefix sums of two per-thread counts over the 256 threads of a block.
__device__ __forceinline__ void block_scan2(int a, int b, int &ea, int &eb, int *sh /*[16]*/) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int ia = a, ib = b;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int ua = __shfl_up(ia, off), ub = __shfl_up(ib, off);
    if (lane >= off) { ia += ua; ib += ub; }
  }
  if (lane == 63) { sh[wv] = ia; sh[4 + wv] = ib; }
  __syncthreads();
  int ba = 0, bb = 0;
  for (int i = 0; i < wv; ++i) { ba += sh[i]; bb += sh[4 + i]; }
  ea = ba + ia - a;
  eb = bb + ib - b;
  __syncthreads();
}

constexpr int EPT = SEL_CHUNK / 256;   // consecutive positions per thread in the emit kernels

__global__ __launch_bounds__(256) void emit_count_kernel(SeqTab st, ChunkTab ct, int h,
                                                         const float *__restrict__ scores,
                                                         const unsigned *__restrict__ thr_g,
                                                         int *__restrict__ chunk_cnt) {
  __shared__ int sh[2];
  const int tid = threadIdx.x;
  const int b = find_seq(ct, st.batch, blockIdx.x);
  const int chunk = blockIdx.x - ct.off[b];
  const int c = blockIdx.y;
  const int n = st.n[b];
  const unsigned thr = thr_g[b * h + c];
  const float *row = scores + st.score_off[b] + (size_t)c * n;
  if (tid < 2) sh[tid] = 0;
  __syncthreads();
  int g = 0, e = 0;
  const int j0 = chunk * SEL_CHUNK, j1 = min(n, j0 + SEL_CHUNK);
  for (int j = j0 + tid; j < j1; j += 256) {
    const unsigned key = key_of(row[j]);
    g += key > thr;
    e += key == thr;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { g += __shfl_xor(g, off); e += __shfl_xor(e, off); }
  if ((tid & 63) == 0) { atomicAdd(&sh[0], g); atomicAdd(&sh[1], e); }
  __syncthreads();
  if (tid < 2) chunk_cnt[((size_t)blockIdx.x * h + c) * 2 + tid] = sh[tid];
}

__global__ __launch_bounds__(256) void emit_write_kernel(
    SeqTab st, ChunkTab ct, int h, int w, const float *__restrict__ scores,
    const unsigned *__restrict__ thr_g, const int *__restrict__ ties_g,
    const int *__restrict__ chunk_cnt, const int *__restrict__ budgets,
    const int *__restrict__ cu, int *__restrict__ indices, int rows_total) {
  __shared__ int sh[16];
  __shared__ int sh_base[2];
  const int tid = threadIdx.x;
  const int b = find_seq(ct, st.batch, blockIdx.x);
  const int chunk = blockIdx.x - ct.off[b];
  const int c = blockIdx.y;
  const int n = st.n[b];
  const int seg = b * h + c;
  const unsigned thr = thr_g[seg];
  const int ties = ties_g[seg];
  const int out0 = cu[seg];
  const float *row = scores + st.score_off[b] + (size_t)c * n;

  // what the earlier chunks of this head hold above / at the threshold
  int pg = 0, pe = 0;
  for (int k = tid; k < chunk; k += 256) {
    const int *cc = chunk_cnt + ((size_t)(ct.off[b] + k) * h + c) * 2;
    pg += cc[0];
    pe += cc[1];
  }
  if (tid < 2) sh_base[tid] = 0;
  __syncthreads();
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { pg += __shfl_xor(pg, off); pe += __shfl_xor(pe, off); }
  if ((tid & 63) == 0) { atomicAdd(&sh_base[0], pg); atomicAdd(&sh_base[1], pe); }
  __syncthreads();
  const int base_g = sh_base[0], base_e = sh_base[1];

  const int j0 = chunk * SEL_CHUNK + tid * EPT;
  unsigned keys[EPT];
  int g = 0, e = 0;
#pragma unroll
  for (int i = 0; i < EPT; ++i) {
    const int j = j0 + i;
    keys[i] = (j < n) ? key_of(row[j]) : 0u;
    const bool valid = j < n;
    g += valid && keys[i] > thr;
    e += valid && keys[i] == thr;
  }
  int eg, ee;
  block_scan2(g, e, eg, ee, sh);
  int ng = base_g + eg, ne = base_e + ee;   // counts over all earlier positions of the head
#pragma unroll
  for (int i = 0; i < EPT; ++i) {
    const int j = j0 + i;
    if (j >= n) break;
    const bool isg = keys[i] > thr, ise = keys[i] == thr;
    const int pos = out0 + ng + min(ne, ties);
    if ((isg || (ise && ne < ties)) && pos < rows_total) indices[pos] = j;
    ng += isg;
    ne += ise;
  }
  if (chunk == 0) {
    const int bud = budgets[seg];
    for (int r = tid; r < w; r += 256)
      if (out0 + bud + r < rows_total) indices[out0 + bud + r] = n + r;
  }
}

}  // namespace

size_t plan_topk_bytes(const SeqTab &st, const Dims &dm) { return plan(st, dm).total; }

template <bool LAYER>
static hipError_t run_passes(const SeqTab &st, const Dims &dm, const float *scores,
                             const int *budgets_in, int *budgets_out, int *cu, char *ws,
                             hipStream_t s) {
  const TopkWs p = plan(st, dm);
  const ChunkTab ct = make_chunks(st, SEL_CHUNK);
  const int h = dm.h_kv;
  unsigned *hist = (unsigned *)(ws + p.hist);
  unsigned *ticket = (unsigned *)(ws + p.ticket);
  int *gt = (int *)(ws + p.gt);
  unsigned *prefix = (unsigned *)(ws + p.prefix);
  int *krem = (int *)(ws + p.krem);
  unsigned *thr = (unsigned *)(ws + p.thr);
  int *ties = (int *)(ws + p.ties);
  const size_t zero_words = p.zero_end / 4;
  int zb = (int)((zero_words + 256 * 8 - 1) / (256 * 8));
  if (zb < 1) zb = 1;
  if (zb > 1024) zb = 1024;
  ADAKV_LAUNCH(LAYER ? "alloc_init" : "select_init", topk_init_kernel, dim3(zb), dim3(256), s, st,
               h, LAYER, budgets_in,
                     (unsigned *)ws, zero_words, prefix, krem);
  dim3 grid(ct.off[st.batch], h), block(256);
#define ADAKV_PASS(P)                                                                          \
  ADAKV_LAUNCH(LAYER ? "alloc_pass" #P : "select_pass" #P, (topk_pass_kernel<P, LAYER>), grid,   \
               block, s, st, ct, h, dm.w, dm.alpha_fix, scores, hist, ticket, gt, prefix, krem,  \
               thr, ties, budgets_out, cu)
  ADAKV_PASS(0);
  ADAKV_PASS(1);
  ADAKV_PASS(2);
#undef ADAKV_PASS
  return hipGetLastError();
}

hipError_t launch_allocate(const SeqTab &st, const Dims &dm, const float *scores, int *budgets,
                           int *cu_seqlens, char *ws, hipStream_t s) {
  return run_passes<true>(st, dm, scores, nullptr, budgets, cu_seqlens, ws, s);
}

hipError_t launch_select(const SeqTab &st, const Dims &dm, const float *scores,
                         const int *budgets, const int *cu_seqlens, int *indices, char *ws,
                         hipStream_t s) {
  hipError_t e = run_passes<false>(st, dm, scores, budgets, nullptr, nullptr, ws, s);
  if (e != hipSuccess) return e;
  const TopkWs p = plan(st, dm);
  const ChunkTab ct = make_chunks(st, SEL_CHUNK);
  dim3 grid(ct.off[st.batch], dm.h_kv), block(256);
  ADAKV_LAUNCH("select_count", emit_count_kernel, grid, block, s, st, ct, dm.h_kv, scores,
                     (const unsigned *)(ws + p.thr), (int *)(ws + p.chunk_cnt));
  ADAKV_LAUNCH("select_emit", emit_write_kernel, grid, block, s, st, ct, dm.h_kv, dm.w, scores,
                     (const unsigned *)(ws + p.thr), (const int *)(ws + p.ties),
                     (const int *)(ws + p.chunk_cnt), budgets, cu_seqlens, indices,
                     st.out_off[st.batch]);
  return hipGetLastError();
}

}  // namespace adakv
