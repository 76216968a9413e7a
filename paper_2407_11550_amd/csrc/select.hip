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
// elements that still match the digits chosen so far.
//
// Blocks of one kernel never talk to each other: integer atomics add the per-block counts into
// global histograms, and the digit that holds the k-th largest element is found by the NEXT
// kernel, whose every block scans the (small) finished histogram in its prologue.  A kernel
// boundary is the cheapest device-wide synchronisation on this part: a device-scope fence
// inside a kernel writes a whole L2 back.
//
// Kernels per call: [clear, pass 0,] pass 1, pass 2, then alloc_finish (layer scope) or
// emit_write (head scope).  The bracketed two are skipped in pipeline mode, where the scoring
// kernels have cleared the histograms and counted the first digits (which do not depend on the
// scope).  The last pass also leaves per-block counts behind (elements above the threshold's
// 22-bit prefix; head scope: the block's own last-digit histogram), so that the kernel after it
// does not have to read the scores once more just to count.
#include "common.h"

namespace adakv {

namespace {

struct TopkWs {             // byte offsets inside the Top-k part of the workspace
  size_t hist;              // u32 [3][batch*h][RADIX_BINS]  per-head digit counts, layer scope
  size_t hist_tot;          // u32 [3][batch][RADIX_BINS]    the same summed over heads
  size_t hist_sel;          // u32 [3][batch*h][RADIX_BINS]  per-head digit counts, head scope
  size_t zero_end;          // everything before this starts at zero
  size_t state;             // uint2 [2][batch*h]: (digits chosen, rank left) after passes 0 and 1
  size_t chunk_hist;        // u16 [chunks][h][1024]  head scope, last pass: each block's own digit counts
  size_t chunk_sure;        // i32 [chunks][h]        last pass of either scope: the block's elements above
                            //                        the threshold's 22-bit prefix
  size_t total;
};

TopkWs plan(const SeqTab &st, const Dims &dm) {
  TopkWs p;
  const size_t nseg = (size_t)st.batch * dm.h_kv;
  size_t o = 0;
  p.hist = o; o += 3 * nseg * RADIX_BINS * 4;
  p.hist_tot = o; o += 3 * (size_t)st.batch * RADIX_BINS * 4;
  p.hist_sel = o; o += 3 * nseg * RADIX_BINS * 4;
  p.zero_end = o;
  p.state = o; o += align_up(2 * nseg * 8, 256);
  const size_t blocks = (size_t)make_chunks(st, SEL_CHUNK).off[st.batch] * dm.h_kv;
  p.chunk_hist = o; o += align_up(blocks * 1024 * 2, 256);
  p.chunk_sure = o; o += align_up(blocks * 4, 256);
  p.total = o;
  return p;
}

// The per-head histograms of the three passes of one scope.  The first digit of a score does not
// depend on the scope, so in pipeline mode the head scope reads the layer scope's pass-0 counts.
struct HistSet {
  unsigned *p[3];           // each [batch*h][RADIX_BINS]
};

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

struct Rank {
  unsigned prefix;   // digits chosen so far, in key position
  int krem;          // rank of the threshold among the elements matching them; 0 = select nothing
};

// This thread's NB/256 consecutive bins of a finished histogram, as 16-byte loads.  Kept apart
// from locate() so that callers can issue these loads together with everything else they need
// from memory (one round trip instead of a chain of them).
template <int NB> struct Bins { unsigned v[NB / 256]; };
template <int NB> __device__ __forceinline__ Bins<NB> load_bins(const unsigned *__restrict__ bins) {
  constexpr int PER = NB / 256;
  Bins<NB> r;
  // threads past the first 256 of a wider block own no bins
  const uint4 *p = reinterpret_cast<const uint4 *>(bins + (threadIdx.x & 255) * PER);
  const unsigned keep = threadIdx.x < 256 ? 0xFFFFFFFFu : 0u;
#pragma unroll
  for (int i = 0; i < PER / 4; ++i) {
    const uint4 q = p[i];
    r.v[4 * i] = q.x & keep; r.v[4 * i + 1] = q.y & keep;
    r.v[4 * i + 2] = q.z & keep; r.v[4 * i + 3] = q.w & keep;
  }
  return r;
}

// All threads of a block (the first 256 hold the bins): given the finished histogram of a pass (NB bins, this thread's part
// in `mine`) and the rank krem >= 1 among the elements it counts, find the digit whose bin holds
// that rank, counting from the largest digit down.  Returns the digit and the rank inside its
// bin (>= 1).
template <int NB>
__device__ __forceinline__ void locate(const Bins<NB> &mine, int krem, unsigned &digit,
                                       int &rank_in_bin, unsigned *sh /*[8]*/) {
  constexpr int PER = NB / 256;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  unsigned s = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) s += mine.v[i];
  unsigned suf = s;                                    // sum over lanes >= this one
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned v = __shfl_down(suf, off);
    if (lane + off < 64) suf += v;
  }
  __syncthreads();                                     // sh may be in use by the caller
  if (lane == 0 && wv < 4) sh[wv] = suf;
  if (tid == 0) { sh[4] = 0u; sh[5] = (unsigned)krem; }   // fallback keeps later reads in bounds
  __syncthreads();
  unsigned above = suf - s;                            // elements in bins owned by higher threads
  for (int i = wv + 1; i < 4; ++i) above += sh[i];
  if (above < (unsigned)krem && (unsigned)krem <= above + s) {
    unsigned acc = above;
#pragma unroll
    for (int i = PER - 1; i >= 0; --i) {
      if (acc < (unsigned)krem && (unsigned)krem <= acc + mine.v[i]) {
        sh[4] = (unsigned)(tid * PER + i);
        sh[5] = (unsigned)krem - acc;
      }
      acc += mine.v[i];
    }
  }
  __syncthreads();
  digit = sh[4];
  rank_in_bin = (int)sh[5];
}

__global__ __launch_bounds__(256) void topk_init_kernel(unsigned *__restrict__ zero_begin,
                                                        size_t zero_words) {
  const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (size_t i = i0; i < zero_words; i += (size_t)gridDim.x * blockDim.x) zero_begin[i] = 0u;
}

// Rank state in front of pass P for scope segment S: pass 0 starts from k; later passes take the
// stored state of the pass before the previous one and scan the previous pass's histogram.
template <int P, bool LAYER>
__device__ __forceinline__ Rank rank_before_pass(const SeqTab &st, int h, int b, int c,
                                                 const int *__restrict__ budgets,
                                                 const HistSet &hist,
                                                 const unsigned *__restrict__ hist_tot,
                                                 const uint2 *__restrict__ state, unsigned *sh) {
  const int nsegs = st.batch * h;
  const int S = LAYER ? b : b * h + c;
  Rank r;
  r.prefix = 0u;
  r.krem = 0;
  if (P == 0) {
    r.krem = LAYER ? st.Bp[b] : budgets[b * h + c];
    return r;
  } else {
    constexpr int Q = P - 1;                           // the pass whose histogram is scanned
    constexpr int NBQ = (Q == 2) ? 1024 : RADIX_BINS;
    const unsigned *bins = LAYER ? hist_tot + ((size_t)Q * st.batch + b) * RADIX_BINS
                                 : hist.p[Q] + (size_t)(b * h + c) * RADIX_BINS;
    // the histogram and the stored state do not depend on each other: both loads go out now
    const Bins<NBQ> mine = load_bins<NBQ>(bins);
    if (P == 1) {
      r.krem = LAYER ? st.Bp[b] : budgets[b * h + c];
    } else {
      const uint2 v = state[(size_t)(P - 2) * nsegs + S];
      r.prefix = v.x;
      r.krem = (int)v.y;
    }
    if (r.krem <= 0) return r;
    unsigned digit;
    int rank;
    locate<NBQ>(mine, r.krem, digit, rank, sh);
    r.prefix = with_digit<Q>(r.prefix, digit);
    r.krem = rank;
    return r;
  }
}

// One histogram pass.  grid.x runs over the SEL_CHUNK-sized chunks of all sequences, grid.y over
// heads.  LAYER: the k-th largest is sought over all heads of a sequence.
template <int P, bool LAYER>
__global__ __launch_bounds__(256) void topk_hist_kernel(SeqTab st, ChunkTab ct, int h,
                                                        const float *__restrict__ scores,
                                                        const int *__restrict__ budgets,
                                                        HistSet hist,
                                                        unsigned *__restrict__ hist_tot,
                                                        uint2 *__restrict__ state,
                                                        unsigned short *__restrict__ chunk_hist,
                                                        int *__restrict__ chunk_sure) {
  constexpr int NB = (P == 2) ? 1024 : RADIX_BINS;
  constexpr bool LAST_HEAD_PASS = (P == 2) && !LAYER;   // also leaves what the emit kernel counts with
  constexpr bool LAST_LAYER_PASS = (P == 2) && LAYER;   // also counts what lies above the last bucket
  __shared__ unsigned lh[RADIX_BINS];
  __shared__ unsigned sh[8];
  __shared__ int sh_sure;
  const int tid = threadIdx.x;
  const int b = find_seq(ct, st.batch, blockIdx.x);
  // the first sequence's facts sit at fixed places of the kernel arguments and arrive with the
  // first scalar fetch; only later sequences of a batch cost a dependent one
  int n = st.n[0], cfirst = ct.off[0], soff = st.score_off[0];
  if (b != 0) { n = st.n[b]; cfirst = ct.off[b]; soff = st.score_off[b]; }
  const int chunk = blockIdx.x - cfirst;
  const int c = blockIdx.y;
  const int nsegs = st.batch * h;
  // the block's scores are requested first, so they arrive while the prologue below waits for
  // the previous pass's histogram (indices past the end are clamped, the values ignored)
  const float *row = scores + soff + (size_t)c * n;
  const int j0 = chunk * SEL_CHUNK;
  const int j1 = min(n, j0 + SEL_CHUNK);
  constexpr int EPB = SEL_CHUNK / 256;
  float sc[EPB];
#pragma unroll
  for (int i = 0; i < EPB; ++i) sc[i] = row[min(j0 + tid + 256 * i, j1 - 1)];
  for (int i = tid; i < NB; i += 256) lh[i] = 0u;
  if (P == 2 && tid == 0) sh_sure = 0;
  const Rank r = rank_before_pass<P, LAYER>(st, h, b, c, budgets, hist, hist_tot, state, sh);
  if (P >= 1 && chunk == 0 && (!LAYER || c == 0) && tid == 0)
    state[(size_t)(P - 1) * nsegs + (LAYER ? b : b * h + c)] = make_uint2(r.prefix, (unsigned)r.krem);
  __syncthreads();
  if (r.krem <= 0) return;                             // nothing to select in this segment
  int sure = 0;
#pragma unroll
  for (int i = 0; i < EPB; ++i) {
    const unsigned key = key_of(sc[i]);
    const bool in = j0 + tid + 256 * i < j1;
    if (in && matches<P>(key, r.prefix)) atomicAdd(&lh[digit_of<P>(key)], 1u);
    if (P == 2) sure += in && (key >> 10) > (r.prefix >> 10);
  }
  if (P == 2) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sure += __shfl_xor(sure, off);
    if ((tid & 63) == 0) atomicAdd(&sh_sure, sure);
  }
  __syncthreads();
  if (LAST_HEAD_PASS) {
    // this block's own counts: the emit kernel adds up those of the chunks in front of its own
    const size_t blk = (size_t)blockIdx.x * h + c;
    for (int i = tid; i < 1024; i += 256) chunk_hist[blk * 1024 + i] = (unsigned short)lh[i];
    if (tid == 0) chunk_sure[blk] = sh_sure;
  }
  // layer scope: one plain store per block, the finishing kernel adds a head's blocks up
  if (LAST_LAYER_PASS && tid == 0) chunk_sure[(size_t)blockIdx.x * h + c] = sh_sure;
  unsigned *gh = hist.p[P] + (size_t)(b * h + c) * RADIX_BINS;
  unsigned *gt = hist_tot + ((size_t)P * st.batch + b) * RADIX_BINS;
  for (int i = tid; i < NB; i += 256) {
    const unsigned v = lh[i];
    if (v) {
      // the layer scope looks at per-head counts only after its last pass
      if (!LAYER || P == 2) atomicAdd(&gh[i], v);
      if (LAYER) atomicAdd(&gt[i], v);
    }
  }
}

// Layer scope, after the third pass: Algorithm 1's counts f_c and the safeguard of Alg. 2 l.8.
// One block of eight wavefronts per sequence.
__global__ __launch_bounds__(512) void alloc_finish_kernel(SeqTab st, ChunkTab ct, int h, int w,
                                                           int alpha_fix,
                                                           HistSet hist,
                                                           const unsigned *__restrict__ hist_tot,
                                                           const int *__restrict__ chunk_sure,
                                                           const uint2 *__restrict__ state,
                                                           int *__restrict__ budgets,
                                                           int *__restrict__ cu) {
  __shared__ unsigned sh[8];
  __shared__ int sh_gt[64], sh_eq[64];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int b = blockIdx.x;
  const int nsegs = st.batch * h;
  if (tid < 64) { sh_gt[tid] = 0; sh_eq[tid] = 0; }
  // Wavefront wv takes heads wv, wv+8, ...: the last pass's digit counts of the head (a lane
  // loads its 16 bins at once) and the number of its elements above the threshold's 22-bit
  // prefix, which the last histogram pass counted.  The first head's loads are issued before the
  // threshold is known (they do not depend on it), so they share its round trip.
  struct HeadBins { uint4 v2[4]; int sure; };
  auto load_head = [&](int c) {
    HeadBins hb;
    const int cc = min(c, h - 1);
    const uint4 *b2 = reinterpret_cast<const uint4 *>(hist.p[2] + (size_t)(b * h + cc) * RADIX_BINS) + lane * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) hb.v2[i] = b2[i];
    int sure = 0;                                      // the lanes stride over the head's blocks
    for (int k = ct.off[b] + lane; k < ct.off[b + 1]; k += 64) sure += chunk_sure[(size_t)k * h + cc];
    hb.sure = sure;
    return hb;
  };
  HeadBins first = load_head(wv);
  const Rank r = rank_before_pass<3, true>(st, h, b, 0, nullptr, hist, hist_tot, state, sh);
  __syncthreads();
  // r.prefix is the threshold key, r.krem how many threshold-valued elements are taken (in
  // flat-index order, i.e. head by head).  Per head: elements strictly above the threshold are
  // those above its 22-bit prefix plus those under the prefix with a larger last digit.
  if (r.krem > 0) {
    const unsigned d2 = digit_of<2>(r.prefix);
    for (int c = wv; c < h; c += 8) {
      const HeadBins hb = (c == wv) ? first : load_head(c);
      int cnt = 0, eq = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const unsigned a2[4] = {hb.v2[i].x, hb.v2[i].y, hb.v2[i].z, hb.v2[i].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const unsigned bin = (unsigned)(lane * 16 + i * 4 + k);
          if (bin > d2) cnt += (int)a2[k];
          if (bin == d2) eq += (int)a2[k];
        }
      }
      cnt += hb.sure;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) { cnt += __shfl_xor(cnt, off); eq += __shfl_xor(eq, off); }
      if (lane == 0) { sh_gt[c] = cnt; sh_eq[c] = eq; }
    }
  }
  __syncthreads();
  // One lane per head (h <= 64): every step below is a count over the other heads, so the lanes
  // never wait for each other and the 64-bit divisions run side by side.
  if (tid >= 64) return;
  __shared__ long long sh_rem[64];
  __shared__ int sh_base[64];
  const int c = tid;
  const bool live = c < h;
  const long long Bp = st.Bp[b];
  const long long one = 65536, a = alpha_fix;
  long long rem = -1;
  int base = 0;
  if (live) {
    long long before = 0;                              // threshold-valued elements of earlier heads
    for (int i = 0; i < c; ++i) before += sh_eq[i];
    long long avail = (long long)r.krem - before;      // ties still to take when head c's turn comes
    if (avail < 0) avail = 0;
    const long long take = sh_eq[c] < avail ? sh_eq[c] : avail;
    const long long f = (long long)sh_gt[c] + take;     // Algorithm 1: B*_c = f_c
    const long long num = (one - a) * h * f + a * Bp;   // x_c = num / den, den = 65536 h
    // num / 65536 = (1-alpha) h f + alpha B' <= h f + B' < 2^32 (both sums are below 2^31), so
    // the division by den is a shift and one 32-bit division; the remainders recombine exactly
    const unsigned t = (unsigned)(num >> 16);
    const unsigned tq = t / (unsigned)h, tr = t - tq * (unsigned)h;
    base = (int)tq;
    rem = ((long long)tr << 16) | (num & 0xFFFF);
  }
  sh_rem[c] = rem;
  sh_base[c] = base;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  if (!live) return;
  long long given = 0;
  int rank = 0;                                        // heads that come first for a spare unit
  for (int i = 0; i < h; ++i) {
    given += sh_base[i];
    rank += (sh_rem[i] > rem) || (sh_rem[i] == rem && i < c);
  }
  const int left = (int)(Bp - given);                  // 0 <= left < h
  if (rank < left) base += 1;                          // largest remainders, ties to the lower head
  budgets[b * h + c] = base;
  sh_base[c] = base;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  int run = st.out_off[b];
  for (int i = 0; i <= c; ++i) run += sh_base[i] + w;
  if (b == 0 && c == 0) cu[0] = 0;
  cu[b * h + c + 1] = run;
}

// Exclusive prefix sums of two per-thread counts over the 256 threads of a block.
__device__ __forceinline__ void block_scan2(int a, int b, int &ea, int &eb, int *sh /*[8]*/) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int ia = a, ib = b;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int ua = __shfl_up(ia, off), ub = __shfl_up(ib, off);
    if (lane >= off) { ia += ua; ib += ub; }
  }
  __syncthreads();
  if (lane == 63) { sh[wv] = ia; sh[4 + wv] = ib; }
  __syncthreads();
  int ba = 0, bb = 0;
  for (int i = 0; i < wv; ++i) { ba += sh[i]; bb += sh[4 + i]; }
  ea = ba + ia - a;
  eb = bb + ib - b;
}

constexpr int EPT = SEL_CHUNK / 256;   // consecutive positions per thread in the emit kernels

// Head scope, after the third pass: (threshold key, number of threshold-valued positions to take)
__device__ __forceinline__ Rank head_threshold(const SeqTab &st, int h, int b, int c,
                                               const HistSet &hist,
                                               const uint2 *__restrict__ state, unsigned *sh) {
  Rank r = rank_before_pass<3, false>(st, h, b, c, nullptr, hist, nullptr, state, sh);
  if (r.krem <= 0) { r.prefix = 0xFFFFFFFFu; r.krem = 0; }   // no key is above, no tie is taken
  return r;
}

__global__ __launch_bounds__(256) void emit_write_kernel(
    SeqTab st, ChunkTab ct, int h, int w, const float *__restrict__ scores,
    HistSet hist, const uint2 *__restrict__ state,
    const unsigned short *__restrict__ chunk_hist, const int *__restrict__ chunk_sure,
    const int *__restrict__ budgets, const int *__restrict__ cu, int *__restrict__ indices,
    int rows_total) {
  __shared__ unsigned sh[8];
  __shared__ int sh_base[2];
  const int tid = threadIdx.x;
  const int b = find_seq(ct, st.batch, blockIdx.x);
  int n = st.n[0], cfirst = ct.off[0], soff = st.score_off[0];   // as in the histogram kernel
  if (b != 0) { n = st.n[b]; cfirst = ct.off[b]; soff = st.score_off[b]; }
  const int chunk = blockIdx.x - cfirst;
  const int c = blockIdx.y;
  const int seg = b * h + c;
  const int out0 = cu[seg];
  const float *row = scores + soff + (size_t)c * n;

  // this thread's 16 consecutive positions (loads issued before the scans below)
  const int j0 = chunk * SEL_CHUNK + tid * EPT;
  unsigned keys[EPT];
#pragma unroll
  for (int i = 0; i < EPT; ++i) keys[i] = (j0 + i < n) ? key_of(row[j0 + i]) : 0u;

  // What the earlier chunks of this head hold above / at the threshold, from what the last
  // histogram pass left per block: elements above the threshold's 22-bit prefix, and the counts
  // of the last digit under that prefix (this thread looks at digits 4*tid .. 4*tid+3).  The loads
  // do not depend on the threshold, so they are issued in front of its scan, 32 chunks at a time.
  constexpr int CB = 32;   // 32 chunks = 131072 positions of a head in one round trip
  int pg = 0, pe = 0;
  for (int k = tid; k < chunk; k += 256) pg += chunk_sure[(size_t)(cfirst + k) * h + c];
  uint2 first[CB];
#pragma unroll
  for (int u = 0; u < CB; ++u) {
    const int k = min(u, max(chunk - 1, 0));
    first[u] = *reinterpret_cast<const uint2 *>(chunk_hist + ((size_t)(cfirst + k) * h + c) * 1024 + tid * 4);
  }
  if (tid < 2) sh_base[tid] = 0;
  const Rank r = head_threshold(st, h, b, c, hist, state, sh);
  const unsigned thr = r.prefix;
  const int ties = r.krem;
  const unsigned d2 = thr & 1023u;
  auto add_counts = [&](const uint2 &v) {
    const unsigned cnt[4] = {v.x & 0xFFFFu, v.x >> 16, v.y & 0xFFFFu, v.y >> 16};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned bin = (unsigned)tid * 4u + i;
      pg += bin > d2 ? (int)cnt[i] : 0;
      pe += bin == d2 ? (int)cnt[i] : 0;
    }
  };
  if (thr == 0xFFFFFFFFu) {
    pg = 0;                                            // nothing is selected in this head: the
  } else {                                             // histogram pass left no counts behind
#pragma unroll
    for (int u = 0; u < CB; ++u)
      if (u < chunk) add_counts(first[u]);
    for (int k0c = CB; k0c < chunk; k0c += CB) {
      uint2 more[CB];
#pragma unroll
      for (int u = 0; u < CB; ++u) {
        const int k = min(k0c + u, chunk - 1);
        more[u] = *reinterpret_cast<const uint2 *>(chunk_hist + ((size_t)(cfirst + k) * h + c) * 1024 + tid * 4);
      }
#pragma unroll
      for (int u = 0; u < CB; ++u)
        if (k0c + u < chunk) add_counts(more[u]);
    }
  }
  __syncthreads();
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { pg += __shfl_xor(pg, off); pe += __shfl_xor(pe, off); }
  if ((tid & 63) == 0) { atomicAdd(&sh_base[0], pg); atomicAdd(&sh_base[1], pe); }

  int g = 0, e = 0;
#pragma unroll
  for (int i = 0; i < EPT; ++i) {
    const bool valid = j0 + i < n;
    g += valid && keys[i] > thr;
    e += valid && keys[i] == thr;
  }
  int eg, ee;
  block_scan2(g, e, eg, ee, (int *)sh);                // its barriers also publish sh_base
  int ng = sh_base[0] + eg, ne = sh_base[1] + ee;      // counts over all earlier positions of the head
#pragma unroll
  for (int i = 0; i < EPT; ++i) {
    const int j = j0 + i;
    if (j >= n) break;
    const bool isg = keys[i] > thr, ise = keys[i] == thr;
    const int pos = out0 + ng + min(ne, ties);
    if ((isg || (ise && ne < ties)) && (unsigned)pos < (unsigned)rows_total) indices[pos] = j;
    ng += isg;
    ne += ise;
  }
  if (chunk == 0) {
    const int bud = budgets[seg];
    for (int rr = tid; rr < w; rr += 256)
      if ((unsigned)(out0 + bud + rr) < (unsigned)rows_total) indices[out0 + bud + rr] = n + rr;
  }
}

}  // namespace

size_t plan_topk_bytes(const SeqTab &st, const Dims &dm) { return plan(st, dm).total; }

// Pipeline mode needs a scoring kernel that files the first digits itself: the MFMA path with the
// max-pool fused into it.
bool carry_supported(const Dims &dm, int dtype) {
  return mfma_path_supported(dm, dtype) && dm.pool_k / 2 <= 32;
}

TopkCarry plan_carry(const SeqTab &st, const Dims &dm, char *ws_topk) {
  const TopkWs p = plan(st, dm);
  TopkCarry tc;
  tc.zero_begin = (unsigned *)ws_topk;
  tc.zero_words = (unsigned)(p.zero_end / 4);
  tc.hist0 = (unsigned *)(ws_topk + p.hist);
  tc.hist_tot0 = (unsigned *)(ws_topk + p.hist_tot);
  return tc;
}

static void launch_clear(const char *name, unsigned *begin, size_t words, hipStream_t s) {
  int zb = (int)((words + 256 * 4 - 1) / (256 * 4));
  if (zb < 1) zb = 1;
  if (zb > 1024) zb = 1024;
  ADAKV_LAUNCH(name, topk_init_kernel, dim3(zb), dim3(256), s, begin, words);
}

void launch_topk_clear(const TopkCarry &tc, hipStream_t s) {
  launch_clear("score_hist_clear", tc.zero_begin, tc.zero_words, s);
}

static HistSet hist_set(char *ws, const TopkWs &p, const SeqTab &st, const Dims &dm, bool layer,
                        bool carried) {
  const size_t per_pass = (size_t)st.batch * dm.h_kv * RADIX_BINS;
  unsigned *own = (unsigned *)(ws + (layer ? p.hist : p.hist_sel));
  HistSet hs;
  for (int q = 0; q < 3; ++q) hs.p[q] = own + q * per_pass;
  if (!layer && carried) hs.p[0] = (unsigned *)(ws + p.hist);   // first digits: scope-independent
  return hs;
}

template <bool LAYER>
static void run_passes(const SeqTab &st, const Dims &dm, const float *scores,
                       const int *budgets_in, const TopkWs &p, const ChunkTab &ct, char *ws,
                       bool carried, hipStream_t s) {
  const int h = dm.h_kv;
  const HistSet hist = hist_set(ws, p, st, dm, LAYER, carried);
  unsigned *hist_tot = (unsigned *)(ws + p.hist_tot);
  uint2 *state = (uint2 *)(ws + p.state);
  dim3 grid(ct.off[st.batch], h), block(256);
#define ADAKV_PASS(P)                                                                          \
  ADAKV_LAUNCH(LAYER ? "alloc_pass" #P : "select_pass" #P, (topk_hist_kernel<P, LAYER>), grid,   \
               block, s, st, ct, h, scores, budgets_in, hist, hist_tot, state,                    \
               (unsigned short *)(ws + p.chunk_hist), (int *)(ws + p.chunk_sure))
  if (!carried) {
    // this scope's own histograms (the layer scope's include the per-sequence totals)
    if (LAYER) launch_clear("alloc_init", (unsigned *)(ws + p.hist), (p.hist_sel - p.hist) / 4, s);
    else launch_clear("select_init", (unsigned *)(ws + p.hist_sel), (p.zero_end - p.hist_sel) / 4, s);
    ADAKV_PASS(0);
  }
  ADAKV_PASS(1);
  ADAKV_PASS(2);
#undef ADAKV_PASS
}

hipError_t launch_allocate(const SeqTab &st, const Dims &dm, const float *scores, int *budgets,
                           int *cu_seqlens, char *ws, bool carried, hipStream_t s) {
  const TopkWs p = plan(st, dm);
  const ChunkTab ct = make_chunks(st, SEL_CHUNK);
  run_passes<true>(st, dm, scores, nullptr, p, ct, ws, carried, s);
  ADAKV_LAUNCH("alloc_finish", alloc_finish_kernel, dim3(st.batch), dim3(512), s, st, ct, dm.h_kv,
               dm.w, dm.alpha_fix, hist_set(ws, p, st, dm, true, carried),
               (const unsigned *)(ws + p.hist_tot), (const int *)(ws + p.chunk_sure),
               (const uint2 *)(ws + p.state), budgets, cu_seqlens);
  return hipGetLastError();
}

hipError_t launch_select(const SeqTab &st, const Dims &dm, const float *scores,
                         const int *budgets, const int *cu_seqlens, int *indices, char *ws,
                         bool carried, hipStream_t s) {
  const TopkWs p = plan(st, dm);
  const ChunkTab ct = make_chunks(st, SEL_CHUNK);
  run_passes<false>(st, dm, scores, budgets, p, ct, ws, carried, s);
  const HistSet hist = hist_set(ws, p, st, dm, false, carried);
  dim3 grid(ct.off[st.batch], dm.h_kv), block(256);
  ADAKV_LAUNCH("select_emit", emit_write_kernel, grid, block, s, st, ct, dm.h_kv, dm.w, scores,
               hist, (const uint2 *)(ws + p.state), (const unsigned short *)(ws + p.chunk_hist),
               (const int *)(ws + p.chunk_sure), budgets, cu_seqlens, indices, st.out_off[st.batch]);
  return hipGetLastError();
}

}  // namespace adakv
