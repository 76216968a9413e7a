// Top-k by radix select, used twice:
//   * layer scope  (Algorithm 1 inside Alg. 2 l.7): the B' largest of a sequence's h*n scores,
//     counted per head, then the safeguard of Alg. 2 l.8 in integer arithmetic;
//   * head scope   (Alg. 2 l.9): the B_c largest of one head's n scores, emitted as ascending
//     positions followed by the window positions.
// Ties are decided by position (lower flat index first) through counts and prefix sums; the
// order in which atomics land never reaches a result, so every output is deterministic.
//
// A score becomes a 32-bit key whose unsigned order is the float order; its digits are the
// key's bits 31..21, 20..10 and 9..0.  Each scope runs two kernels (a kernel boundary is the
// cheapest device-wide synchronisation on this part; a device-scope fence inside a kernel writes
// a whole L2 back), so the whole Top-k is four launches after the first-digit histograms, which
// the scoring kernel leaves behind in pipeline mode (two small kernels make them otherwise):
//
//   gather   every block of 4096 positions finds the first digit d0 of its scope's threshold from
//            the finished first-digit histogram, adds the second digits of its elements under d0
//            to the scope's second-digit histogram, and leaves these elements behind sorted by
//            second digit (a counting sort inside the block: bucket starts + entries), together
//            with the number of its elements above d0;
//   finish / emit
//            finds the second digit d1 from the finished histogram.  The elements that share
//            the threshold's 22-bit prefix are then the bucket d1 of every block: few, and
//            found through the bucket starts without touching the scores again.  The last digit
//            and the number of ties to take come from them inside the block.  The layer scope
//            then counts per head and applies the safeguard; the head scope places every kept
//            position by prefix counts (earlier blocks' counts from the bucket starts, then a
//            block scan over 16 consecutive positions per thread).
//
// When more elements share a 22-bit prefix than a block can hold at once (plateaus: equal or
// almost equal scores), the finishing kernels stream the buckets instead of holding them.
#include "common.h"

namespace adakv {

namespace {

constexpr int ENT_PER_BLOCK = SEL_CHUNK;       // a block's elements under d0: at most all of them
constexpr int HOLD_LAYER = 4096;               // prefix-sharing elements the finishing kernel keeps in LDS
constexpr int HOLD_HEAD = 2048;                // the same for an emit block
constexpr int SERIAL_MAX = 64;                 // longest bucket a single thread copies by itself

struct TopkWs {             // byte offsets inside the Top-k part of the workspace
  size_t hist0;             // u32 [batch*h][RADIX_BINS]  first digits per head
  size_t hist_tot0;         // u32 [batch][RADIX_BINS]    first digits per sequence
  size_t hist1_tot;         // u32 [batch][RADIX_BINS]    layer scope: second digits under the sequence's d0
  size_t hist1;             // u32 [batch*h][RADIX_BINS]  head scope: second digits under the head's d0
  size_t zero_end;          // everything before this starts at zero
  size_t starts;            // u16 [blocks][RADIX_BINS]   bucket starts of a block's sorted entries
  size_t note;              // BlockNote [blocks]
  size_t entries;           // u16 [blocks][SEL_CHUNK]    last digits of a block's elements under d0, by bucket
  size_t bytes;
};

struct BlockNote {          // per gather block
  int entries;              // elements under d0 (= end of the last bucket)
  int above;                // elements above d0
};

TopkWs plan(const SeqTab &st, const Dims &dm) {
  TopkWs p;
  const size_t nseg = (size_t)st.batch * dm.h_kv;
  size_t o = 0;
  p.hist0 = o; o += nseg * RADIX_BINS * 4;
  p.hist_tot0 = o; o += (size_t)st.batch * RADIX_BINS * 4;
  p.hist1_tot = o; o += (size_t)st.batch * RADIX_BINS * 4;
  p.hist1 = o; o += nseg * RADIX_BINS * 4;
  p.zero_end = o;
  const size_t blocks = (size_t)make_chunks(st, SEL_CHUNK).off[st.batch] * dm.h_kv;
  p.starts = o; o += align_up(blocks * RADIX_BINS * 2, 256);
  p.note = o; o += align_up(blocks * sizeof(BlockNote), 256);
  p.entries = o; o += align_up(blocks * ENT_PER_BLOCK * 2, 256);
  p.bytes = o;
  return p;
}

// What the kernels of one scope share.
struct TopkBufs {
  const unsigned *hist0;     // first digits: per head
  const unsigned *hist_tot0; // first digits: per sequence
  unsigned *hist1;           // head scope: second digits under the head's d0
  unsigned *hist1_tot;       // layer scope: second digits under the sequence's d0
  unsigned short *starts;
  BlockNote *note;
  unsigned short *entries;   // last digits (10 bits each)
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

// All threads of a block (the first 256 hold the bins): given a finished histogram (NB bins, this
// thread's part in `mine`) and the rank krem >= 1 among the elements it counts, find the digit
// whose bin holds that rank, counting from the largest digit down.  Returns the digit and the
// rank inside its bin (>= 1).  A rank beyond the histogram's total gives digit 0 and the rank
// unchanged (callers clamp what they derive from it).
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
  if (tid < 256 && above < (unsigned)krem && (unsigned)krem <= above + s) {
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

// First digits of every score, per head and per sequence (outside pipeline mode, where the
// scoring kernel counts them).  grid.x runs over the SEL_CHUNK-sized chunks of all sequences,
// grid.y over heads.
__global__ __launch_bounds__(256) void topk_digit0_kernel(SeqTab st, ChunkTab ct, int h,
                                                          const float *__restrict__ scores,
                                                          unsigned *__restrict__ hist0,
                                                          unsigned *__restrict__ hist_tot0) {
  __shared__ unsigned lh[RADIX_BINS];
  const int tid = threadIdx.x;
  const int b = find_seq(ct, st.batch, blockIdx.x);
  const int n = st.n[b];
  const int chunk = blockIdx.x - ct.off[b];
  const int c = blockIdx.y;
  const float *row = scores + st.score_off[b] + (size_t)c * n;
  const int j0 = chunk * SEL_CHUNK, j1 = min(n, j0 + SEL_CHUNK);
  for (int i = tid; i < RADIX_BINS; i += 256) lh[i] = 0u;
  __syncthreads();
  for (int j = j0 + tid; j < j1; j += 256) atomicAdd(&lh[key_of(row[j]) >> 21], 1u);
  __syncthreads();
  unsigned *gh = hist0 + (size_t)(b * h + c) * RADIX_BINS;
  unsigned *gt = hist_tot0 + (size_t)b * RADIX_BINS;
  for (int i = tid; i < RADIX_BINS; i += 256) {
    const unsigned v = lh[i];
    if (v) {
      atomicAdd(&gh[i], v);
      atomicAdd(&gt[i], v);
    }
  }
}

// The gather kernel of either scope.  grid as above.  LAYER: the threshold is sought over all
// heads of a sequence (rank B'), else inside the block's own head (rank budgets[segment]).
template <bool LAYER>
__global__ __launch_bounds__(256) void topk_gather_kernel(SeqTab st, ChunkTab ct, int h,
                                                          const float *__restrict__ scores,
                                                          const int *__restrict__ budgets,
                                                          TopkBufs tb) {
  __shared__ unsigned lh[RADIX_BINS];                  // second-digit counts, then running bucket fill
  __shared__ unsigned sh[8];
  __shared__ int sh_above, sh_wave[4];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int b = find_seq(ct, st.batch, blockIdx.x);
  // the first sequence's facts sit at fixed places of the kernel arguments and arrive with the
  // first scalar fetch; only later sequences of a batch cost a dependent one
  int n = st.n[0], cfirst = ct.off[0], soff = st.score_off[0];
  if (b != 0) { n = st.n[b]; cfirst = ct.off[b]; soff = st.score_off[b]; }
  const int chunk = blockIdx.x - cfirst;
  const int c = blockIdx.y;
  const int seg = b * h + c;
  const size_t blk = (size_t)blockIdx.x * h + c;
  // the block's scores are requested first, so they arrive while the prologue below waits for
  // the histogram (indices past the end are clamped, the values ignored)
  const float *row = scores + soff + (size_t)c * n;
  const int j0 = chunk * SEL_CHUNK;
  const int j1 = min(n, j0 + SEL_CHUNK);
  constexpr int EPB = SEL_CHUNK / 256;
  float sc[EPB];
#pragma unroll
  for (int i = 0; i < EPB; ++i) sc[i] = row[min(j0 + tid + 256 * i, j1 - 1)];
  const Bins<RADIX_BINS> mine = load_bins<RADIX_BINS>(
      LAYER ? tb.hist_tot0 + (size_t)b * RADIX_BINS : tb.hist0 + (size_t)seg * RADIX_BINS);
  const int krem = LAYER ? st.Bp[b] : budgets[seg];
  for (int i = tid; i < RADIX_BINS; i += 256) lh[i] = 0u;
  if (tid == 0) sh_above = 0;
  if (krem <= 0) {                                     // nothing to select in this scope
    if (tid == 0) { tb.note[blk].entries = 0; tb.note[blk].above = 0; }
    return;
  }
  unsigned d0;
  int r0;
  locate<RADIX_BINS>(mine, krem, d0, r0, sh);          // its barriers also publish the cleared lh
  unsigned keys[EPB];
  int above = 0;
#pragma unroll
  for (int i = 0; i < EPB; ++i) {
    const bool in = j0 + tid + 256 * i < j1;
    const unsigned key = key_of(sc[i]);
    keys[i] = key;
    const unsigned dg = key >> 21;
    if (in && dg == d0) atomicAdd(&lh[(key >> 10) & 2047u], 1u);
    above += in && dg > d0;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) above += __shfl_xor(above, off);
  if (lane == 0) atomicAdd(&sh_above, above);
  __syncthreads();
  // bucket starts, largest digit first is not needed: buckets are addressed by digit.  Thread t
  // owns bins 8t .. 8t+7: exclusive scan over the block.
  unsigned cnt[8];
  unsigned tsum = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) { cnt[i] = lh[tid * 8 + i]; tsum += cnt[i]; }
  unsigned inc = tsum;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned v = __shfl_up(inc, off);
    if (lane >= off) inc += v;
  }
  if (lane == 63) sh_wave[wv] = (int)inc;
  __syncthreads();
  unsigned base = inc - tsum;
  for (int i = 0; i < wv; ++i) base += (unsigned)sh_wave[i];
  // starts to memory (one 16-byte store), counts to the scope's histograms, starts into lh
  unsigned stt[8];
  unsigned run = base;
#pragma unroll
  for (int i = 0; i < 8; ++i) { stt[i] = run; run += cnt[i]; }
  uint4 packed;
  packed.x = stt[0] | (stt[1] << 16); packed.y = stt[2] | (stt[3] << 16);
  packed.z = stt[4] | (stt[5] << 16); packed.w = stt[6] | (stt[7] << 16);
  reinterpret_cast<uint4 *>(tb.starts + blk * RADIX_BINS)[tid] = packed;
  if (tid == 255) { tb.note[blk].entries = (int)run; tb.note[blk].above = sh_above; }
  unsigned *gh = LAYER ? tb.hist1_tot + (size_t)b * RADIX_BINS : tb.hist1 + (size_t)seg * RADIX_BINS;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (cnt[i]) atomicAdd(&gh[tid * 8 + i], cnt[i]);
    lh[tid * 8 + i] = stt[i];
  }
  __syncthreads();
  // (the order inside a bucket follows the atomics, but only the multiset of a bucket's last
  // digits is ever used)
  unsigned short *ent = tb.entries + blk * ENT_PER_BLOCK;
#pragma unroll
  for (int i = 0; i < EPB; ++i) {
    const bool in = j0 + tid + 256 * i < j1;
    if (in && (keys[i] >> 21) == d0) {
      const unsigned slot = atomicAdd(&lh[(keys[i] >> 10) & 2047u], 1u);
      if (slot < (unsigned)ENT_PER_BLOCK) ent[slot] = (unsigned short)(keys[i] & 1023u);
    }
  }
}

// Bucket d1 of one gather block: [first, first + count) in its entries.
__device__ __forceinline__ void bucket_of(const TopkBufs &tb, size_t blk, unsigned d1, int &first,
                                          int &count) {
  const unsigned short *s = tb.starts + blk * RADIX_BINS;
  const int total = min(max(tb.note[blk].entries, 0), ENT_PER_BLOCK);
  const int a = min((int)s[d1], total);
  const int e = d1 + 1 < (unsigned)RADIX_BINS ? min((int)s[d1 + 1], total) : total;
  first = a;
  count = max(e - a, 0);
}

// Inclusive scan of one int over the threads of a block of NT threads; returns the block total.
template <int NT>
__device__ __forceinline__ int block_scan_incl(int v, int &incl, int *sh /*[NT/64]*/) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int x = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int u = __shfl_up(x, off);
    if (lane >= off) x += u;
  }
  __syncthreads();
  if (lane == 63) sh[wv] = x;
  __syncthreads();
  int before = 0, total = 0;
  for (int i = 0; i < NT / 64; ++i) {
    if (i < wv) before += sh[i];
    total += sh[i];
  }
  incl = before + x;
  return total;
}

// Last digits of a streamed bucket go to a visitor with two members: same(v, ok, times) when all
// of a lane's `times` entries carry the digit v, in every lane with ok set (a plateau of one
// value), and one(v, ok) for a single entry otherwise.  Both are called by a whole wavefront.
//
// The visitor that files them in a 1024-bin histogram in LDS.  64 atomics on one LDS word run one
// after the other, so while the lanes agree, call after call, the wavefront only keeps a running
// (digit, count) pair and adds it when the digit changes (and in flush() at the end).
struct WaveHist {
  unsigned *lh;
  unsigned run_digit, run_count;                       // the same in all lanes
  __device__ __forceinline__ explicit WaveHist(unsigned *bins) : lh(bins), run_digit(0u), run_count(0u) {}
  __device__ __forceinline__ void flush() {
    if (run_count && (threadIdx.x & 63) == 0) atomicAdd(&lh[run_digit], run_count);
    run_count = 0u;
  }
  __device__ __forceinline__ void same(unsigned digit, bool ok, unsigned times) {
    const unsigned long long act = __ballot(ok);
    if (act == 0) return;
    const int leader = __ffsll((long long)act) - 1;
    const unsigned dl = (unsigned)__builtin_amdgcn_readlane((int)digit, leader);
    if (__ballot(ok && digit != dl) == 0) {
      if (dl != run_digit) flush();
      run_digit = dl;
      run_count += (unsigned)__popcll(act) * times;
    } else if (ok) {
      atomicAdd(&lh[digit], times);
    }
  }
  __device__ __forceinline__ void one(unsigned digit, bool ok) {
    if (ok) atomicAdd(&lh[digit], 1u);
  }
};

// The visitor that counts the entries above and at the last digit d2.
struct CountAbove {
  unsigned d2;
  int gt, eq;
  __device__ __forceinline__ explicit CountAbove(unsigned digit) : d2(digit), gt(0), eq(0) {}
  __device__ __forceinline__ void same(unsigned v, bool ok, unsigned times) {
    gt += (ok && v > d2) ? (int)times : 0;
    eq += (ok && v == d2) ? (int)times : 0;
  }
  __device__ __forceinline__ void one(unsigned v, bool ok) {
    gt += ok && v > d2;
    eq += ok && v == d2;
  }
};

// Every entry of a bucket goes to the visitor f, called by a whole wavefront the same number of
// times in every lane.  Long buckets only occur on plateaus, where a block's elements under d0 all
// share one bucket that starts at entry 0: 16-byte loads (eight entries) when the bucket starts at
// a multiple of eight entries, eight of them in flight per lane (a whole block's 4096 entries in
// one round trip); two-byte loads, eight in flight, otherwise and for the tail.
template <class F>
__device__ __forceinline__ void for_bucket(const unsigned short *ent, int first, int count, F &f) {
  const int lane = threadIdx.x & 63;
  const unsigned short *p = ent + first;
  int done = 0;
  if ((first & 7) == 0) {
    const uint4 *q = reinterpret_cast<const uint4 *>(p);
    const int vecs = count / 8;                        // whole 16-byte words
    for (int v0 = 0; v0 < vecs; v0 += 512) {
      uint4 w[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) w[u] = q[min(v0 + u * 64 + lane, vecs - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool ok = v0 + u * 64 + lane < vecs;
        const unsigned x[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
        const bool all8 = x[0] == x[1] && x[1] == x[2] && x[2] == x[3] && (x[0] >> 16) == (x[0] & 0xFFFFu);
        if (__ballot(ok && !all8) == 0) {
          f.same(x[0] & 1023u, ok, 8u);
        } else {
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            f.one(x[k] & 1023u, ok);
            f.one((x[k] >> 16) & 1023u, ok);
          }
        }
      }
    }
    done = vecs * 8;
  }
  for (int i0 = done; i0 < count; i0 += 512) {
    unsigned v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p[min(i0 + u * 64 + lane, count - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u) f.one(v[u] & 1023u, i0 + u * 64 + lane < count);
  }
}

// Last digit among the elements sharing the 22-bit prefix, from a finished 1024-bin histogram in
// LDS: digit d2 whose bin holds rank r1, and the rank inside it = the number of ties to take.
__device__ __forceinline__ void locate_last(const unsigned *lh2, int r1, unsigned &d2, int &ties,
                                            unsigned *sh) {
  Bins<1024> m;
  const int t = threadIdx.x & 255;
  const unsigned keep = threadIdx.x < 256 ? 0xFFFFFFFFu : 0u;
#pragma unroll
  for (int i = 0; i < 4; ++i) m.v[i] = lh2[t * 4 + i] & keep;
  locate<1024>(m, r1, d2, ties, sh);
}

// Layer scope, second kernel: Algorithm 1's counts f_c and the safeguard of Alg. 2 l.8.
// One block of sixteen wavefronts per sequence.
constexpr int FIN_NT = 1024;
__global__ __launch_bounds__(FIN_NT) void alloc_finish_kernel(SeqTab st, ChunkTab ct, int h, int w,
                                                              int alpha_fix, TopkBufs tb,
                                                              int *__restrict__ budgets,
                                                              int *__restrict__ cu) {
  __shared__ unsigned sh[8];
  __shared__ int sh_scan[FIN_NT / 64];
  __shared__ unsigned lh2[1024];
  __shared__ unsigned held[HOLD_LAYER];                // (last digit << 6) | head
  __shared__ int sh_gt[64], sh_eq[64];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int b = blockIdx.x;
  const int Bp = st.Bp[b];
  if (tid < 64) { sh_gt[tid] = 0; sh_eq[tid] = 0; }
  for (int i = tid; i < 1024; i += FIN_NT) lh2[i] = 0u;
  const Bins<RADIX_BINS> m0 = load_bins<RADIX_BINS>(tb.hist_tot0 + (size_t)b * RADIX_BINS);
  const Bins<RADIX_BINS> m1 = load_bins<RADIX_BINS>(tb.hist1_tot + (size_t)b * RADIX_BINS);
  unsigned d0 = 0, d1 = 0, d2 = 0;
  int r0 = 0, r1 = 0, ties = 0;
  const int blk0 = ct.off[b] * h, blk1 = ct.off[b + 1] * h;      // this sequence's gather blocks
  if (Bp > 0) {
    locate<RADIX_BINS>(m0, Bp, d0, r0, sh);
    locate<RADIX_BINS>(m1, r0, d1, r1, sh);
    // the elements under (d0, d1): bucket d1 of every block.  Count them first.
    // The block's elements above the prefix go to its head's count right away: those above d0,
    // and under d0 those in the buckets after d1.
    int mine_cnt = 0, longest = 0;
    int first0 = 0, count0 = 0;                        // the first of this thread's blocks, kept
    for (int k = blk0 + tid; k < blk1; k += FIN_NT) {
      int first, count;
      bucket_of(tb, (size_t)k, d1, first, count);
      if (k == blk0 + tid) { first0 = first; count0 = count; }
      mine_cnt += count;
      longest = max(longest, count);
      const int total = min(max(tb.note[k].entries, 0), ENT_PER_BLOCK);
      const int over = tb.note[k].above + (total - first - count);
      if (over) atomicAdd(&sh_gt[k % h], over);
    }
    int incl;
    const int total = block_scan_incl<FIN_NT>(mine_cnt, incl, sh_scan);
    // (a thread copies its blocks' buckets one element after the other: only short ones)
    if (total <= HOLD_LAYER && !__syncthreads_or(longest > SERIAL_MAX)) {
      // few: every thread copies its blocks' buckets into LDS, then digit and counts from there
      int at = incl - mine_cnt;
      for (int k = blk0 + tid; k < blk1; k += FIN_NT) {
        int first = first0, count = count0;
        if (k != blk0 + tid) bucket_of(tb, (size_t)k, d1, first, count);
        const unsigned short *ent = tb.entries + (size_t)k * ENT_PER_BLOCK + first;
        const unsigned head = (unsigned)(k % h);
        for (int i = 0; i < count; ++i) {
          const unsigned v = (((unsigned)ent[i] & 1023u) << 6) | head;
          held[at++] = v;
          atomicAdd(&lh2[v >> 6], 1u);
        }
      }
      __syncthreads();
      locate_last(lh2, r1, d2, ties, sh);
      for (int i = tid; i < total; i += FIN_NT) {
        const unsigned v = held[i];
        if ((v >> 6) > d2) atomicAdd(&sh_gt[v & 63u], 1);
        if ((v >> 6) == d2) atomicAdd(&sh_eq[v & 63u], 1);
      }
    } else {
      // a plateau: stream the buckets, a wavefront per block, once for the digit and once for
      // the counts
      // (the next block's bucket is looked up while the current one streams)
      WaveHist wh(lh2);
      int nfirst = 0, ncount = 0;
      if (blk0 + wv < blk1) bucket_of(tb, (size_t)(blk0 + wv), d1, nfirst, ncount);
      for (int k = blk0 + wv; k < blk1; k += FIN_NT / 64) {
        const int first = nfirst, count = ncount;
        if (k + FIN_NT / 64 < blk1) bucket_of(tb, (size_t)(k + FIN_NT / 64), d1, nfirst, ncount);
        for_bucket(tb.entries + (size_t)k * ENT_PER_BLOCK, first, count, wh);
      }
      wh.flush();
      __syncthreads();
      locate_last(lh2, r1, d2, ties, sh);
      if (blk0 + wv < blk1) bucket_of(tb, (size_t)(blk0 + wv), d1, nfirst, ncount);
      for (int k = blk0 + wv; k < blk1; k += FIN_NT / 64) {
        const int first = nfirst, count = ncount;
        if (k + FIN_NT / 64 < blk1) bucket_of(tb, (size_t)(k + FIN_NT / 64), d1, nfirst, ncount);
        CountAbove ca(d2);
        for_bucket(tb.entries + (size_t)k * ENT_PER_BLOCK, first, count, ca);
        int gt = ca.gt, eq = ca.eq;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) { gt += __shfl_xor(gt, off); eq += __shfl_xor(eq, off); }
        if (lane == 0) { atomicAdd(&sh_gt[k % h], gt); atomicAdd(&sh_eq[k % h], eq); }
      }
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
  const long long one = 65536, a = alpha_fix;
  long long rem = -1;
  int base = 0;
  if (live) {
    long long before = 0;                              // threshold-valued elements of earlier heads
    for (int i = 0; i < c; ++i) before += sh_eq[i];
    long long avail = (long long)ties - before;        // ties still to take when head c's turn comes
    if (avail < 0) avail = 0;
    const long long take = sh_eq[c] < avail ? sh_eq[c] : avail;
    const long long f = (long long)sh_gt[c] + take;     // Algorithm 1: B*_c = f_c
    const long long num = (one - a) * h * f + a * (long long)Bp;   // x_c = num / den, den = 65536 h
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
  const int left = (int)((long long)Bp - given);       // 0 <= left < h
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

constexpr int EPT = SEL_CHUNK / 256;   // consecutive positions per thread in the emit kernel

// Head scope, second kernel.  Block (chunk, head) writes the kept positions of its 4096.
__global__ __launch_bounds__(256) void emit_write_kernel(
    SeqTab st, ChunkTab ct, int h, int w, const float *__restrict__ scores, TopkBufs tb,
    const int *__restrict__ budgets, const int *__restrict__ cu, int *__restrict__ indices,
    int rows_total) {
  __shared__ unsigned sh[8];
  __shared__ int sh_scan[4];
  __shared__ unsigned lh2[1024];
  __shared__ unsigned held[HOLD_HEAD];                 // (last digit << 1) | (lies in an earlier block)
  __shared__ int sh_cnt[2];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int b = find_seq(ct, st.batch, blockIdx.x);
  int n = st.n[0], cfirst = ct.off[0], soff = st.score_off[0];   // as in the gather kernel
  if (b != 0) { n = st.n[b]; cfirst = ct.off[b]; soff = st.score_off[b]; }
  const int chunk = blockIdx.x - cfirst;
  const int nchunks = (b != 0 ? ct.off[b + 1] : ct.off[1]) - cfirst;
  const int c = blockIdx.y;
  const int seg = b * h + c;
  const int out0 = cu[seg];
  const int bud = budgets[seg];
  const float *row = scores + soff + (size_t)c * n;

  // this thread's 16 consecutive positions (loads issued before the scans below)
  const int j0 = chunk * SEL_CHUNK + tid * EPT;
  unsigned keys[EPT];
#pragma unroll
  for (int i = 0; i < EPT; ++i) keys[i] = (j0 + i < n) ? key_of(row[j0 + i]) : 0u;
  const Bins<RADIX_BINS> m0 = load_bins<RADIX_BINS>(tb.hist0 + (size_t)seg * RADIX_BINS);
  const Bins<RADIX_BINS> m1 = load_bins<RADIX_BINS>(tb.hist1 + (size_t)seg * RADIX_BINS);
  for (int i = tid; i < 1024; i += 256) lh2[i] = 0u;
  if (tid < 2) sh_cnt[tid] = 0;

  unsigned thr = 0xFFFFFFFFu;                          // no key is above, no tie is taken
  int ties = 0;
  int pg = 0, pe = 0;                                  // kept / threshold-valued positions of earlier blocks
  if (bud > 0) {
    unsigned d0, d1, d2;
    int r0, r1;
    locate<RADIX_BINS>(m0, bud, d0, r0, sh);
    locate<RADIX_BINS>(m1, r0, d1, r1, sh);
    // Every block of the head (thread k takes block k, k + 256, ...): how many of its elements
    // share the prefix (d0, d1), and, for the blocks in front of this one, how many lie above it:
    // those above d0, and under d0 those in the buckets after d1.
    int mine_cnt = 0, longest = 0;
    int first0 = 0, count0 = 0;                        // the first of this thread's blocks, kept
    for (int k = tid; k < nchunks; k += 256) {
      const size_t kb = (size_t)(cfirst + k) * h + c;
      int first, count;
      bucket_of(tb, kb, d1, first, count);
      if (k == tid) { first0 = first; count0 = count; }
      mine_cnt += count;
      longest = max(longest, count);
      if (k < chunk) {
        const int total = min(max(tb.note[kb].entries, 0), ENT_PER_BLOCK);
        pg += tb.note[kb].above + (total - first - count);
      }
    }
    int incl;
    const int total = block_scan_incl<256>(mine_cnt, incl, sh_scan);
    if (total <= HOLD_HEAD && !__syncthreads_or(longest > SERIAL_MAX)) {
      int at = incl - mine_cnt;
      for (int k = tid; k < nchunks; k += 256) {
        const size_t kb = (size_t)(cfirst + k) * h + c;
        int first = first0, count = count0;
        if (k != tid) bucket_of(tb, kb, d1, first, count);
        const unsigned short *ent = tb.entries + kb * ENT_PER_BLOCK + first;
        const unsigned earlier = k < chunk ? 1u : 0u;
        for (int i = 0; i < count; ++i) {
          const unsigned v = ent[i] & 1023u;
          held[at++] = (v << 1) | earlier;
          atomicAdd(&lh2[v], 1u);
        }
      }
      __syncthreads();
      locate_last(lh2, r1, d2, ties, sh);
      for (int i = tid; i < total; i += 256) {
        const unsigned v = held[i];
        if (v & 1u) {
          pg += (v >> 1) > d2;
          pe += (v >> 1) == d2;
        }
      }
    } else {
      // a plateau: stream the buckets, a wavefront per block
      WaveHist wh(lh2);
      int nfirst = 0, ncount = 0;
      if (wv < nchunks) bucket_of(tb, (size_t)(cfirst + wv) * h + c, d1, nfirst, ncount);
      for (int k = wv; k < nchunks; k += 4) {
        const size_t kb = (size_t)(cfirst + k) * h + c;
        const int first = nfirst, count = ncount;
        if (k + 4 < nchunks) bucket_of(tb, (size_t)(cfirst + k + 4) * h + c, d1, nfirst, ncount);
        for_bucket(tb.entries + kb * ENT_PER_BLOCK, first, count, wh);
      }
      wh.flush();
      __syncthreads();
      locate_last(lh2, r1, d2, ties, sh);
      CountAbove ca(d2);
      if (wv < chunk) bucket_of(tb, (size_t)(cfirst + wv) * h + c, d1, nfirst, ncount);
      for (int k = wv; k < chunk; k += 4) {
        const size_t kb = (size_t)(cfirst + k) * h + c;
        const int first = nfirst, count = ncount;
        if (k + 4 < chunk) bucket_of(tb, (size_t)(cfirst + k + 4) * h + c, d1, nfirst, ncount);
        for_bucket(tb.entries + kb * ENT_PER_BLOCK, first, count, ca);
      }
      pg += ca.gt;
      pe += ca.eq;
    }
    thr = (d0 << 21) | (d1 << 10) | d2;
  }
  __syncthreads();
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { pg += __shfl_xor(pg, off); pe += __shfl_xor(pe, off); }
  if (lane == 0) { atomicAdd(&sh_cnt[0], pg); atomicAdd(&sh_cnt[1], pe); }

  int g = 0, e = 0;
#pragma unroll
  for (int i = 0; i < EPT; ++i) {
    const bool valid = j0 + i < n;
    g += valid && keys[i] > thr;
    e += valid && keys[i] == thr;
  }
  // both counts in one scan (a block holds 4096 positions: 13 bits each)
  int ige;
  block_scan_incl<256>((g << 16) | e, ige, sh_scan);   // its barriers also publish sh_cnt
  int ng = sh_cnt[0] + (ige >> 16) - g, ne = sh_cnt[1] + (ige & 0xFFFF) - e;   // over all earlier positions of the head
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
    for (int rr = tid; rr < w; rr += 256)
      if ((unsigned)(out0 + bud + rr) < (unsigned)rows_total) indices[out0 + bud + rr] = n + rr;
  }
}

}  // namespace

size_t plan_topk_bytes(const SeqTab &st, const Dims &dm) { return plan(st, dm).bytes; }

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
  tc.hist0 = (unsigned *)(ws_topk + p.hist0);
  tc.hist_tot0 = (unsigned *)(ws_topk + p.hist_tot0);
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

static TopkBufs bufs_of(char *ws, const TopkWs &p) {
  TopkBufs tb;
  tb.hist0 = (const unsigned *)(ws + p.hist0);
  tb.hist_tot0 = (const unsigned *)(ws + p.hist_tot0);
  tb.hist1 = (unsigned *)(ws + p.hist1);
  tb.hist1_tot = (unsigned *)(ws + p.hist1_tot);
  tb.starts = (unsigned short *)(ws + p.starts);
  tb.note = (BlockNote *)(ws + p.note);
  tb.entries = (unsigned short *)(ws + p.entries);
  return tb;
}

// Outside pipeline mode a call is self-contained: it clears the histograms and counts the first
// digits itself.
static void first_digits(const char *init_name, const char *pass_name, const SeqTab &st,
                         const ChunkTab &ct, int h, const float *scores, char *ws, const TopkWs &p,
                         hipStream_t s) {
  launch_clear(init_name, (unsigned *)ws, p.zero_end / 4, s);
  dim3 grid(ct.off[st.batch], h), block(256);
  ADAKV_LAUNCH(pass_name, topk_digit0_kernel, grid, block, s, st, ct, h, scores,
               (unsigned *)(ws + p.hist0), (unsigned *)(ws + p.hist_tot0));
}

hipError_t launch_allocate(const SeqTab &st, const Dims &dm, const float *scores, int *budgets,
                           int *cu_seqlens, char *ws, bool carried, hipStream_t s) {
  const TopkWs p = plan(st, dm);
  const ChunkTab ct = make_chunks(st, SEL_CHUNK);
  const int h = dm.h_kv;
  if (!carried) first_digits("alloc_init", "alloc_pass0", st, ct, h, scores, ws, p, s);
  const TopkBufs tb = bufs_of(ws, p);
  dim3 grid(ct.off[st.batch], h), block(256);
  ADAKV_LAUNCH("alloc_gather", (topk_gather_kernel<true>), grid, block, s, st, ct, h, scores,
               (const int *)nullptr, tb);
  ADAKV_LAUNCH("alloc_finish", alloc_finish_kernel, dim3(st.batch), dim3(FIN_NT), s, st, ct, h, dm.w,
               dm.alpha_fix, tb, budgets, cu_seqlens);
  return hipGetLastError();
}

hipError_t launch_select(const SeqTab &st, const Dims &dm, const float *scores,
                         const int *budgets, const int *cu_seqlens, int *indices, char *ws,
                         bool carried, hipStream_t s) {
  const TopkWs p = plan(st, dm);
  const ChunkTab ct = make_chunks(st, SEL_CHUNK);
  const int h = dm.h_kv;
  if (!carried) first_digits("select_init", "select_pass0", st, ct, h, scores, ws, p, s);
  const TopkBufs tb = bufs_of(ws, p);
  dim3 grid(ct.off[st.batch], h), block(256);
  ADAKV_LAUNCH("select_gather", (topk_gather_kernel<false>), grid, block, s, st, ct, h, scores,
               budgets, tb);
  ADAKV_LAUNCH("select_emit", emit_write_kernel, grid, block, s, st, ct, h, dm.w, scores, tb, budgets,
               cu_seqlens, indices, st.out_off[st.batch]);
  return hipGetLastError();
}

}  // namespace adakv
