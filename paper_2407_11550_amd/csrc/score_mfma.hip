// Observation-window scoring (Alg. 2 lines 1-5, group mean of Section 3.5) for bf16 and fp16
// inputs on the gfx950 matrix cores: logits = Q_win K^T as v_mfma_f32_32x32x16 tiles with fp32
// accumulation, softmax and reductions in fp32 on the vector ALUs.
//
// The softmax of Alg. 2 l.3 needs every window row's denominator before the rows of a head can
// be added up, so K is swept twice:
//   sweep 1 (PASS 1)  per-row (max, sum of exp) over the keys        -> partial statistics
//   sweep 2 (PASS 2)  exp(logit - lse) summed over the g*w rows      -> pre-pool scores
// A caller-supplied row_lse skips sweep 1.
//
// Work split.  In sweep 2 a workgroup owns CHUNK consecutive keys of one KV head (the fused
// max-pool wants neighbours); in sweep 1 the workgroups of a head take the head's tile sets in
// turn (set c, c + nch, ...), because a (max, sum) pair does not care which keys it saw and the
// chip then streams one dense region of K at a time.  All g query heads of the group share
// every K tile.  A wavefront keeps at most 64 window rows of Q in registers as MFMA
// operands for the whole chunk (MB blocks of 32 rows), which leaves room for two wavefronts per
// SIMD, so one wavefront's exponentials overlap the other's matrix work.  RS wavefronts split
// the rows of a head, and the KG = NW/RS groups of wavefronts take the 32-key tiles of the
// chunk in turn.  A K tile travels HBM -> registers (coalesced 16-byte loads of whole rows,
// issued by the whole workgroup, two iterations ahead) -> LDS (padded rows, shared by the
// wavefronts that need the tile) -> registers in operand layout.
//
// Operand roles differ between the sweeps because of what the accumulator layout makes cheap
// (D[i][j]: lane = column j, 16 rows i per lane):
//   sweep 1: D = K_tile Q^T, a lane owns ONE window row and 16 keys: running (max, sum) per
//            lane, nothing crosses lanes until the chunk is done;
//   sweep 2: D = Q K_tile^T, a lane owns ONE key and 16 window rows: the sum over rows is
//            lane-local adds plus one cross-half add; partial sums of the RS row groups meet
//            in LDS when the chunk is done and are added in a fixed order.
#include <math.h>

#include <type_traits>

#include "common.h"

namespace adakv {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int TILE = 32;           // keys per MFMA tile
constexpr long long CHUNK_SWITCH_WGS = 512;   // fewer workgroups than this: halve the chunk
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr int MFMA_POOL_ROWS_MAX_RADIUS = 7;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// The value of the neighbouring lane: CTRL 0x130 = wave_shl:1 (lane i reads lane i+1), 0x138 =
// wave_shr:1 (lane i reads lane i-1); the last / first lane of the wavefront reads 0.
template <int CTRL> __device__ __forceinline__ unsigned wave_shift(unsigned x) {
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, false);
}
__device__ __forceinline__ bf16x8 as_bf16(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// One 32x32x16 product-accumulate on eight 16-bit elements per lane and operand; the fragments are
// carried as raw 16-byte words (typed bf16x8 above) whatever the element type is.
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
template <bool F16>
__device__ __forceinline__ floatx16 mfma16(bf16x8 a, bf16x8 b, floatx16 c) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// PR (sweep 2 only): the printed order of Alg. 2 l.4, max-pool along the keys in every window row
// first, mean over the rows afterwards.  A lane of sweep 2 owns one key and 16 rows per row block,
// so the pool is a sliding maximum across neighbouring lanes, with whole-wavefront shifts by one
// lane.  Tiles then overlap by the pool radius on either side: only the inner 32 - 2r
// lanes of a tile have all their neighbours and produce a score.
template <int D, int MB, int RS, int KG, int CHUNK, int PASS, bool F16, bool PR = false>
__global__ __launch_bounds__(64 * RS * KG) void score_mfma_kernel(
    SeqTab st, ChunkTab ct, Dims dm, float c_log2, const unsigned short *__restrict__ q,
    const unsigned short *__restrict__ K, const float *__restrict__ lse,
    float2 *__restrict__ part, float *__restrict__ out, int halo,
    TopkCarry tc) {
  constexpr int NW = RS * KG;                // wavefronts per workgroup
  constexpr int NT = 64 * NW;
  constexpr int KS = D / 16;                 // MFMA k-steps per tile
  constexpr int ROW16 = D * 2 / 16;          // 16-byte words per K row
  constexpr int STRIDE16 = ROW16 + 1;        // padded LDS row, in 16-byte words
  constexpr int RW = 32 * MB;                // window rows per wavefront
  constexpr int RPAD = RW * RS;              // window rows per workgroup (padded)

  __shared__ u32x4 kt[2][KG * TILE * STRIDE16];  // two buffers of one iteration's KG tiles
  __shared__ float sh_rows[2][NW][RW];       // sweep 1: per-wave row (max, sum); sweep 2: [0][0] lse
  constexpr int HALO = TILE;                 // keys scored on either side of the chunk for the pool
  __shared__ float sh_part[PASS == 2 ? RS : 1][PASS == 2 ? CHUNK + 2 * HALO : 1];
  constexpr int NCOMB = NT > RPAD ? NT : RPAD;   // (thread slices) x (rows) of the statistics combination
  __shared__ float sh_cm[PASS == 2 ? NCOMB : 1], sh_cl[PASS == 2 ? NCOMB : 1];
  // first radix digits of the chunk's scores: only needed once the tile loop is over, in the
  // place of the K tiles (which leaves room for 4096-key chunks of eight row groups)
  static_assert(sizeof(kt) >= RADIX_BINS * sizeof(unsigned), "the digit histogram must fit into the tile buffers");
  unsigned *sh_hist = reinterpret_cast<unsigned *>(&kt[0][0]);

  const int tid = threadIdx.x, lane = tid & 63;
  // Pipeline mode: the statistics sweep clears the Top-k histograms (they are first touched by
  // the kernel after it), the weights sweep counts the first digit of every score it writes.
  if (PASS == 1 && tc.zero_begin) {
    for (unsigned i = blockIdx.x * NT + tid; i < tc.zero_words; i += gridDim.x * NT)
      tc.zero_begin[i] = 0u;
  }

  // the wavefront index is the same in all lanes: telling the compiler keeps everything derived
  // from it (tile numbers, K addresses, loop conditions) in scalar registers
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, l32 = lane & 31;
  const int kg = wv / RS, rs = wv % RS;
  const int h = dm.h_kv;
  const int c = blockIdx.x % h;
  int cg = blockIdx.x / h;
  if (PASS == 2) cg = ct.off[st.batch] - 1 - cg;
  const int b = find_seq(ct, st.batch, cg);
  const int chunk = cg - ct.off[b];
  const int n = st.n[b];
  const int R = dm.g * dm.w, RQ = dm.h_q * dm.w;
  const int kc0 = chunk * CHUNK;             // first key of the chunk
  const int kc1 = min(n, kc0 + CHUNK);
  // sweep 2 with the pool fused also scores the neighbours the pool looks at: a whole tile in
  // front of the chunk (tiles stay aligned), the pool radius behind it.  No tile may start past
  // the last key somebody needs: the row clamp in load_set counts rows from the tile set's
  // first key and must never go below it.
  const int pool_r = (PASS == 2 && (halo || PR)) ? dm.pool_k / 2 : 0;
  const int tstep = PR ? TILE - 2 * pool_r : TILE;     // keys a tile advances by
  // Sweep 1 does not need a workgroup's keys to be neighbours (its result is a (max, sum) pair
  // per row over whatever keys it saw), so there the tile sets of a head's workgroups are
  // interleaved: workgroup `chunk` of the sequence's nch takes sets chunk, chunk + nch, ...
  // of the whole sequence.  At any moment the workgroups of a head then read neighbouring sets,
  // i.e. the chip streams one dense region of K instead of 64 regions 4 MiB apart (measured
  // with a plain-read kernel of the same shape: 6.2 against 5.5 TB/s).
  constexpr bool INTER = PASS == 1;
  const int nch = ct.off[b + 1] - ct.off[b];
  const int k0 = INTER ? 0 : (PASS == 2 && halo && kc0 > 0) ? kc0 - HALO : kc0;
  const int k1 = INTER ? n : (PASS == 2 && halo) ? min(n, kc1 + pool_r) : kc1;
  const int ntiles = (k1 - k0 + tstep - 1) / tstep;
  const int row0 = rs * RW;                  // first window row of this wavefront
  const size_t head_row0 = (size_t)b * RQ + (size_t)c * R;

  // ---- K path ---------------------------------------------------------------------------------
  // An iteration covers KG consecutive tiles (one per wavefront group).  All threads of the
  // workgroup load the iteration's rows together: 16 lanes per 256-byte row, every byte read
  // once per workgroup, addressed as a wave-uniform 64-bit base (scalar registers) plus a
  // 32-bit per-lane offset.  The loads of iterations it+1 .. it+DEPTH are in flight while
  // iteration it is computed (DEPTH register sets, two LDS buffers, one barrier per iteration).
  // register sets = iterations of loads in flight (a third set fits the statistics sweep's
  // registers and was measured: no faster; nor are four or six sets on the 512-row shape,
  // where a set is a single word per thread)
  constexpr int DEPTH = 2;
  constexpr int TW = TILE * ROW16;                     // 16-byte words per tile
  constexpr int LDPT = KG * TW / NT;                   // loads per thread per iteration
  static_assert(KG * TW % NT == 0 && LDPT >= 1, "tile set must split evenly over the threads");
  const char *kbase = reinterpret_cast<const char *>(K) +
                      ((size_t)st.tok_off[b] * dm.k_stride_tok + (size_t)c * dm.k_stride_head) * 2;
  const size_t tok_bytes = (size_t)dm.k_stride_tok * 2;
  // word tid + i*NT of the iteration's KG*TW words: row (relative to the iteration's first key)
  // and 16-byte column
  int ld_rel[LDPT];
  int wr_off[LDPT];                                    // word offset in an LDS buffer
  const unsigned col_bytes = (unsigned)(tid % ROW16) * 16u;
#pragma unroll
  for (int i = 0; i < LDPT; ++i) {
    const int wi = tid + i * NT;
    const int tl = wi / TW, row = (wi % TW) / ROW16;
    ld_rel[i] = tl * TILE + row;
    wr_off[i] = tl * (TILE * STRIDE16) + row * STRIDE16 + tid % ROW16;
  }
  // (with overlapping tiles the wavefront groups' tiles start tstep rows apart in the buffer)
  const int rd_off = kg * (tstep * STRIDE16) + l32 * STRIDE16 + half;
  // interleaved: ceil(n / CHUNK) workgroups share ceil(n / (KG*TILE)) >= nch sets, at least one each
  const int sets_all = (ntiles + KG - 1) / KG;
  const int iters = INTER ? (sets_all - chunk + nch - 1) / nch : sets_all;
  // The workgroups of a head run side by side and their chunks lie a fixed power-of-two number
  // of bytes apart; if all of them walked their chunk from its first row, they would ask for
  // addresses that are equal modulo that distance at the same time, i.e. the same memory
  // channels.  Each workgroup therefore starts at a different point of its chunk and wraps
  // around (neither sweep depends on the order of the tiles).
  const int rot = (int)(((long long)chunk * iters) / nch);
  // Sweep 1 walks its chunk forwards from the rotated start; sweep 2 walks it backwards from
  // there, i.e. it begins with what sweep 1 read last.  Both sweeps have every chunk in flight
  // at once, so this, and not the order of the chunks, decides what the memory-side cache still
  // holds: reading a set slightly larger than a cache twice in the same direction hits nothing,
  // reading it back hits most of it.
  auto phys = [&](int it) {
    if (INTER) return chunk + it * nch;                // a set of the whole sequence
    if (PASS == 2) {
      const int p = rot - 1 - it;
      return p < 0 ? p + iters : p;
    }
    const int p = it + rot;
    return p >= iters ? p - iters : p;
  };

  // Branch-free on purpose (the compiler can only keep older loads in flight across a wait if
  // the loads in between are issued on every path).  Rows are clamped into the range somebody
  // reads: past the end of the sequence they re-read row n-1 (masked out later), and of the two
  // halo tiles only the pool radius next to the chunk is fetched, the other rows repeat the
  // nearest needed one (a cache hit) and their results are never looked at.
  // tok_bytes < 2^24 is checked on the host.
  const int need_lo = INTER ? 0 : max(kc0 - pool_r, 0);
  const int need_hi = INTER ? n - 1 : min(kc1 - 1 + pool_r, n - 1);
  auto load_set = [&](u32x4 (&g)[LDPT], int it) {
    const int key0 = k0 + it * KG * tstep - (PR ? pool_r : 0);   // first key of the iteration
    // both bounds are kept at or above zero, so the clamped row is never negative (it goes
    // through an unsigned 24-bit multiply); key0 <= need_hi holds by the choice of k1 above
    const int lim = max(need_hi - key0, 0), lo = max(need_lo - key0, 0);
    const char *sb = kbase + (size_t)key0 * tok_bytes;
#pragma unroll
    for (int i = 0; i < LDPT; ++i) {
      const unsigned off =
          __umul24((unsigned)max(min(ld_rel[i], lim), lo), (unsigned)tok_bytes) + col_bytes;
      g[i] = *reinterpret_cast<const u32x4 *>(sb + off);
    }
  };
  auto store_set = [&](const u32x4 (&g)[LDPT], int buf) {
#pragma unroll
    for (int i = 0; i < LDPT; ++i) kt[buf][wr_off[i]] = g[i];
  };

  // Sweep 2 without a caller's log-sum-exp combines sweep 1's partial (max, sum) of this head's
  // rows over the sequence's chunks.  With at least as many threads as (padded) rows, SL
  // threads share a row and each takes every SL-th chunk; with fewer, a thread combines RPT
  // rows one after the other.  CB chunks are loaded at a time, and the first CB of the first
  // row are requested before anything else: loads return in order, and these come from the
  // cache while the K rows below come from memory, so the combination runs in the shadow of
  // the first K round trip instead of after it.
  constexpr int CB = 32;
  constexpr int SL = NT >= RPAD ? NT / RPAD : 1;
  constexpr int RPT = NT >= RPAD ? 1 : RPAD / NT;
  constexpr int RSTEP = RPAD / RPT;            // rows combined side by side
  static_assert(SL * RSTEP == NT && RPT * RSTEP == RPAD, "threads and rows must tile each other");
  const int qi = tid % RSTEP, sl = tid / RSTEP;
  const int kend = ct.off[b + 1];
  float2 pml[PASS == 2 ? CB : 1];              // (max, sum) of CB chunks
  auto load_parts = [&](int k0c, int row) {
#pragma unroll
    for (int u = 0; u < CB; ++u) {
      const int k = min(k0c + u * SL, kend - 1);
      const size_t o = (size_t)k * RQ + (size_t)c * R + min(row, R - 1);
      pml[u] = part[o];
    }
  };
  if (PASS == 2 && !lse) load_parts(ct.off[b] + sl, qi);

  // The first two tile sets are requested next; the combination and the loads of the query
  // fragments (further down, so that they do not hold registers while the partials do) happen
  // in the shadow of that round trip.
  u32x4 g[DEPTH][LDPT];
#pragma unroll
  for (int j = 0; j < DEPTH; ++j) load_set(g[j], phys(min(j, iters - 1)));

  // sweep 2: log2-domain log-sum-exp of the 16 rows a lane sees in each row block; +inf on the
  // padding rows makes their weights exactly zero
  float l2[PASS == 2 ? MB : 1][16];
  if (PASS == 2) {
    float *sh_lse = &sh_rows[0][0][0];       // RPAD floats
    if (lse) {
      for (int i = tid; i < RPAD; i += NT) sh_lse[i] = (i < R) ? lse[head_row0 + i] * LOG2E : INFINITY;
    } else {
      // fold the partials in: first the largest maximum of a batch, then every sum scaled to it
      // (independent exponentials instead of a chain of rescalings)
#pragma unroll
      for (int rr = 0; rr < RPT; ++rr) {
        const int row = qi + rr * RSTEP;
        float M = -INFINITY, L = 0.0f;
        for (int k0c = ct.off[b] + sl; k0c < kend; k0c += CB * SL) {
          if (rr > 0 || k0c != ct.off[b] + sl) load_parts(k0c, row);
          float bm = -INFINITY;
#pragma unroll
          for (int u = 0; u < CB; ++u)
            if (k0c + u * SL < kend) bm = fmaxf(bm, pml[u].x * LOG2E);
          const float nm = fmaxf(M, bm);
          const float ref = (nm == -INFINITY) ? 0.0f : nm;
          float acc = L * fast_exp2(M - ref);
#pragma unroll
          for (int u = 0; u < CB; ++u)
            if (k0c + u * SL < kend) acc += pml[u].y * fast_exp2(pml[u].x * LOG2E - ref);
          L = acc;
          M = nm;
        }
        sh_cm[sl * RPAD + row] = M;
        sh_cl[sl * RPAD + row] = L;
      }
      __syncthreads();
      for (int row = tid; row < RPAD; row += NT) {
        float Mt = -INFINITY;
#pragma unroll
        for (int i = 0; i < SL; ++i) Mt = fmaxf(Mt, sh_cm[i * RPAD + row]);
        const float ref = (Mt == -INFINITY) ? 0.0f : Mt;
        float Lt = 0.0f;
#pragma unroll
        for (int i = 0; i < SL; ++i) Lt += sh_cl[i * RPAD + row] * fast_exp2(sh_cm[i * RPAD + row] - ref);
        sh_lse[row] = (row < R) ? Mt + __builtin_amdgcn_logf(Lt) : INFINITY;
      }
    }
    __syncthreads();
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        l2[mb][r] = sh_lse[row0 + mb * 32 + 8 * (r / 4) + 4 * half + (r % 4)];
  }
  // ---- window queries of this wavefront as MFMA operands, kept for the whole chunk ----------
  // (rows past R are loaded from row R-1 and zeroed, so every load is unconditional)
  bf16x8 qf[MB][KS];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int row = row0 + mb * 32 + l32;
    const unsigned keep = row < R ? 0xFFFFFFFFu : 0u;
    const unsigned short *src = q + (head_row0 + min(row, R - 1)) * D + half * 8;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      u32x4 v = *reinterpret_cast<const u32x4 *>(src + s * 16);
      v &= keep;
      qf[mb][s] = as_bf16(v);
    }
  }

  // sweep 1: running statistics of the window row this lane owns in each row block
  float rm[MB], rl[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) { rm[mb] = -INFINITY; rl[mb] = 0.0f; }
  bool have_ref = false;                       // (the same for all lanes) a first tile has set rm
  constexpr bool LAZY_REF = RPAD > 128;


  // The matrix products of a tile and the softmax arithmetic on the PREVIOUS tile's products are
  // independent, so they are written back to back in one basic block: the scheduler interleaves
  // them and the exponentials of tile t run in the shadow of the MFMAs of tile t+1 (within one
  // wavefront, not only between the two wavefronts of a SIMD).
  auto mma = [&](const bf16x8 (&kf)[KS], floatx16 (&acc)[MB]) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      floatx16 a = {0};
#pragma unroll
      for (int s = 0; s < KS; ++s)
        a = PASS == 1 ? mfma16<F16>(kf[s], qf[mb][s], a) : mfma16<F16>(qf[mb][s], kf[s], a);
      acc[mb] = a;
    }
  };
  // softmax arithmetic of one finished tile; RAGGED masks keys at or past n
  auto epilogue = [&](auto ragged_tag, floatx16 (&acc)[MB], int tile) {
    constexpr bool RAGGED = decltype(ragged_tag)::value;
    const int base = k0 + tile * TILE;
    if (PASS == 1) {
      // acc[mb][r]: key base + 8*(r/4) + 4*half + r%4, window row row0 + mb*32 + l32
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        if (RAGGED) {
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (base + 8 * (r / 4) + 4 * half + (r % 4) >= n) acc[mb][r] = -INFINITY;
        }
        float tm = acc[mb][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) tm = fmaxf(tm, acc[mb][r]);
        const float nm = fmaxf(rm[mb], tm * c_log2);
        const float ref = (nm == -INFINITY) ? 0.0f : nm;
        float sum = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(acc[mb][r], c_log2, -ref));
        rl[mb] = rl[mb] * fast_exp2(rm[mb] - ref) + sum;
        rm[mb] = nm;
      }
    } else if (PR) {
      // acc[mb][r]: window row row0 + mb*32 + 8*(r/4) + 4*half + r%4, key k0 + tile*tstep - pool_r + l32.
      // The weights themselves are pooled: they are non-negative floats, whose order is the order
      // of their bit patterns, so one integer max with the neighbouring lane as its operand does a
      // step of the sliding maximum.  Keys outside the sequence count as weight 0, which never
      // wins (the pool window is clipped to the sequence).
      const int j = tile * tstep - pool_r + l32;       // key, counted from k0
      const unsigned inseq = (k0 + j >= 0 && k0 + j < n) ? 0xFFFFFFFFu : 0u;
      unsigned p[MB][16];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          p[mb][r] = __float_as_uint(fast_exp2(fmaf(acc[mb][r], c_log2, -l2[mb][r]))) & inseq;
      for (int t = 0; t < pool_r; ++t) {               // keys j .. j + pool_r
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) p[mb][r] = max(p[mb][r], wave_shift<0x130>(p[mb][r]));
      }
      for (int t = 0; t < pool_r; ++t) {               // keys j - pool_r .. j + pool_r
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) p[mb][r] = max(p[mb][r], wave_shift<0x138>(p[mb][r]));
      }
      float sum = 0.0f;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += __uint_as_float(p[mb][r]);
      sum += __shfl_xor(sum, 32);
      if (half == 0 && l32 >= pool_r && l32 < TILE - pool_r && j < k1 - k0) sh_part[rs][j] = sum;
    } else {
      // acc[mb][r]: window row row0 + mb*32 + 8*(r/4) + 4*half + r%4, key base + l32
      float sum = 0.0f;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(acc[mb][r], c_log2, -l2[mb][r]));
      sum += __shfl_xor(sum, 32);
      // keys past n in a ragged tile get a value nobody reads
      if (half == 0) sh_part[rs][tile * TILE + l32] = sum;   // key k0 + tile*TILE + l32
    }
  };
  // The common case of the loop below in one piece: the matrix instructions of the current tile
  // with the vector arithmetic of the previous (full) tile dealt out between them, a share in
  // front of every MFMA (the first share covers the wait for the tile's LDS operands), and a scheduling fence after every share so that the order survives: an MFMA
  // runs for tens of cycles in the matrix core while the wavefront goes on issuing vector
  // instructions, but only if vector instructions follow it in program order.
  auto fused_tile = [&](const bf16x8 (&kf)[KS], floatx16 (&accn)[MB], floatx16 (&acc)[MB], int tile,
                        auto &&between) {
    constexpr int SLOTS = MB * KS;               // matrix instructions per tile
    constexpr int BETWEEN_SLOT = 6;              // between() runs after this slot's matrix instruction
    constexpr int VALS = MB * 16;                // products of the previous tile per lane
    floatx16 a[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) a[mb] = floatx16{0};
    if (PASS == 1 && LAZY_REF && have_ref) {
      // (shapes with more than 128 window rows per KV head, which are bound by their arithmetic;
      // on the 128-row shapes the sweep is bound by memory and the shorter code measured 2 us slower)
      // Once a row has a reference, its tiles' exponentials are taken against that same reference
      // without looking for the tile's maximum first: a sum of exp2(x - ref) is as accurate for one
      // reference as for another as long as nothing overflows (x - ref < 128), and what underflows
      // (x - ref < -126) is negligible beside the term that set the reference, which is 1.  An
      // overflow shows as a sum that is not finite; the tile is then folded in again the careful way.
      float sum[MB];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) sum[mb] = 0.0f;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const int slot = s * MB + mb;
#pragma unroll
          for (int v = slot * VALS / SLOTS; v < (slot + 1) * VALS / SLOTS; ++v)
            sum[v / 16] += fast_exp2(fmaf(acc[v / 16][v % 16], c_log2, -rm[v / 16]));
          a[mb] = mfma16<F16>(kf[s], qf[mb][s], a[mb]);
          __builtin_amdgcn_sched_barrier(0);
          if (slot == BETWEEN_SLOT) { between(); __builtin_amdgcn_sched_barrier(0); }
        }
      }
      bool bad = false;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) bad |= !(sum[mb] < INFINITY);
      if (__any(bad)) {
        epilogue(std::false_type{}, acc, tile);
      } else {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) rl[mb] += sum[mb];
      }
    } else if (PASS == 1) {
      // slots 0 .. MB-1 find the row blocks' tile maxima, the others share the exponentials
      constexpr int ESLOTS = SLOTS - MB;
      float ref[MB], nmx[MB], sum[MB];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const int slot = s * MB + mb;
          if (slot < MB) {
            float tm = acc[slot][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tm = fmaxf(tm, acc[slot][r]);
            nmx[slot] = fmaxf(rm[slot], tm * c_log2);
            ref[slot] = (nmx[slot] == -INFINITY) ? 0.0f : nmx[slot];
            sum[slot] = 0.0f;
          } else {
            const int e = slot - MB;
#pragma unroll
            for (int v = e * VALS / ESLOTS; v < (e + 1) * VALS / ESLOTS; ++v)
              sum[v / 16] += fast_exp2(fmaf(acc[v / 16][v % 16], c_log2, -ref[v / 16]));
          }
          a[mb] = mfma16<F16>(kf[s], qf[mb][s], a[mb]);
          __builtin_amdgcn_sched_barrier(0);
          if (slot == BETWEEN_SLOT) { between(); __builtin_amdgcn_sched_barrier(0); }
        }
      }
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        rl[mb] = rl[mb] * fast_exp2(rm[mb] - ref[mb]) + sum[mb];
        rm[mb] = nmx[mb];
      }
      have_ref = true;
    } else {
      // The exponentials end two slots early, so that the exchange between the lane halves
      // travels through the LDS crossbar while the last two matrix instructions are issued.
      constexpr int ESLOTS = SLOTS - 2;
      float sum = 0.0f, other = 0.0f;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const int slot = s * MB + mb;
          if (slot < ESLOTS) {
#pragma unroll
            for (int v = slot * VALS / ESLOTS; v < (slot + 1) * VALS / ESLOTS; ++v)
              sum += fast_exp2(fmaf(acc[v / 16][v % 16], c_log2, -l2[v / 16][v % 16]));
          } else if (slot == ESLOTS) {
            other = __shfl_xor(sum, 32);
          }
          a[mb] = mfma16<F16>(qf[mb][s], kf[s], a[mb]);
          __builtin_amdgcn_sched_barrier(0);
          if (slot == BETWEEN_SLOT) { between(); __builtin_amdgcn_sched_barrier(0); }
        }
      }
      sum += other;
      // key k0 + tile*TILE + l32; both lane halves hold the same sum and store it (no branch)
      sh_part[rs][tile * TILE + l32] = sum;
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) accn[mb] = a[mb];
  };
  auto is_full = [&](int tile) { return k0 + tile * TILE + TILE <= n; };

  floatx16 accp[MB];                                   // products of the tile before the current one
  int prev_tile = -1;                                  // -1: none pending

  // iteration it: LDS buffer it%2 holds its tiles; register set gb is in flight with the loads of
  // it+1; set ga is free and takes it+DEPTH's
  auto step = [&](int it, u32x4 (&ga)[LDPT], u32x4 (&gb)[LDPT]) {
    bf16x8 kf[KS];
    const u32x4 *buf = kt[it & 1];
#pragma unroll
    for (int s = 0; s < KS; ++s) kf[s] = as_bf16(buf[rd_off + s * 2]);
    // always issued (the last iterations re-read the final set): a conditional load would make
    // the compiler wait for every outstanding load before the stores below.  With eight
    // wavefronts, all of a compute unit's wavefronts leave the barrier together and nothing
    // overlaps with the scalar address arithmetic of the load at the top of a tile; the weights
    // sweep issues it between the tile's matrix instructions instead (measured on the 512-row
    // shape: 153.5 -> 150.2 us; the statistics sweep, which has less other work between its
    // matrix instructions to hide a late load behind, lost 7 us and keeps it at the top).
    constexpr bool LOAD_BETWEEN = NW == 8 && PASS == 2;
    auto ask = [&]() { load_set(ga, phys(min(it + DEPTH, iters - 1))); };
    auto between = [&]() {
      if constexpr (LOAD_BETWEEN) ask();
    };
    if constexpr (!LOAD_BETWEEN) ask();
    const int tile = phys(it) * KG + kg;
    const bool have = tile < ntiles;
    if (!PR && have && prev_tile >= 0 && is_full(prev_tile)) {
      // the common case, straight-line: products of this tile, arithmetic of the previous one
      floatx16 accn[MB];
      fused_tile(kf, accn, accp, prev_tile, between);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) accp[mb] = accn[mb];
      prev_tile = tile;
    } else {
      if (prev_tile >= 0) {
        if (is_full(prev_tile)) epilogue(std::false_type{}, accp, prev_tile);
        else epilogue(std::true_type{}, accp, prev_tile);
      }
      prev_tile = -1;
      between();
      if (have) {
        mma(kf, accp);
        prev_tile = tile;
      }
    }
    store_set(gb, (it + 1) & 1);               // (after the last iteration nobody reads it: no branch)
    __syncthreads();
  };
  // Two iterations in one piece, for an even it (LDS buffers 0, 1 and register sets g[0], g[1] in
  // this order) whose two tile sets are full and follow a full tile: no decisions inside, and
  // the products alternate between two register sets instead of being copied.  Runs of such
  // pairs form a loop of their own, so that what the general step needs (which tile is ragged,
  // which is missing, whether anything is pending) is looked at once per run, not once per tile:
  // in the 512-row shapes a wavefront issued 185 to 200 instructions per tile, 40 to 48 of them
  // scalar and 6 to 9 branches, against the tile's own 16 + 96.
  constexpr bool PAIRS = !PR && DEPTH == 2 && NW == 8;   // (the smaller shapes are bound by memory and would pay with registers)
  const int plain_sets = min(ntiles / KG, (n - k0) / (KG * TILE));   // sets [0, plain_sets): every tile there and full
  auto pair = [&](int it) {
    constexpr bool LOAD_BETWEEN = NW == 8 && PASS == 2;
    bf16x8 kf[KS];
    floatx16 accq[MB];
    const int t0 = phys(it) * KG + kg, t1 = phys(it + 1) * KG + kg;
    auto ask0 = [&]() { load_set(g[0], phys(min(it + 2, iters - 1))); };
    auto ask1 = [&]() { load_set(g[1], phys(min(it + 3, iters - 1))); };
    auto nothing = [&]() {};
#pragma unroll
    for (int s = 0; s < KS; ++s) kf[s] = as_bf16(kt[0][rd_off + s * 2]);
    if constexpr (LOAD_BETWEEN) {
      fused_tile(kf, accq, accp, prev_tile, ask0);
    } else {
      ask0();
      fused_tile(kf, accq, accp, prev_tile, nothing);
    }
    store_set(g[1], 1);
    __syncthreads();
#pragma unroll
    for (int s = 0; s < KS; ++s) kf[s] = as_bf16(kt[1][rd_off + s * 2]);
    if constexpr (LOAD_BETWEEN) {
      fused_tile(kf, accp, accq, t0, ask1);
    } else {
      ask1();
      fused_tile(kf, accp, accq, t0, nothing);
    }
    store_set(g[0], 0);
    __syncthreads();
    prev_tile = t1;
  };
  {
    store_set(g[0], 0);
    __syncthreads();
    if constexpr (PAIRS) {
      int it = 0;
      while (it < iters) {
        if (!(it & 1) && it + 2 <= iters && prev_tile >= 0 && is_full(prev_tile) &&
            phys(it) < plain_sets && phys(it + 1) < plain_sets) {
          do {
            pair(it);
            it += 2;
          } while (it + 2 <= iters && phys(it) < plain_sets && phys(it + 1) < plain_sets);
        } else {
          if (it & 1) step(it, g[1], g[0]);
          else step(it, g[0], g[1]);
          ++it;
        }
      }
    } else {
      for (int it = 0; it < iters; it += DEPTH) {
#pragma unroll
        for (int j = 0; j < DEPTH; ++j)
          if (it + j < iters) step(it + j, g[j], g[(j + 1) % DEPTH]);
      }
    }
    if (prev_tile >= 0) {
      if (is_full(prev_tile)) epilogue(std::false_type{}, accp, prev_tile);
      else epilogue(std::true_type{}, accp, prev_tile);
    }
  }

  if (PASS == 1) {
    // merge the two lane halves (same window row, different keys), then the KG wavefront groups
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const float m2 = __shfl_xor(rm[mb], 32), s2 = __shfl_xor(rl[mb], 32);
      const float M = fmaxf(rm[mb], m2);
      const float ref = (M == -INFINITY) ? 0.0f : M;
      const float L = rl[mb] * fast_exp2(rm[mb] - ref) + s2 * fast_exp2(m2 - ref);
      if (half == 0) { sh_rows[0][wv][mb * 32 + l32] = M; sh_rows[1][wv][mb * 32 + l32] = L; }
    }
    __syncthreads();
    for (int qi = tid; qi < RPAD; qi += NT) {
      const int rsi = qi / RW, wi = qi % RW;
      float M = -INFINITY;
#pragma unroll
      for (int k = 0; k < KG; ++k) M = fmaxf(M, sh_rows[0][k * RS + rsi][wi]);
      const float ref = (M == -INFINITY) ? 0.0f : M;
      float L = 0.0f;
#pragma unroll
      for (int k = 0; k < KG; ++k)
        L += sh_rows[1][k * RS + rsi][wi] * fast_exp2(sh_rows[0][k * RS + rsi][wi] - ref);
      if (qi < R) {
        const size_t o = (size_t)cg * RQ + (size_t)c * R + qi;
        part[o] = make_float2(M * LN2, L);         // the maximum back in the natural-log domain
      }
    }
  } else {
    __syncthreads();
    // add the RS row groups in a fixed order, take the mean, then (halo != 0) the max-pool:
    // stride 1, same length, window clipped to the sequence (Section 4.1: kernel 7)
    const float inv = 1.0f / (float)R;
    const int span = k1 - k0;
    if (tc.hist0) {                              // (the barrier above was the last use of the K tiles)
      for (int i = tid; i < RADIX_BINS; i += NT) sh_hist[i] = 0u;
    }
    for (int j = tid; j < span; j += NT) {
      float tot = 0.0f;
#pragma unroll
      for (int i = 0; i < RS; ++i) tot += sh_part[i][j];
      sh_part[0][j] = tot * inv;
    }
    __syncthreads();
    float *dst = out + st.score_off[b] + (size_t)c * n;
    const int r = halo ? dm.pool_k / 2 : 0;
    // A thread pools KPT keys at once, one window offset at a time, so that KPT independent LDS
    // reads are in flight instead of one chain per key.  Offsets that leave the sequence are
    // clamped onto its ends (taking an element of the window twice does not change a maximum);
    // a thread's keys past the chunk end repeat the last key and are not written.
    constexpr int KPT = CHUNK / NT;
    static_assert(CHUNK % NT == 0, "every thread pools the same number of keys");
    float pooled[KPT];
    int pk[KPT];
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      pk[i] = min(kc0 + tid + i * NT, kc1 - 1);
      pooled[i] = -INFINITY;
    }
    for (int t = -r; t <= r; ++t) {
#pragma unroll
      for (int i = 0; i < KPT; ++i)
        pooled[i] = fmaxf(pooled[i], sh_part[0][min(max(pk[i] + t, 0), n - 1) - k0]);
    }
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      if (kc0 + tid + i * NT < kc1) {
        dst[pk[i]] = pooled[i];
        if (tc.hist0) atomicAdd(&sh_hist[key_of(pooled[i]) >> 21], 1u);
      }
    }
    if (tc.hist0) {
      __syncthreads();
      unsigned *gh = tc.hist0 + (size_t)(b * h + c) * RADIX_BINS;
      unsigned *gt = tc.hist_tot0 + (size_t)b * RADIX_BINS;
      for (int i = tid; i < RADIX_BINS; i += NT) {
        const unsigned v = sh_hist[i];
        if (v) {
          atomicAdd(&gh[i], v);
          atomicAdd(&gt[i], v);
        }
      }
    }
  }
}

template <bool F16, int D, int MB, int RS, int KG, int CHUNK>
void run_mfma(const MfmaVariant &v, const SeqTab &st, const Dims &dm, const void *q, const void *K,
              const float *row_lse, float *scores, char *ws, const ScorePlan &pl,
              const TopkCarry &tc, bool pool_rows, hipStream_t s) {
  const ChunkTab ct = make_chunks(st, CHUNK);
  const int nblk = ct.off[st.batch] * dm.h_kv;
  const float c_log2 = dm.scale * LOG2E;
  float2 *part = (float2 *)(ws + pl.part);
  float *lse = (float *)(ws + pl.lse), *raw = (float *)(ws + pl.raw);
  const dim3 block(64 * RS * KG);
  const bool fuse_lse = v.fuse_lse, fuse_pool = v.fuse_pool;
  const float *use_lse = row_lse;
  if (!row_lse) {
    ADAKV_LAUNCH("score_stats_mfma", (score_mfma_kernel<D, MB, RS, KG, CHUNK, 1, F16>), dim3(nblk),
                 block, s, st, ct, dm, c_log2, (const unsigned short *)q,
                 (const unsigned short *)K, (const float *)nullptr, part,
                 (float *)nullptr, 0, tc);
    if (!fuse_lse) {
      launch_lse_combine(st, ct, dm.h_q * dm.w, part, lse, s);
      use_lse = lse;
    }
  } else if (tc.zero_begin) {
    launch_topk_clear(tc, s);                 // no statistics sweep to do the clearing
  }
  if (pool_rows) {
    // the printed order of Alg. 2 l.4: the sweep pools every row itself and writes final scores
    ADAKV_LAUNCH("score_weights_mfma", (score_mfma_kernel<D, MB, RS, KG, CHUNK, 2, F16, true>),
                 dim3(nblk), block, s, st, ct, dm, c_log2, (const unsigned short *)q,
                 (const unsigned short *)K, use_lse, part, scores, 0, tc);
    return;
  }
  ADAKV_LAUNCH("score_weights_mfma", (score_mfma_kernel<D, MB, RS, KG, CHUNK, 2, F16>), dim3(nblk),
               block, s, st, ct, dm, c_log2, (const unsigned short *)q, (const unsigned short *)K,
               use_lse, part, fuse_pool ? scores : raw, fuse_pool ? 1 : 0, tc);
  if (!fuse_pool) launch_pool(st, dm, raw, scores, s);
}

template <int D, bool F16>
hipError_t run_mfma_d(const MfmaVariant &v, const SeqTab &st, const Dims &dm, const void *q,
                      const void *K, const float *row_lse, float *scores, char *ws,
                      const ScorePlan &pl, const TopkCarry &tc, bool pool_rows, hipStream_t s) {
#define ADAKV_MFMA_CASE(MB, RS, KG, CHUNK)                                                      \
  if (v.mb == MB && v.rs == RS && v.kg == KG && v.chunk == CHUNK) {                             \
    run_mfma<F16, D, MB, RS, KG, CHUNK>(v, st, dm, q, K, row_lse, scores, ws, pl, tc, pool_rows, s); \
    return hipGetLastError();                                                                   \
  }
  ADAKV_MFMA_CASE(1, 1, 4, 2048)
  ADAKV_MFMA_CASE(2, 1, 4, 2048)
  ADAKV_MFMA_CASE(2, 2, 2, 4096)
  ADAKV_MFMA_CASE(2, 2, 2, 2048)
  ADAKV_MFMA_CASE(2, 2, 2, 1024)
  ADAKV_MFMA_CASE(2, 2, 2, 512)
  ADAKV_MFMA_CASE(2, 4, 1, 2048)
  ADAKV_MFMA_CASE(2, 4, 1, 1024)
  if constexpr (D == 128) { ADAKV_MFMA_CASE(2, 8, 1, 2048) ADAKV_MFMA_CASE(2, 8, 1, 4096) }
  else { ADAKV_MFMA_CASE(4, 4, 1, 1024) }
#undef ADAKV_MFMA_CASE
  return hipErrorInvalidValue;                 // a variant nobody instantiated
}

}  // namespace

// The instantiations are split over four translation units by head dimension and element type,
// so that they compile side by side: ADAKV_MFMA_PART = 1 .. 4 builds one quarter (part 1 also the
// host functions below), 0 or undefined everything.
#ifndef ADAKV_MFMA_PART
#define ADAKV_MFMA_PART 0
#endif
#define ADAKV_MFMA_ARGS                                                                          \
  const MfmaVariant &v, const SeqTab &st, const Dims &dm, const void *q, const void *K,          \
      const float *row_lse, float *scores, char *ws, const ScorePlan &pl, const TopkCarry &tc,   \
      bool pool_rows, hipStream_t s
hipError_t run_mfma_d64_bf16(ADAKV_MFMA_ARGS);
hipError_t run_mfma_d64_fp16(ADAKV_MFMA_ARGS);
hipError_t run_mfma_d128_bf16(ADAKV_MFMA_ARGS);
hipError_t run_mfma_d128_fp16(ADAKV_MFMA_ARGS);
#if ADAKV_MFMA_PART == 0 || ADAKV_MFMA_PART == 1
hipError_t run_mfma_d64_bf16(ADAKV_MFMA_ARGS) { return run_mfma_d<64, false>(v, st, dm, q, K, row_lse, scores, ws, pl, tc, pool_rows, s); }
#endif
#if ADAKV_MFMA_PART == 0 || ADAKV_MFMA_PART == 2
hipError_t run_mfma_d64_fp16(ADAKV_MFMA_ARGS) { return run_mfma_d<64, true>(v, st, dm, q, K, row_lse, scores, ws, pl, tc, pool_rows, s); }
#endif
#if ADAKV_MFMA_PART == 0 || ADAKV_MFMA_PART == 3
hipError_t run_mfma_d128_bf16(ADAKV_MFMA_ARGS) { return run_mfma_d<128, false>(v, st, dm, q, K, row_lse, scores, ws, pl, tc, pool_rows, s); }
#endif
#if ADAKV_MFMA_PART == 0 || ADAKV_MFMA_PART == 4
hipError_t run_mfma_d128_fp16(ADAKV_MFMA_ARGS) { return run_mfma_d<128, true>(v, st, dm, q, K, row_lse, scores, ws, pl, tc, pool_rows, s); }
#endif
#undef ADAKV_MFMA_ARGS

#if ADAKV_MFMA_PART == 0 || ADAKV_MFMA_PART == 1
// 16-bit inputs with at most 512 window rows per KV head (g*w); anything else takes the FMA path.
bool mfma_path_supported(const Dims &dm, int dtype) {
  return (dtype == ADAKV_BF16 || dtype == ADAKV_FP16) && dm.g * dm.w <= 512 && (dm.d == 64 || dm.d == 128) &&
         dm.k_stride_tok * 2 < (1ll << 24);   // 24-bit multiplies address a row inside a tile set
}

// The one place that decides which instantiation scores a layer: rows per wavefront and the
// split of a workgroup's wavefronts over window rows (RS) and keys (KG) follow the number of
// window rows per KV head; the chunk length follows the number of workgroups.
MfmaVariant choose_mfma_variant(const SeqTab &st, const Dims &dm) {
  MfmaVariant v;
  const int R = dm.g * dm.w;
  if (R <= 32) v = {1, 1, 4, 2048, false, false};
  else if (R <= 64) v = {2, 1, 4, 2048, false, false};
  else if (R <= 128) {
    // chunk length: long chunks amortise the per-workgroup set-up, but every compute unit wants
    // a few workgroups to choose from
    long long keys = 0;
    for (int b = 0; b < st.batch; ++b) keys += st.n[b];
    const long long wg2048 = (keys / 2048 + st.batch) * dm.h_kv;
    // 4096 keys when that alone nearly fills the 512 workgroups the chip holds at a time (seven
    // eighths of them): one round of long workgroups instead of almost two of short ones
    // (`llama8b_ragged`: 904 workgroups of 2048 keys or 472 of 4096, 279 -> 271 us per layer)
    long long wg4096 = 0;
    for (int b = 0; b < st.batch; ++b) wg4096 += (st.n[b] + 4095) / 4096;
    wg4096 *= dm.h_kv;
    const int chunk = 8 * wg4096 >= 7 * CHUNK_SWITCH_WGS ? 4096
                      : wg2048 >= CHUNK_SWITCH_WGS ? 2048 : 2 * wg2048 >= CHUNK_SWITCH_WGS ? 1024 : 512;
    v = {2, 2, 2, chunk, false, false};
  } else if (R <= 256) {
    // (the same rule one chunk length down: these workgroups carry twice the rows)
    long long wg2048 = 0;
    for (int b = 0; b < st.batch; ++b) wg2048 += (st.n[b] + 2047) / 2048;
    wg2048 *= dm.h_kv;
    v = {2, 4, 1, 8 * wg2048 >= 7 * CHUNK_SWITCH_WGS ? 2048 : 1024, false, false};
  }
  // 512 rows: eight wavefronts of 64 rows; with d = 64 a row block needs half the registers and
  // a tile half the loads, so four wavefronts of 128 rows.  Eight wavefronts fill a compute unit,
  // so nothing overlaps with a workgroup's set-up and epilogue (about 4 and 7 us in the two
  // sweeps): chunks of 2048 keys halve their number (measured on 131072 keys: 157 -> 145 and
  // 175 -> 155 us for the two sweeps).
  else if (dm.d == 128) {
    long long keys = 0;
    for (int b = 0; b < st.batch; ++b) keys += st.n[b];
    // 4096 keys when that still gives every compute unit a workgroup (one round instead of two)
    const long long wg4096 = (keys / 4096 + st.batch) * dm.h_kv;
    v = {2, 8, 1, wg4096 >= 256 ? 4096 : 2048, false, false};
  }
  else v = {4, 4, 1, 1024, false, false};
  // Fused forms: sweep 2 combines sweep 1's partial statistics itself unless a head has so many
  // (chunks x rows) that every workgroup re-reading them would cost more than a kernel, and it
  // applies the max-pool itself when the pool radius fits into the one-tile halo.
  const ChunkTab ct = make_chunks(st, v.chunk);
  int max_chunks = 0;
  for (int b = 0; b < st.batch; ++b)
    max_chunks = ct.off[b + 1] - ct.off[b] > max_chunks ? ct.off[b + 1] - ct.off[b] : max_chunks;
  v.fuse_lse = (long long)max_chunks * R <= 8192;
  v.fuse_pool = dm.pool_k / 2 <= TILE;
  return v;
}

hipError_t launch_score_mfma(const SeqTab &st, const Dims &dm, int dtype, const void *q,
                             const void *K, const float *row_lse, float *scores, char *ws,
                             const ScorePlan &pl, const TopkCarry &tc, bool pool_rows,
                             hipStream_t s) {
  const MfmaVariant v = choose_mfma_variant(st, dm);
  if (dtype == ADAKV_FP16)
    return dm.d == 64 ? run_mfma_d64_fp16(v, st, dm, q, K, row_lse, scores, ws, pl, tc, pool_rows, s)
                      : run_mfma_d128_fp16(v, st, dm, q, K, row_lse, scores, ws, pl, tc, pool_rows, s);
  return dm.d == 64 ? run_mfma_d64_bf16(v, st, dm, q, K, row_lse, scores, ws, pl, tc, pool_rows, s)
                    : run_mfma_d128_bf16(v, st, dm, q, K, row_lse, scores, ws, pl, tc, pool_rows, s);
}

// The printed order of Alg. 2 l.4 (pool every row, then average) runs on the matrix cores as long
// as a tile keeps at least 18 of its 32 lanes (pool radius up to 7); wider pools take the FMA path.
bool mfma_pool_rows_supported(const Dims &dm, int dtype) {
  return mfma_path_supported(dm, dtype) && dm.pool_k / 2 <= MFMA_POOL_ROWS_MAX_RADIUS;
}
#endif  // ADAKV_MFMA_PART == 0 || ADAKV_MFMA_PART == 1

}  // namespace adakv
