// Observation-window scoring (Alg. 2 lines 1-5, group mean of Section 3.5) for bf16 inputs on
// the gfx950 matrix cores: logits = Q_win K^T as v_mfma_f32_32x32x16_bf16 tiles with fp32
// accumulation, softmax and reductions in fp32 on the vector ALUs.
//
// The softmax of Alg. 2 l.3 needs every window row's denominator before the rows of a head can
// be added up, so K is swept twice:
//   sweep 1 (PASS 1)  per-row (max, sum of exp) over the keys        -> partial statistics
//   sweep 2 (PASS 2)  exp(logit - lse) summed over the g*w rows      -> pre-pool scores
// Sweep 2 walks the key chunks in the opposite order, so it starts on what sweep 1 left in the
// memory-side cache.  A caller-supplied row_lse skips sweep 1.
//
// Work split.  A workgroup (4 wavefronts) owns CHUNK consecutive keys of one KV head; all g
// query heads of the group share every K tile.  A wavefront keeps up to 128 window rows of Q in
// registers as MFMA operands for the whole chunk (MB blocks of 32 rows); RS wavefronts split
// the rows when the head has more than 128, and the 4/RS groups of wavefronts take the 32-key
// tiles of the chunk in turn.  A K tile travels HBM -> registers (coalesced 16-byte loads, whole
// 256-byte rows) -> the wavefront's own LDS slot (padded rows) -> registers in operand layout.
//
// Operand roles differ between the sweeps because of what the accumulator layout makes cheap
// (D[i][j]: lane = column j, 16 rows i per lane):
//   sweep 1: D = K_tile Q^T, a lane owns ONE window row and 16 keys: running (max, sum) per
//            lane, nothing crosses lanes until the chunk is done;
//   sweep 2: D = Q K_tile^T, a lane owns ONE key and 16 window rows: the sum over rows is
//            lane-local adds plus one cross-half add.
#include <math.h>

#include "common.h"

namespace adakv {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int MFMA_CHUNK = 2048;   // keys per workgroup
constexpr int TILE = 32;           // keys per MFMA tile

union Frag {
  uint4 u;
  bf16x8 v;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D, int MB, int RS, int PASS>
__global__ __launch_bounds__(256) void score_mfma_kernel(
    SeqTab st, ChunkTab ct, Dims dm, float c_log2, const unsigned short *__restrict__ q,
    const unsigned short *__restrict__ K, const float *__restrict__ lse,
    float *__restrict__ part_m, float *__restrict__ part_l, float *__restrict__ raw) {
  constexpr int KS = D / 16;                 // MFMA k-steps per tile
  constexpr int ROW16 = D * 2 / 16;          // 16-byte words per K row
  constexpr int STRIDE16 = ROW16 + 1;        // padded LDS row, in 16-byte words
  constexpr int LPR = ROW16;                 // lanes that load one row
  constexpr int RPI = 64 / LPR;              // rows per load instruction
  constexpr int NLD = TILE / RPI;            // load instructions per tile
  constexpr int KG = 4 / RS;                 // wavefront groups that take different tiles
  constexpr int RW = 32 * MB;                // window rows per wavefront

  __shared__ uint4 kt[4][TILE * STRIDE16];   // one K tile slot per wavefront
  __shared__ float sh_a[4][RW];              // sweep 1: per-wave row max; sweep 2: partial sums
  __shared__ float sh_b[4][RW];              // sweep 1: per-wave row sum

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const int kg = wv / RS, rs = wv % RS;
  const int h = dm.h_kv;
  const int total_chunks = ct.off[st.batch];
  const int c = blockIdx.x % h;
  int cg = blockIdx.x / h;
  if (PASS == 2) cg = total_chunks - 1 - cg;
  const int b = find_seq(ct, st.batch, cg);
  const int chunk = cg - ct.off[b];
  const int n = st.n[b];
  const int R = dm.g * dm.w, RQ = dm.h_q * dm.w;
  const int k0 = chunk * MFMA_CHUNK;
  const int k1 = min(n, k0 + MFMA_CHUNK);
  const int ntiles = (k1 - k0 + TILE - 1) / TILE;
  const int row0 = rs * RW;                  // first window row of this wavefront

  // ---- window queries of this wavefront as MFMA operands, kept for the whole chunk ----------
  Frag qf[MB][KS];
  {
    const unsigned short *qhead = q + ((size_t)b * RQ + (size_t)c * R) * D;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int row = row0 + mb * 32 + l32;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        if (row < R)
          qf[mb][s].u = *reinterpret_cast<const uint4 *>(qhead + (size_t)row * D + s * 16 + half * 8);
        else
          qf[mb][s].u = make_uint4(0u, 0u, 0u, 0u);
      }
    }
  }

  // sweep 2: log2-domain log-sum-exp of the 16 rows a lane sees in each row block
  float l2[PASS == 2 ? MB : 1][16];
  if (PASS == 2) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = row0 + mb * 32 + 8 * (r / 4) + 4 * half + (r % 4);
        l2[mb][r] = (row < R) ? lse[(size_t)b * RQ + (size_t)c * R + row] * 1.4426950408889634f
                              : INFINITY;
      }
  }
  // sweep 1: running statistics of the window row this lane owns in each row block
  float rm[MB], rl[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) { rm[mb] = -INFINITY; rl[mb] = 0.0f; }

  const char *kbase = reinterpret_cast<const char *>(K) +
                      ((size_t)st.tok_off[b] * dm.k_stride_tok + (size_t)c * dm.k_stride_head) * 2;
  const size_t tok_bytes = (size_t)dm.k_stride_tok * 2;
  const int ld_row = lane / LPR, ld_col = lane % LPR;
  uint4 *slot = kt[wv];

  uint4 g[NLD];
  auto load_tile = [&](int tile) {
    const int base = k0 + tile * TILE;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int key = min(base + i * RPI + ld_row, n - 1);   // rows past the end re-read the last
      g[i] = *reinterpret_cast<const uint4 *>(kbase + (size_t)key * tok_bytes + ld_col * 16);
    }
  };

  const int iters = (ntiles + KG - 1) / KG;
  if (kg < ntiles) load_tile(kg);
  for (int it = 0; it < iters; ++it) {
    const int tile = it * KG + kg;
    const bool active = tile < ntiles;
    Frag kf[KS];
    if (active) {
      // registers -> LDS slot -> operand layout (same wavefront writes and reads)
#pragma unroll
      for (int i = 0; i < NLD; ++i) slot[(i * RPI + ld_row) * STRIDE16 + ld_col] = g[i];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int s = 0; s < KS; ++s) kf[s].u = slot[l32 * STRIDE16 + s * 2 + half];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (tile + KG < ntiles) load_tile(tile + KG);           // next tile's loads fly during the math
    }
    const int base = k0 + tile * TILE;
    const bool ragged = base + TILE > n;

    if (PASS == 1) {
      if (active) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          floatx16 acc = {0};
#pragma unroll
          for (int s = 0; s < KS; ++s)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s].v, qf[mb][s].v, acc, 0, 0, 0);
          // acc[r]: key base + 8*(r/4) + 4*half + r%4, window row row0 + mb*32 + l32
          if (ragged) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (base + 8 * (r / 4) + 4 * half + (r % 4) >= n) acc[r] = -INFINITY;
          }
          float tm = acc[0];
#pragma unroll
          for (int r = 1; r < 16; ++r) tm = fmaxf(tm, acc[r]);
          const float nm = fmaxf(rm[mb], tm * c_log2);
          const float ref = (nm == -INFINITY) ? 0.0f : nm;
          float sum = 0.0f;
#pragma unroll
          for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(acc[r], c_log2, -ref));
          rl[mb] = rl[mb] * fast_exp2(rm[mb] - ref) + sum;
          rm[mb] = nm;
        }
      }
    } else {
      float sum = 0.0f;
      if (active) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          floatx16 acc = {0};
#pragma unroll
          for (int s = 0; s < KS; ++s)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[mb][s].v, kf[s].v, acc, 0, 0, 0);
          // acc[r]: window row row0 + mb*32 + 8*(r/4) + 4*half + r%4, key base + l32
#pragma unroll
          for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(acc[r], c_log2, -l2[mb][r]));
        }
        sum += __shfl_xor(sum, 32);
      }
      const int key = base + l32;
      if (RS == 1) {
        if (active && half == 0 && key < n)
          raw[st.score_off[b] + (size_t)c * n + key] = sum * (1.0f / (float)R);
      } else {
        // the RS wavefronts of a group hold partial sums over their own rows: add in fixed order
        if (active && half == 0) sh_a[wv][l32] = sum;
        __syncthreads();
        if (active && rs == 0 && half == 0 && key < n) {
          float tot = 0.0f;
#pragma unroll
          for (int i = 0; i < RS; ++i) tot += sh_a[kg * RS + i][l32];
          raw[st.score_off[b] + (size_t)c * n + key] = tot * (1.0f / (float)R);
        }
        __syncthreads();
      }
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
      if (half == 0) { sh_a[wv][mb * 32 + l32] = M; sh_b[wv][mb * 32 + l32] = L; }
    }
    __syncthreads();
    for (int qi = tid; qi < RW * RS; qi += 256) {
      const int rsi = qi / RW, wi = qi % RW;
      float M = -INFINITY;
#pragma unroll
      for (int k = 0; k < KG; ++k) M = fmaxf(M, sh_a[k * RS + rsi][wi]);
      const float ref = (M == -INFINITY) ? 0.0f : M;
      float L = 0.0f;
#pragma unroll
      for (int k = 0; k < KG; ++k) L += sh_b[k * RS + rsi][wi] * fast_exp2(sh_a[k * RS + rsi][wi] - ref);
      if (qi < R) {
        const size_t o = (size_t)cg * RQ + (size_t)c * R + qi;
        part_m[o] = M * 0.6931471805599453f;      // back to the natural-log domain
        part_l[o] = L;
      }
    }
  }
}

template <int D, int MB, int RS>
void run_mfma(const SeqTab &st, const Dims &dm, const void *q, const void *K,
              const float *row_lse, float *scores, char *ws, const ScorePlan &pl, hipStream_t s) {
  const ChunkTab ct = make_chunks(st, MFMA_CHUNK);
  const int nblk = ct.off[st.batch] * dm.h_kv;
  const float c_log2 = dm.scale * 1.4426950408889634f;
  float *part_m = (float *)(ws + pl.part_m), *part_l = (float *)(ws + pl.part_l);
  float *lse = (float *)(ws + pl.lse), *raw = (float *)(ws + pl.raw);
  const float *use_lse = row_lse;
  if (!row_lse) {
    ADAKV_LAUNCH("score_stats_mfma", (score_mfma_kernel<D, MB, RS, 1>), dim3(nblk), dim3(256), s,
                 st, ct, dm, c_log2, (const unsigned short *)q, (const unsigned short *)K,
                 (const float *)nullptr, part_m, part_l, (float *)nullptr);
    launch_lse_combine(st, ct, dm.h_q * dm.w, part_m, part_l, lse, s);
    use_lse = lse;
  }
  ADAKV_LAUNCH("score_weights_mfma", (score_mfma_kernel<D, MB, RS, 2>), dim3(nblk), dim3(256), s,
               st, ct, dm, c_log2, (const unsigned short *)q, (const unsigned short *)K, use_lse,
               (float *)nullptr, (float *)nullptr, raw);
  launch_pool(st, dm, raw, scores, s);
}

template <int D>
void run_mfma_d(const SeqTab &st, const Dims &dm, const void *q, const void *K,
                const float *row_lse, float *scores, char *ws, const ScorePlan &pl,
                hipStream_t s) {
  const int R = dm.g * dm.w;
  if (R <= 32) run_mfma<D, 1, 1>(st, dm, q, K, row_lse, scores, ws, pl, s);
  else if (R <= 64) run_mfma<D, 2, 1>(st, dm, q, K, row_lse, scores, ws, pl, s);
  else if (R <= 128) run_mfma<D, 4, 1>(st, dm, q, K, row_lse, scores, ws, pl, s);
  else if (R <= 256) run_mfma<D, 4, 2>(st, dm, q, K, row_lse, scores, ws, pl, s);
  else run_mfma<D, 4, 4>(st, dm, q, K, row_lse, scores, ws, pl, s);
}

}  // namespace

// bf16 inputs with at most 512 window rows per KV head (g*w); anything else takes the FMA path.
bool mfma_path_supported(const Dims &dm, int dtype) {
  return dtype == ADAKV_BF16 && dm.g * dm.w <= 512 && (dm.d == 64 || dm.d == 128);
}

hipError_t launch_score_mfma(const SeqTab &st, const Dims &dm, const void *q, const void *K,
                             const float *row_lse, float *scores, char *ws, const ScorePlan &pl,
                             hipStream_t s) {
  if (dm.d == 64) run_mfma_d<64>(st, dm, q, K, row_lse, scores, ws, pl, s);
  else run_mfma_d<128>(st, dm, q, K, row_lse, scores, ws, pl, s);
  return hipGetLastError();
}

}  // namespace adakv
