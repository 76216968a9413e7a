// Internal declarations shared by the translation units of libadakv.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include "adakv.h"

namespace adakv {

// Per-sequence facts, passed to kernels by value (kernel argument segment): the layer
// struct's host arrays never have to be copied to the device.
struct SeqTab {
  int batch;
  int n[ADAKV_MAX_BATCH];               // prefix length
  int Bp[ADAKV_MAX_BATCH];              // B' = B - w*h_kv
  long long tok_off[ADAKV_MAX_BATCH];   // first K/V row
  int score_off[ADAKV_MAX_BATCH + 1];   // h_kv * sum of earlier n: start of the sequence's scores
  int out_off[ADAKV_MAX_BATCH + 1];     // sum of earlier B: start of the sequence's output rows
};

// Start of each sequence's run of blocks along grid.x when a kernel cuts every sequence
// into fixed-size chunks of positions.
struct ChunkTab {
  int off[ADAKV_MAX_BATCH + 1];
};

inline ChunkTab make_chunks(const SeqTab &st, int chunk) {
  ChunkTab ct;
  ct.off[0] = 0;
  for (int b = 0; b < st.batch; ++b) ct.off[b + 1] = ct.off[b] + (st.n[b] + chunk - 1) / chunk;
  for (int b = st.batch + 1; b <= ADAKV_MAX_BATCH; ++b) ct.off[b] = ct.off[st.batch];
  return ct;
}

__device__ __forceinline__ int find_seq(const ChunkTab &ct, int batch, int blk) {
  int b = 0;
  while (b + 1 < batch && blk >= ct.off[b + 1]) ++b;
  return b;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Dims {
  int h_q, h_kv, g, d, w, pool_k;
  float scale;      // logit scale actually applied
  int alpha_fix;    // alpha in 16 fractional bits, rounded to nearest
  long long k_stride_tok, k_stride_head, v_stride_tok, v_stride_head;
};

constexpr int RADIX_BINS = 2048;   // 11-bit digits: passes take bits 31..21, 20..10, 9..0
constexpr int SEL_CHUNK = 4096;    // positions per block in the histogram and emit kernels
constexpr int GEN_CHUNK = 256;     // keys per block in the plain-FMA scoring kernels

struct TopkCarry;

// Which instantiation of the MFMA scoring kernels a layer gets (score_mfma.hip).
struct MfmaVariant {
  int mb, rs, kg;      // 32-row blocks per wavefront; wavefronts along window rows, along keys
  int chunk;           // keys per workgroup
  bool fuse_lse;       // sweep 2 combines sweep 1's partial statistics itself
  bool fuse_pool;      // sweep 2 applies the max-pool itself
};
MfmaVariant choose_mfma_variant(const SeqTab &st, const Dims &dm);

// ---- scoring (score_generic.hip, score_mfma.hip) ------------------------------------------
struct ScorePlan {                  // byte offsets into the workspace
  size_t part;                      // [chunks][h_q*w] float2: partial row max, sum of exp
  size_t lse;                       // [batch][h_q][w]
  size_t raw;                       // [num_scores] pre-pool scores
  size_t total;
  int part_chunk;                   // keys per partial-statistics chunk
};
ScorePlan plan_score(const SeqTab &st, const Dims &dm, int dtype, bool on_mfma);
bool mfma_path_supported(const Dims &dm, int dtype);

hipError_t launch_score_generic(const SeqTab &st, const Dims &dm, int dtype, const void *q,
                                const void *K, const float *row_lse, float *scores, char *ws,
                                const ScorePlan &pl, bool pool_first, hipStream_t s);
hipError_t launch_score_mfma(const SeqTab &st, const Dims &dm, int dtype, const void *q,
                             const void *K, const float *row_lse, float *scores, char *ws,
                             const ScorePlan &pl, const TopkCarry &tc, bool pool_rows,
                             hipStream_t s);
bool mfma_pool_rows_supported(const Dims &dm, int dtype);   // ADAKV_FLAG_POOL_THEN_MEAN on the matrix cores

// ---- allocation and selection (select.hip) --------------------------------------------------
// A score becomes a 32-bit key whose unsigned order is the float order (+0.0f turns -0 into +0;
// non-negative floats order like their bit patterns, the general transform keeps the order for
// negative inputs too).  The first radix digit is the key's top 11 bits.
__device__ __forceinline__ unsigned key_of(float x) {
  const unsigned u = __float_as_uint(x + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Pipeline mode (ADAKV_FLAG_PIPELINE): the scoring call clears the Top-k histograms and files
// the first radix digit of every score it writes, so that allocation and selection start at
// their second pass.  Pointers into the Top-k part of the workspace; all null when off.
struct TopkCarry {
  unsigned *zero_begin;    // cleared before anything is counted
  unsigned zero_words;
  unsigned *hist0;         // u32 [batch*h][RADIX_BINS]  first-digit counts per head
  unsigned *hist_tot0;     // u32 [batch][RADIX_BINS]    the same summed over the heads of a sequence
};
bool carry_supported(const Dims &dm, int dtype);
TopkCarry plan_carry(const SeqTab &st, const Dims &dm, char *ws_topk);
void launch_topk_clear(const TopkCarry &tc, hipStream_t s);

size_t plan_topk_bytes(const SeqTab &st, const Dims &dm);
// carried: the first-digit histograms are already in the workspace and the rest is cleared
hipError_t launch_allocate(const SeqTab &st, const Dims &dm, const float *scores, int *budgets,
                           int *cu_seqlens, char *ws, bool carried, hipStream_t s);
hipError_t launch_select(const SeqTab &st, const Dims &dm, const float *scores,
                         const int *budgets, const int *cu_seqlens, int *indices, char *ws,
                         bool carried, hipStream_t s);

// ---- compaction (compact.hip) ---------------------------------------------------------------
hipError_t launch_compact(const SeqTab &st, const Dims &dm, int dtype, const void *K,
                          const void *V, const int *indices, const int *cu_seqlens, void *K_out,
                          void *V_out, int headroom, int *seg_len, hipStream_t s);

// ---- plain streaming read, a measurement aid (probe.hip) -------------------------------------
hipError_t launch_probe_read(const void *src, long long n16, void *sink, int blocks, hipStream_t s);
int probe_waves_per_block();

// ---- decode side of the flattened layout (decode.hip) -----------------------------------------
struct DecodePlan {
  int split;                        // rows of a segment per workgroup
  int nblk;                         // workgroups launched: an upper bound on what the lengths need
  size_t part_acc, part_ml;         // byte offsets of the per-workgroup partial results
  size_t seg_tab, total;            // per segment: first partial, partials, rows, appended
};
bool decode_supported(const Dims &dm);
DecodePlan plan_decode(const SeqTab &st, const Dims &dm, int headroom);
// k_new == nullptr: attention only (cache and lengths are only read)
hipError_t launch_decode_attn(const SeqTab &st, const Dims &dm, int dtype, int headroom,
                              const void *q, const void *k_new, const void *v_new, const int *cu,
                              void *Kc, void *Vc, int *seg_len, int *overflow, float *out,
                              float *lse, char *ws, hipStream_t s);
hipError_t launch_append(const SeqTab &st, const Dims &dm, int dtype, int headroom,
                         const void *k_new, const void *v_new, const int *cu, void *Kc, void *Vc,
                         int *seg_len, int *overflow, hipStream_t s);


// Profiling aid (adakv_trace_arm): while armed on this host thread, every kernel launch carries
// a pair of the caller's events that receive the kernel's own start and end timestamps.
bool trace_pair(const char *name, hipEvent_t *start, hipEvent_t *stop);
void launch_lse_combine(const SeqTab &st, const ChunkTab &ct, int RQ, const float2 *part,
                        float *lse, hipStream_t s);
void launch_pool(const SeqTab &st, const Dims &dm, const float *raw, float *scores,
                 hipStream_t s);

#define ADAKV_LAUNCH(name, kernel, grid, block, stream, ...)                                   \
  do {                                                                                         \
    hipEvent_t ev0_, ev1_;                                                                     \
    if (::adakv::trace_pair(name, &ev0_, &ev1_))                                               \
      hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, ev0_, ev1_, 0, __VA_ARGS__);       \
    else                                                                                       \
      hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);                         \
  } while (0)

}  // namespace adakv
