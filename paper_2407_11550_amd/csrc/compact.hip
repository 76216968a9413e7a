// Gather of the retained K/V rows into the flattened per-head cache (Alg. 2 lines 10-11,
// layout of Section 3.5).  Pure byte movement: a row of d elements is ROWB bytes, moved as
// 16-byte words by LPR = ROWB/16 neighbouring lanes, so a wavefront reads 64/LPR whole rows per
// load instruction and writes them to consecutive output rows (fully coalesced stores).
// With head-room (the decode-side layout) segment s is shifted down by s*headroom rows and its
// length is written to seg_len[s].
#include "common.h"

namespace adakv {

template <int LPR>
__global__ __launch_bounds__(256) void compact_kernel(
    SeqTab st, int h, int nseg, long long k_tok_b, long long k_head_b, long long v_tok_b,
    long long v_head_b, const char *__restrict__ K, const char *__restrict__ V,
    const int *__restrict__ indices, const int *__restrict__ cu, char *__restrict__ K_out,
    char *__restrict__ V_out, int rows_total, int w, int headroom, int *__restrict__ seg_len) {
  constexpr int RPB = 256 / LPR;   // rows per block
  const int t = blockIdx.x * RPB + threadIdx.x / LPR;
  const int lane = threadIdx.x % LPR;
  if (t >= rows_total) return;
  // segment s with cu[s] <= t < cu[s+1]; every segment holds at least the w window rows
  int lo = 0, hi = nseg;
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid;
  }
  const int b = lo / h, c = lo % h;
  // clamped into the sequence's own rows, so that a corrupt index can never leave the tensor
  const long long row = st.tok_off[b] + min(max(indices[t], 0), st.n[b] + w - 1);
  const uint4 kv = *reinterpret_cast<const uint4 *>(K + row * k_tok_b + c * k_head_b + lane * 16);
  const uint4 vv = *reinterpret_cast<const uint4 *>(V + row * v_tok_b + c * v_head_b + lane * 16);
  const long long o = (((long long)t + (long long)lo * headroom) * LPR + lane) * 16;
  if (seg_len && lane == 0 && t == cu[lo]) seg_len[lo] = cu[lo + 1] - cu[lo];
  *reinterpret_cast<uint4 *>(K_out + o) = kv;
  *reinterpret_cast<uint4 *>(V_out + o) = vv;
}

hipError_t launch_compact(const SeqTab &st, const Dims &dm, int dtype, const void *K,
                          const void *V, const int *indices, const int *cu_seqlens, void *K_out,
                          void *V_out, int headroom, int *seg_len, hipStream_t s) {
  const int esz = dtype == ADAKV_FP32 ? 4 : 2;
  const int rowb = dm.d * esz;
  const int lpr = rowb / 16;
  const int rows = st.out_off[st.batch];
  if (rows == 0) return hipSuccess;
  const int nseg = st.batch * dm.h_kv;
  const int rpb = 256 / lpr;
  dim3 grid((rows + rpb - 1) / rpb), block(256);
#define ADAKV_LAUNCH_COMPACT(LPR)                                                              \
  ADAKV_LAUNCH(seg_len ? "cache_build" : "compact", compact_kernel<LPR>, grid, block, s, st,   \
                     dm.h_kv, nseg,                                                            \
                     dm.k_stride_tok * esz, dm.k_stride_head * esz, dm.v_stride_tok * esz,     \
                     dm.v_stride_head * esz, (const char *)K, (const char *)V, indices,        \
                     cu_seqlens, (char *)K_out, (char *)V_out, rows, dm.w, headroom, seg_len)
  switch (lpr) {
    case 8: ADAKV_LAUNCH_COMPACT(8); break;
    case 16: ADAKV_LAUNCH_COMPACT(16); break;
    case 32: ADAKV_LAUNCH_COMPACT(32); break;
    default: return hipErrorInvalidValue;
  }
#undef ADAKV_LAUNCH_COMPACT
  return hipGetLastError();
}

}  // namespace adakv
