// Decode side of the flattened per-head cache (Section 3.5): the cache update of Eq. (1) and
// one decoding step of Eq. (2) per query head over segments of different lengths.
//
// Layout: segment s = b*h_kv + c starts at row cu[s] + s*headroom of K_cache / V_cache and holds
// seg_len[s] rows of ROWB = d*sizeof(T) bytes, so a segment is one contiguous byte range.
//
// Attention: HBM-bound (every cached K and V row is read once, 2*ROWB bytes for 4*g*d flops),
// and with g <= 8 query rows per segment far too thin for the matrix cores, so the products
// run on the vector ALUs.  A row is read by LPR = ROWB/16 neighbouring lanes, 16 bytes each:
// every load instruction of a wavefront fetches 64/LPR whole rows = 1 KB of consecutive memory.
// Segment lengths live on the device, so the host launches an upper bound of workgroups
// (capacity / split + segments); each workgroup finds its (segment, split) from a prefix sum of
// the lengths, writes partial (max, sum, weighted value sum) per query head, and a second kernel
// merges the splits of each segment.
#include <math.h>

#include "common.h"

namespace adakv {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float M_INIT = -1.0e30f;    // finite "no row seen yet" maximum: exp2(-inf - M_INIT) = 0

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false);
  return x + __builtin_bit_cast(float, y);
}

// Sum over the LPR neighbouring lanes that share a row; every one of them gets the sum.
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
  x = dpp_add<0xB1>(x);                       // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);                       // quad_perm [2,3,0,1]
  if (LPR >= 8) x = dpp_add<0x141>(x);        // row_half_mirror: lane i <-> 7-i
  if (LPR >= 16) x = dpp_add<0x140>(x);       // row_mirror: lane i <-> 15-i
  if (LPR >= 32) x += __shfl_xor(x, 16);
  return x;
}

template <typename T> struct Elem;
template <> struct Elem<unsigned short> {     // bf16: 8 elements per 16 bytes
  static constexpr int EPL = 8;
  static __device__ __forceinline__ void widen(u32x4 v, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __builtin_bit_cast(float, v[i] << 16);
      f[2 * i + 1] = __builtin_bit_cast(float, v[i] & 0xffff0000u);
    }
  }
};
struct f16_t { unsigned short bits; };        // IEEE half: tag type, same size as the bf16 tag
template <> struct Elem<f16_t> {
  static constexpr int EPL = 8;
  static __device__ __forceinline__ void widen(u32x4 v, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = (float)__builtin_bit_cast(_Float16, (unsigned short)(v[i] & 0xFFFFu));
      f[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (unsigned short)(v[i] >> 16));
    }
  }
};
template <> struct Elem<float> {
  static constexpr int EPL = 4;
  static __device__ __forceinline__ void widen(u32x4 v, float (&f)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned int word = v[i];          // a copy: bit_cast of the vector element itself
      f[i] = __builtin_bit_cast(float, word);  // reads element 0 for every i
    }
  }
};

// Rows of segment s this call works on: the rows held, plus the row the call itself appends
// (`grow` = 1) if the segment has room for it.
__device__ __forceinline__ int rows_held(const int *cu, const int *seg_len, int s, int headroom,
                                         int grow) {
  const int cap = cu[s + 1] - cu[s] + headroom;
  const int held = min(max(seg_len[s], 0), cap);   // a corrupt length can never leave the segment
  return held + (held < cap ? grow : 0);
}

// Blocks of `split` rows per segment, summed over the segments in front of segment `s_first` of
// this thread's run (thread t owns segments t*per .. t*per+per-1).  Returns the exclusive prefix;
// *total gets the sum over all segments.  One call per kernel, by all NWV wavefronts of the
// workgroup; uses sh[0..NWV-1].
template <int NWV = 4>
__device__ __forceinline__ int scan_blocks(int nseg, int per, int split, int headroom, int grow,
                                           const int *cu, const int *seg_len, int *sh,
                                           int *total) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int mine = 0;
  for (int i = 0; i < per; ++i) {
    const int s = tid * per + i;
    if (s < nseg) mine += (rows_held(cu, seg_len, s, headroom, grow) + split - 1) / split;
  }
  int inc = mine;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int y = __shfl_up(inc, o);
    if (lane >= o) inc += y;
  }
  if (lane == 63) sh[wv] = inc;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int i = 0; i < NWV; ++i) {
    const int v = sh[i];
    if (i < wv) before += v;
    all += v;
  }
  *total = all;
  return before + inc - mine;
}

// ---------------------------------------------------------------------------------------------
// Query heads one wavefront carries: at most four (queries and accumulators take 2*GW*EPL
// registers).  A larger group is split over NGRP sets of four wavefronts that read the
// same rows at the same time (the second read of a row is a cache hit).
template <typename T, int G> struct HeadSplit {
  static constexpr int GW = G > 4 ? 4 : G;
  static constexpr int NGRP = G / GW;
};

template <typename T, int D, int G>
__global__ __launch_bounds__((256 * HeadSplit<T, G>::NGRP)) void decode_attn_kernel(
    int nseg, int h, int per, int split, int headroom, float c_log2, const T *__restrict__ q,
    const char *__restrict__ k_new, const char *__restrict__ v_new, const int *__restrict__ cu,
    const int *__restrict__ seg_len, char *Kc, char *Vc, float *__restrict__ part_acc,
    float *__restrict__ part_ml, int4 *__restrict__ seg_tab) {
  constexpr int EPL = Elem<T>::EPL;
  constexpr int ROWB = D * (int)sizeof(T);
  constexpr int LPR = ROWB / 16;               // lanes per row
  constexpr int RPW = 64 / LPR;                // rows per wavefront load
  constexpr int NW = 4;                        // wavefronts that share the rows of a split
  constexpr int GW = HeadSplit<T, G>::GW, NGRP = HeadSplit<T, G>::NGRP;
  constexpr int NT = 256 * NGRP;
  constexpr int U = 4;                         // row loads in flight per lane, for K and for V

  __shared__ int sh_scan[24];                  // [0..15] the prefix sum's wavefront totals, [16..20] results
  __shared__ float sh_acc[NW][G][D];
  __shared__ float sh_m[NW][G], sh_l[NW][G];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv_all = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wv_all / NW, wv = wv_all % NW; // head set, and place among the set's wavefronts
  const int col = lane % LPR, slot = lane / LPR;

  // ---- which (segment, split) is this workgroup? -------------------------------------------
  // With k_new/v_new the call appends one row per segment (Eq. 1) and attends over it as well:
  // the row is taken from k_new/v_new by the lanes it falls to, which also store it in the cache.
  const int grow = k_new != nullptr ? 1 : 0;
  int total;
  const int excl = scan_blocks<NW * NGRP>(nseg, per, split, headroom, grow, cu, seg_len, sh_scan, &total);
  {
    int first = excl;
    for (int i = 0; i < per; ++i) {
      const int s = tid * per + i;
      if (s >= nseg) break;
      const int now = rows_held(cu, seg_len, s, headroom, grow);
      const int nb = (now + split - 1) / split;
      if ((int)blockIdx.x >= first && (int)blockIdx.x < first + nb) {
        sh_scan[16] = s;
        sh_scan[17] = (int)blockIdx.x - first;
        sh_scan[18] = now;
        sh_scan[19] = cu[s];
        sh_scan[20] = now - rows_held(cu, seg_len, s, headroom, 0);  // 1: the last row is the new one
      }
      // the merge kernel finds a segment's partial results through this table; the launch has at
      // least one workgroup per segment, and workgroup s files the entry of segment s
      if (s == (int)blockIdx.x)
        seg_tab[s] = make_int4(first, nb, now, now - rows_held(cu, seg_len, s, headroom, 0));
      first += nb;
    }
  }
  if ((int)blockIdx.x >= total) return;        // uniform: the launch is an upper bound
  __syncthreads();
  const int s = sh_scan[16], j = sh_scan[17], len = sh_scan[18];
  const int b = s / h, c = s % h;
  const int r0 = j * split, r1 = min(len, r0 + split);
  const int new_row = sh_scan[20] ? len - 1 : -1;
  const long long seg_byte = ((long long)sh_scan[19] + (long long)s * headroom) * ROWB + col * 16;
  char *Kb = Kc + seg_byte;
  char *Vb = Vc + seg_byte;
  const long long new_byte = (long long)s * ROWB + col * 16;

  // ---- the g query rows of this KV head, pre-scaled so that exp() becomes exp2() --------------
  float qf[GW][EPL];
#pragma unroll
  for (int gi = 0; gi < GW; ++gi) {
    const T *qp = q + ((long long)(b * h + c) * G + grp * GW + gi) * D + col * EPL;
    Elem<T>::widen(*reinterpret_cast<const u32x4 *>(qp), qf[gi]);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[gi][e] *= c_log2;
  }

  float m[GW], l[GW], acc[GW][EPL];
#pragma unroll
  for (int gi = 0; gi < GW; ++gi) {
    m[gi] = M_INIT; l[gi] = 0.0f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[gi][e] = 0.0f;
  }

  const int rows = r1 - r0;
  const int iters = (rows + U * NW * RPW - 1) / (U * NW * RPW);
  for (int it = 0; it < iters; ++it) {
    u32x4 kk[U], vv[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = r0 + ((it * U + u) * NW + wv) * RPW + slot;
      ok[u] = r < r1;
      const int rr = min(r, r1 - 1);                           // r1 >= 1: the block exists
      const long long o = (long long)rr * ROWB;
      // lanes past the end re-read the block's last row (and ignore it): if that is the new row,
      // they too must take it from k_new/v_new, its place in the cache is not written yet
      const bool fresh = rr == new_row;
      kk[u] = *reinterpret_cast<const u32x4 *>(fresh ? k_new + new_byte : Kb + o);
      vv[u] = *reinterpret_cast<const u32x4 *>(fresh ? v_new + new_byte : Vb + o);
      if (r == new_row && grp == 0) {
        *reinterpret_cast<u32x4 *>(Kb + o) = kk[u];
        *reinterpret_cast<u32x4 *>(Vb + o) = vv[u];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPL], sc[GW];
      Elem<T>::widen(kk[u], kf);
      bool grow = false;
#pragma unroll
      for (int gi = 0; gi < GW; ++gi) {
        float a = 0.0f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) a = fmaf(qf[gi][e], kf[e], a);
        a = row_sum<LPR>(a);
        sc[gi] = ok[u] ? a : -INFINITY;
        grow |= sc[gi] > m[gi];
      }
      if (__any(grow)) {                       // a new running maximum somewhere in the wavefront
#pragma unroll
        for (int gi = 0; gi < GW; ++gi) {
          const float mn = fmaxf(m[gi], sc[gi]);
          const float corr = fast_exp2(m[gi] - mn);
          l[gi] *= corr;
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[gi][e] *= corr;
          m[gi] = mn;
        }
      }
      float vf[EPL];
      Elem<T>::widen(vv[u], vf);
#pragma unroll
      for (int gi = 0; gi < GW; ++gi) {
        const float p = fast_exp2(sc[gi] - m[gi]);
        l[gi] += p;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[gi][e] = fmaf(p, vf[e], acc[gi][e]);
      }
    }
  }

  // ---- merge the RPW row slots of the wavefront, then the NW wavefronts of each head set --------
#pragma unroll
  for (int gi = 0; gi < GW; ++gi) {
    float M = m[gi];
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) M = fmaxf(M, __shfl_xor(M, o));
    const float f = fast_exp2(m[gi] - M);
    float ll = l[gi] * f;
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) ll += __shfl_xor(ll, o);
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float a = acc[gi][e] * f;
#pragma unroll
      for (int o = LPR; o < 64; o <<= 1) a += __shfl_xor(a, o);
      acc[gi][e] = a;
    }
    if (slot == 0) {
      const int head = grp * GW + gi;
#pragma unroll
      for (int e = 0; e < EPL; ++e) sh_acc[wv][head][col * EPL + e] = acc[gi][e];
      if (col == 0) { sh_m[wv][head] = M; sh_l[wv][head] = ll; }
    }
  }
  __syncthreads();
  for (int t = tid; t < G * D; t += NT) {
    const int gi = t / D, e = t % D;
    float M = sh_m[0][gi];
#pragma unroll
    for (int w2 = 1; w2 < NW; ++w2) M = fmaxf(M, sh_m[w2][gi]);
    float a = 0.0f, ll = 0.0f;
#pragma unroll
    for (int w2 = 0; w2 < NW; ++w2) {
      const float f = fast_exp2(sh_m[w2][gi] - M);
      a = fmaf(sh_acc[w2][gi][e], f, a);
      ll = fmaf(sh_l[w2][gi], f, ll);
    }
    part_acc[((long long)blockIdx.x * G + gi) * D + e] = a;
    if (e == 0) {
      part_ml[((long long)blockIdx.x * G + gi) * 2] = M;
      part_ml[((long long)blockIdx.x * G + gi) * 2 + 1] = ll;
    }
  }
}

// One workgroup per (segment, query head of its group) merges that segment's splits and
// normalises.  A long segment has hundreds of splits, so they are merged NSLOT side by side
// (each by D/4 lanes holding a float4 of the value sum), four loads deep, then across slots.
template <int D, int G>
__global__ __launch_bounds__(1024) void decode_combine_kernel(
    const int4 *__restrict__ seg_tab, int *__restrict__ seg_len, int *__restrict__ overflow,
    const float *__restrict__ part_acc, const float *__restrict__ part_ml,
    float *__restrict__ out, float *__restrict__ lse) {
  constexpr int LPE = D / 4;
  constexpr int NSLOT = 1024 / LPE;
  constexpr int UC = 4;
  __shared__ float sh_a[NSLOT][D];
  __shared__ float sh_m[NSLOT], sh_l[NSLOT];
  const int tid = threadIdx.x;
  const int s = blockIdx.x, gi = blockIdx.y;
  const int4 ent = seg_tab[s];                 // first partial, partials, rows now, 1 if a row was appended
  const int p0 = ent.x, cnt = ent.y;
  if (seg_len && gi == 0 && tid == 0) {        // the call appended: the new lengths become visible
    if (ent.w) seg_len[s] = ent.z;
    else if (overflow) *overflow = 1;          // the segment was full, its new row was dropped
  }
  const int e4 = tid % LPE, slot = tid / LPE;

  float m = M_INIT, l = 0.0f;
  float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  for (int p = slot; p < cnt; p += NSLOT * UC) {
    float2 ml[UC];
    float4 pa[UC];
#pragma unroll
    for (int u = 0; u < UC; ++u) {
      const int pp = p + u * NSLOT;
      const long long pg = (long long)(p0 + (pp < cnt ? pp : p)) * G + gi;
      ml[u] = *reinterpret_cast<const float2 *>(part_ml + pg * 2);
      pa[u] = *reinterpret_cast<const float4 *>(part_acc + pg * D + e4 * 4);
      if (pp >= cnt) { ml[u] = make_float2(M_INIT, 0.0f); pa[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f); }
    }
#pragma unroll
    for (int u = 0; u < UC; ++u) {
      const float mn = fmaxf(m, ml[u].x);
      const float fo = fast_exp2(m - mn), fn = fast_exp2(ml[u].x - mn);
      l = l * fo + ml[u].y * fn;
      a.x = a.x * fo + pa[u].x * fn; a.y = a.y * fo + pa[u].y * fn;
      a.z = a.z * fo + pa[u].z * fn; a.w = a.w * fo + pa[u].w * fn;
      m = mn;
    }
  }
  *reinterpret_cast<float4 *>(&sh_a[slot][e4 * 4]) = a;
  if (e4 == 0) { sh_m[slot] = m; sh_l[slot] = l; }
  __syncthreads();
  if (tid < D) {
    float M = sh_m[0];
#pragma unroll
    for (int k = 1; k < NSLOT; ++k) M = fmaxf(M, sh_m[k]);
    float acc = 0.0f, ll = 0.0f;
#pragma unroll 8
    for (int k = 0; k < NSLOT; ++k) {
      const float f = fast_exp2(sh_m[k] - M);
      acc = fmaf(sh_a[k][tid], f, acc);
      ll = fmaf(sh_l[k], f, ll);
    }
    const long long row = (long long)s * G + gi;       // = (b*h + c)*G + gi
    out[row * D + tid] = ll > 0.0f ? acc / ll : 0.0f;
    if (lse && tid == 0) lse[row] = ll > 0.0f ? (M + log2f(ll)) * LN2 : -INFINITY;
  }
}

// Eq. (1) for every segment: LPR lanes move the new K row and the new V row of one segment.
template <int LPR>
__global__ __launch_bounds__(256) void append_kernel(
    int nseg, int headroom, const char *__restrict__ k_new, const char *__restrict__ v_new,
    const int *__restrict__ cu, char *__restrict__ Kc, char *__restrict__ Vc,
    int *__restrict__ seg_len, int *__restrict__ overflow) {
  const int s = (blockIdx.x * 256 + threadIdx.x) / LPR;
  const int col = threadIdx.x % LPR;
  if (s >= nseg) return;
  const int cap = cu[s + 1] - cu[s] + headroom;
  const int len = seg_len[s];                  // read by all LPR lanes before lane 0 stores
  if (len < 0 || len >= cap) {
    if (col == 0 && overflow) *overflow = 1;
    return;
  }
  const uint4 kv = *reinterpret_cast<const uint4 *>(k_new + ((long long)s * LPR + col) * 16);
  const uint4 vv = *reinterpret_cast<const uint4 *>(v_new + ((long long)s * LPR + col) * 16);
  const long long o = (((long long)cu[s] + (long long)s * headroom + len) * LPR + col) * 16;
  *reinterpret_cast<uint4 *>(Kc + o) = kv;
  *reinterpret_cast<uint4 *>(Vc + o) = vv;
  if (col == 0) seg_len[s] = len + 1;
}

template <typename T, int D, int G>
void run_decode(const SeqTab &st, const Dims &dm, int headroom, const DecodePlan &pl,
                const void *q, const void *k_new, const void *v_new, const int *cu, void *Kc,
                void *Vc, int *seg_len, int *overflow, float *out, float *lse, char *ws,
                hipStream_t s) {
  const int nseg = st.batch * dm.h_kv;
  const int per = (nseg + 255) / 256;
  float *part_acc = (float *)(ws + pl.part_acc);
  float *part_ml = (float *)(ws + pl.part_ml);
  int4 *seg_tab = (int4 *)(ws + pl.seg_tab);
  ADAKV_LAUNCH("decode_attn", (decode_attn_kernel<T, D, G>), dim3(pl.nblk),
               dim3(256 * HeadSplit<T, G>::NGRP), s, nseg,
               dm.h_kv, per, pl.split, headroom, dm.scale * LOG2E, (const T *)q,
               (const char *)k_new, (const char *)v_new, cu, (const int *)seg_len, (char *)Kc,
               (char *)Vc, part_acc, part_ml, seg_tab);
  // only a call that appends hands the lengths to the merge kernel for updating
  ADAKV_LAUNCH("decode_combine", (decode_combine_kernel<D, G>), dim3(nseg, G), dim3(1024), s,
               (const int4 *)seg_tab, k_new ? seg_len : nullptr, overflow, (const float *)part_acc,
               (const float *)part_ml, out, lse);
}

struct DecodeArgs {
  const void *q, *k_new, *v_new;
  const int *cu;
  void *Kc, *Vc;
  int *seg_len, *overflow;
  float *out, *lse;
  char *ws;
};

template <typename T, int D>
bool run_decode_g(const SeqTab &st, const Dims &dm, int headroom, const DecodePlan &pl,
                  const DecodeArgs &a, hipStream_t s) {
#define ADAKV_DECODE_G(G)                                                                       \
  run_decode<T, D, G>(st, dm, headroom, pl, a.q, a.k_new, a.v_new, a.cu, a.Kc, a.Vc, a.seg_len,   \
                      a.overflow, a.out, a.lse, a.ws, s)
  switch (dm.g) {
    case 1: ADAKV_DECODE_G(1); return true;
    case 2: ADAKV_DECODE_G(2); return true;
    case 4: ADAKV_DECODE_G(4); return true;
    case 8: ADAKV_DECODE_G(8); return true;
    default: return false;
  }
#undef ADAKV_DECODE_G
}

}  // namespace

bool decode_supported(const Dims &dm) {
  return (dm.g == 1 || dm.g == 2 || dm.g == 4 || dm.g == 8) && (dm.d == 64 || dm.d == 128);
}

DecodePlan plan_decode(const SeqTab &st, const Dims &dm, int headroom) {
  DecodePlan pl;
  const long long nseg = (long long)st.batch * dm.h_kv;
  const long long cap = (long long)st.out_off[st.batch] + nseg * headroom;
  // Rows per workgroup.  Three workgroups fit on a compute unit, 768 on the chip: the split is
  // the multiple of 64 rows (one load round of a workgroup) that fills one such resident round,
  // so that all workgroups start together and none is left for a thin second round.
  constexpr long long ROUND_WGS = 752;                       // a little under the 768 resident at once
  const long long room = ROUND_WGS - nseg;                   // the segments' last, partial splits
  long long want = room > 64 ? (cap + room - 1) / room : cap / 512;
  if (want < 64) want = 64;
  const int split = (int)((want + 63) / 64 * 64);
  pl.split = split;
  pl.nblk = (int)(cap / split + nseg);          // >= sum over segments of ceil(len / split)
  pl.part_acc = 0;
  pl.part_ml = align_up((size_t)pl.nblk * dm.g * dm.d * sizeof(float), 256);
  pl.seg_tab = pl.part_ml + align_up((size_t)pl.nblk * dm.g * 2 * sizeof(float), 256);
  pl.total = pl.seg_tab + align_up((size_t)nseg * sizeof(int4), 256);
  return pl;
}

hipError_t launch_decode_attn(const SeqTab &st, const Dims &dm, int dtype, int headroom,
                              const void *q, const void *k_new, const void *v_new, const int *cu,
                              void *Kc, void *Vc, int *seg_len, int *overflow, float *out,
                              float *lse, char *ws, hipStream_t s) {
  const DecodePlan pl = plan_decode(st, dm, headroom);
  const DecodeArgs a = {q, k_new, v_new, cu, Kc, Vc, seg_len, overflow, out, lse, ws};
  bool ok;
  if (dtype == ADAKV_BF16) {
    ok = dm.d == 64 ? run_decode_g<unsigned short, 64>(st, dm, headroom, pl, a, s)
                    : run_decode_g<unsigned short, 128>(st, dm, headroom, pl, a, s);
  } else if (dtype == ADAKV_FP16) {
    ok = dm.d == 64 ? run_decode_g<f16_t, 64>(st, dm, headroom, pl, a, s)
                    : run_decode_g<f16_t, 128>(st, dm, headroom, pl, a, s);
  } else {
    ok = dm.d == 64 ? run_decode_g<float, 64>(st, dm, headroom, pl, a, s)
                    : run_decode_g<float, 128>(st, dm, headroom, pl, a, s);
  }
  if (!ok) return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_append(const SeqTab &st, const Dims &dm, int dtype, int headroom,
                         const void *k_new, const void *v_new, const int *cu, void *Kc, void *Vc,
                         int *seg_len, int *overflow, hipStream_t s) {
  const int lpr = dm.d * (dtype == ADAKV_FP32 ? 4 : 2) / 16;
  const int nseg = st.batch * dm.h_kv;
  dim3 grid((nseg * lpr + 255) / 256), block(256);
#define ADAKV_LAUNCH_APPEND(LPR)                                                               \
  ADAKV_LAUNCH("append", append_kernel<LPR>, grid, block, s, nseg, headroom,                   \
               (const char *)k_new, (const char *)v_new, cu, (char *)Kc, (char *)Vc, seg_len,  \
               overflow)
  switch (lpr) {
    case 8: ADAKV_LAUNCH_APPEND(8); break;
    case 16: ADAKV_LAUNCH_APPEND(16); break;
    case 32: ADAKV_LAUNCH_APPEND(32); break;
    default: return hipErrorInvalidValue;
  }
#undef ADAKV_LAUNCH_APPEND
  return hipGetLastError();
}

}  // namespace adakv
