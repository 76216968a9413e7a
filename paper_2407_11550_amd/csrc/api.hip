// C ABI entry points: argument checks, workspace planning, kernel launches.
// Each call only enqueues work on the caller's stream.
#include <math.h>
#include <stdio.h>

#include <mutex>

#include "common.h"

namespace adakv {

static int build_tables(const adakv_layer *L, SeqTab &st, Dims &dm) {
  if (!L || !L->n || !L->B) return ADAKV_EINVAL;
  if (L->h_q < 1 || L->h_kv < 1 || L->h_q % L->h_kv != 0) return ADAKV_EINVAL;
  if (L->w < 1 || L->pool_k < 1 || L->pool_k % 2 == 0) return ADAKV_EINVAL;
  if (!(L->alpha >= 0.0f && L->alpha <= 1.0f)) return ADAKV_EINVAL;
  if (!(L->scale >= 0.0f) || isinf(L->scale)) return ADAKV_EINVAL;
  if (L->batch < 1 || L->batch > ADAKV_MAX_BATCH) return ADAKV_EINVAL;
  if (L->batch > 1 && !L->tok_off) return ADAKV_EINVAL;
  if (L->d < 1) return ADAKV_EINVAL;
  long long sc = 0, out = 0;
  st.batch = L->batch;
  for (int b = 0; b < L->batch; ++b) {
    long long n = L->n[b], B = L->B[b];
    long long wh = (long long)L->w * L->h_kv;
    if (n < 1 || B < wh || B - wh > (long long)L->h_kv * n) return ADAKV_EINVAL;
    long long t0 = L->tok_off ? L->tok_off[b] : 0;
    if (t0 < 0) return ADAKV_EINVAL;
    if (L->tok_off && L->tok_off[b + 1] - t0 < n + L->w) return ADAKV_EINVAL;
    st.n[b] = (int)n;
    st.Bp[b] = (int)(B - wh);
    st.tok_off[b] = t0;
    st.score_off[b] = (int)sc;
    st.out_off[b] = (int)out;
    sc += (long long)L->h_kv * n;
    out += B;
    if (sc >= (1ll << 31) || out >= (1ll << 31)) return ADAKV_EUNSUPPORTED;
  }
  for (int b = L->batch; b < ADAKV_MAX_BATCH; ++b) {
    st.n[b] = 0; st.Bp[b] = 0; st.tok_off[b] = 0;
  }
  for (int b = L->batch; b <= ADAKV_MAX_BATCH; ++b) {
    st.score_off[b] = (int)sc;
    st.out_off[b] = (int)out;
  }
  if (L->dtype != ADAKV_BF16 && L->dtype != ADAKV_FP32 && L->dtype != ADAKV_FP16) return ADAKV_EUNSUPPORTED;
  if (L->d != 64 && L->d != 128) return ADAKV_EUNSUPPORTED;
  if (L->h_kv > 64 || (long long)L->h_q * L->w > (1 << 20)) return ADAKV_EUNSUPPORTED;
  const long long esz = L->dtype == ADAKV_FP32 ? 4 : 2;
  const long long strides[4] = {L->k_stride_tok, L->k_stride_head, L->v_stride_tok,
                                L->v_stride_head};
  for (long long sd : strides) {
    if (sd < L->d) return ADAKV_EINVAL;
    if ((sd * esz) % 16 != 0) return ADAKV_EUNSUPPORTED;   // rows are moved as 16-byte words
  }
  dm.h_q = L->h_q; dm.h_kv = L->h_kv; dm.g = L->h_q / L->h_kv; dm.d = L->d; dm.w = L->w;
  dm.pool_k = L->pool_k;
  dm.scale = L->scale > 0.0f ? L->scale : 1.0f / sqrtf((float)L->d);
  dm.alpha_fix = (int)floor((double)L->alpha * 65536.0 + 0.5);
  dm.k_stride_tok = L->k_stride_tok; dm.k_stride_head = L->k_stride_head;
  dm.v_stride_tok = L->v_stride_tok; dm.v_stride_head = L->v_stride_head;
  return ADAKV_OK;
}

// Workspace: the scoring part first, the Top-k part behind it (they must not overlap: in
// pipeline mode the scoring call already writes into the Top-k part).
static bool pool_first(const adakv_layer *L) { return (L->flags & ADAKV_FLAG_POOL_THEN_MEAN) != 0; }
// Which kernel family scores the layer: the matrix cores (16-bit inputs, at most 512 window rows
// per KV head; with ADAKV_FLAG_POOL_THEN_MEAN a pool radius of at most 7), else the plain-FMA path.
static bool on_mfma(const Dims &dm, const adakv_layer *L) {
  return pool_first(L) ? mfma_pool_rows_supported(dm, L->dtype) : mfma_path_supported(dm, L->dtype);
}
static size_t topk_offset(const SeqTab &st, const Dims &dm, const adakv_layer *L) {
  return align_up(plan_score(st, dm, L->dtype, on_mfma(dm, L)).total, 256);
}
static size_t workspace_for(const SeqTab &st, const Dims &dm, const adakv_layer *L) {
  return topk_offset(st, dm, L) + plan_topk_bytes(st, dm) + 256;
}
static bool pipeline_mode(const adakv_layer *L, const Dims &dm) {
  return (L->flags & ADAKV_FLAG_PIPELINE) != 0 && carry_supported(dm, L->dtype) && on_mfma(dm, L);
}

static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

static thread_local struct {
  void *const *events = nullptr;
  int capacity = 0, used = 0;
  const char *names[ADAKV_TRACE_MAX];
} g_trace;

bool trace_pair(const char *name, hipEvent_t *start, hipEvent_t *stop) {
  if (!g_trace.events || g_trace.used + 2 > g_trace.capacity) return false;
  g_trace.names[g_trace.used] = name;
  g_trace.names[g_trace.used + 1] = name;
  *start = (hipEvent_t)g_trace.events[g_trace.used];
  *stop = (hipEvent_t)g_trace.events[g_trace.used + 1];
  g_trace.used += 2;
  return true;
}

}  // namespace adakv

// Scratch for adakv_compress_static.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address differs per GPU and is looked up once per device.
static __device__ __align__(256) unsigned char scratch[ADAKV_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (nullptr if HIP refuses).
void *static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

using namespace adakv;

extern "C" {

size_t adakv_workspace_bytes(const adakv_layer *L) {
  SeqTab st; Dims dm;
  if (build_tables(L, st, dm) != ADAKV_OK) return 0;
  return workspace_for(st, dm, L);
}

int adakv_pyramid_budgets(int32_t n_layers, int64_t avg_budget, double ratio, int64_t *out) {
  if (n_layers < 1 || avg_budget < 0 || !(ratio >= 1.0) || isinf(ratio) || !out) return ADAKV_EINVAL;
  if (avg_budget > (1ll << 40) || n_layers > (1 << 24) || ratio > 1048576.0) return ADAKV_EUNSUPPORTED;
  if (n_layers == 1) { out[0] = avg_budget; return ADAKV_OK; }
  // Exact integer arithmetic (a product of doubles can land one unit in the last place off an
  // integer and the floor below would then be wrong by one).  A finite double is p / q with q a
  // power of two, so with L = n_layers
  //   real_l = b_max - (b_max - b_min) l / (L-1),  b_min = 2 avg / (1 + r),  b_max = r b_min
  //          = 2 avg (p (L-1) - (p - q) l) / ((p + q) (L-1)).
  // p < 2^53, q <= 2^52, avg <= 2^40, L <= 2^24: the numerator stays below 2^119.
  int e = 0;
  const double mant = frexp(ratio, &e);                        // ratio = mant * 2^e, 0.5 <= mant < 1
  unsigned __int128 p = (unsigned __int128)(uint64_t)ldexp(mant, 53), q = 1;   // ratio = p * 2^(e-53)
  if (e >= 53) p <<= (e - 53); else q <<= (53 - e);
  while (!(p & 1) && !(q & 1)) { p >>= 1; q >>= 1; }
  const unsigned __int128 Lm1 = (unsigned __int128)(n_layers - 1);
  const unsigned __int128 den = (p + q) * Lm1;
  int64_t given = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    const unsigned __int128 num = (unsigned __int128)(2 * avg_budget) * (p * Lm1 - (p - q) * (unsigned __int128)l);
    out[l] = (int64_t)(num / den);                             // floor: everything is non-negative
    given += out[l];
  }
  // the real values sum to exactly L * avg, and every floor lost less than one unit
  int64_t left = (int64_t)n_layers * avg_budget - given;
  for (int32_t l = 0; l < n_layers && left > 0; ++l, --left) out[l] += 1;
  return left == 0 ? ADAKV_OK : ADAKV_EINVAL;
}

int adakv_trace_arm(void *const *events, int n_events) {
  if (!events || n_events < 2 || n_events > ADAKV_TRACE_MAX) return ADAKV_EINVAL;
  g_trace.events = events;
  g_trace.capacity = n_events;
  g_trace.used = 0;
  return ADAKV_OK;
}

int adakv_trace_disarm(void) {
  const int used = g_trace.used;
  g_trace.events = nullptr;
  g_trace.capacity = 0;
  return used;
}

const char *adakv_trace_name(int i) {
  return (i >= 0 && i < g_trace.used) ? g_trace.names[i] : "";
}

const char *adakv_strerror(int status) {
  switch (status) {
    case ADAKV_OK: return "ok";
    case ADAKV_EINVAL: return "invalid argument (NULL pointer or parameter outside its domain)";
    case ADAKV_EUNSUPPORTED: return "shape, dtype or alignment not supported by this build";
    case ADAKV_EWORKSPACE: return "workspace missing or smaller than adakv_workspace_bytes";
    case ADAKV_EHIP: return "a HIP runtime call failed";
    case ADAKV_ESCRATCH: return "the layer needs more scratch memory than the built-in array of adakv_compress_static holds";
    default: return "unknown status";
  }
}

int adakv_score(const adakv_layer *L, const void *q_window, const void *K, const float *row_lse,
                float *scores, void *ws, size_t ws_bytes, void *hip_stream) {
  SeqTab st; Dims dm;
  int rc = build_tables(L, st, dm);
  if (rc != ADAKV_OK) return rc;
  if (!q_window || !K || !scores) return ADAKV_EINVAL;
  if (!aligned16(q_window) || !aligned16(K) || !aligned16(scores)) return ADAKV_EUNSUPPORTED;
  if (!ws || ws_bytes < workspace_for(st, dm, L)) return ADAKV_EWORKSPACE;
  char *wsp = (char *)(((uintptr_t)ws + 255) & ~(uintptr_t)255);
  ScorePlan pl = plan_score(st, dm, L->dtype, on_mfma(dm, L));
  hipStream_t s = (hipStream_t)hip_stream;
  if (pool_first(L) && dm.pool_k / 2 > 100) return ADAKV_EUNSUPPORTED;
  TopkCarry tc = {nullptr, 0u, nullptr, nullptr};
  if (pipeline_mode(L, dm)) tc = plan_carry(st, dm, wsp + topk_offset(st, dm, L));
  hipError_t e = on_mfma(dm, L)
                     ? launch_score_mfma(st, dm, L->dtype, q_window, K, row_lse, scores, wsp, pl, tc,
                                         pool_first(L), s)
                     : launch_score_generic(st, dm, L->dtype, q_window, K, row_lse, scores, wsp,
                                            pl, pool_first(L), s);
  return e == hipSuccess ? ADAKV_OK : ADAKV_EHIP;
}

int adakv_allocate(const adakv_layer *L, const float *scores, int32_t *budgets,
                   int32_t *cu_seqlens, void *ws, size_t ws_bytes, void *hip_stream) {
  SeqTab st; Dims dm;
  int rc = build_tables(L, st, dm);
  if (rc != ADAKV_OK) return rc;
  if (!scores || !budgets || !cu_seqlens) return ADAKV_EINVAL;
  if (!aligned16(scores)) return ADAKV_EUNSUPPORTED;
  if (!ws || ws_bytes < workspace_for(st, dm, L)) return ADAKV_EWORKSPACE;
  char *wsp = (char *)(((uintptr_t)ws + 255) & ~(uintptr_t)255);
  hipError_t e = launch_allocate(st, dm, scores, budgets, cu_seqlens,
                                 wsp + topk_offset(st, dm, L), pipeline_mode(L, dm),
                                 (hipStream_t)hip_stream);
  return e == hipSuccess ? ADAKV_OK : ADAKV_EHIP;
}

int adakv_select(const adakv_layer *L, const float *scores, const int32_t *budgets,
                 const int32_t *cu_seqlens, int32_t *indices, void *ws, size_t ws_bytes,
                 void *hip_stream) {
  SeqTab st; Dims dm;
  int rc = build_tables(L, st, dm);
  if (rc != ADAKV_OK) return rc;
  if (!scores || !budgets || !cu_seqlens || !indices) return ADAKV_EINVAL;
  if (!aligned16(scores)) return ADAKV_EUNSUPPORTED;
  if (!ws || ws_bytes < workspace_for(st, dm, L)) return ADAKV_EWORKSPACE;
  char *wsp = (char *)(((uintptr_t)ws + 255) & ~(uintptr_t)255);
  hipError_t e = launch_select(st, dm, scores, budgets, cu_seqlens, indices,
                               wsp + topk_offset(st, dm, L), pipeline_mode(L, dm),
                               (hipStream_t)hip_stream);
  return e == hipSuccess ? ADAKV_OK : ADAKV_EHIP;
}

int adakv_compact(const adakv_layer *L, const void *K, const void *V, const int32_t *indices,
                  const int32_t *cu_seqlens, void *K_out, void *V_out, void *hip_stream) {
  SeqTab st; Dims dm;
  int rc = build_tables(L, st, dm);
  if (rc != ADAKV_OK) return rc;
  if (!K || !V || !indices || !cu_seqlens || !K_out || !V_out) return ADAKV_EINVAL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(K_out) || !aligned16(V_out))
    return ADAKV_EUNSUPPORTED;
  hipError_t e = launch_compact(st, dm, L->dtype, K, V, indices, cu_seqlens, K_out, V_out, 0,
                                nullptr, (hipStream_t)hip_stream);
  return e == hipSuccess ? ADAKV_OK : ADAKV_EHIP;
}

int adakv_compress(const adakv_layer *L, const void *q_window, const void *K, const void *V,
                   const float *row_lse, float *scores, int32_t *budgets, int32_t *cu_seqlens,
                   int32_t *indices, void *K_out, void *V_out, void *ws, size_t ws_bytes,
                   void *hip_stream) {
  // every argument is checked before the first kernel is enqueued
  SeqTab st; Dims dm;
  int rc = build_tables(L, st, dm);
  if (rc != ADAKV_OK) return rc;
  if (!q_window || !K || !V || !scores || !budgets || !cu_seqlens || !indices || !K_out || !V_out)
    return ADAKV_EINVAL;
  if (!aligned16(q_window) || !aligned16(K) || !aligned16(V) || !aligned16(scores) ||
      !aligned16(K_out) || !aligned16(V_out))
    return ADAKV_EUNSUPPORTED;
  if (pool_first(L) && dm.pool_k / 2 > 100) return ADAKV_EUNSUPPORTED;
  if (!ws || ws_bytes < workspace_for(st, dm, L)) return ADAKV_EWORKSPACE;
  adakv_layer P = *L;
  P.flags |= ADAKV_FLAG_PIPELINE;
  if ((rc = adakv_score(&P, q_window, K, row_lse, scores, ws, ws_bytes, hip_stream)) != ADAKV_OK) return rc;
  if ((rc = adakv_allocate(&P, scores, budgets, cu_seqlens, ws, ws_bytes, hip_stream)) != ADAKV_OK) return rc;
  if ((rc = adakv_select(&P, scores, budgets, cu_seqlens, indices, ws, ws_bytes, hip_stream)) != ADAKV_OK) return rc;
  return adakv_compact(&P, K, V, indices, cu_seqlens, K_out, V_out, hip_stream);
}

// ---- the whole step without a workspace argument ------------------------------------------------
int adakv_compress_static(const adakv_layer *L, const void *q_window, const void *K, const void *V,
                          const float *row_lse, float *scores, int32_t *budgets,
                          int32_t *cu_seqlens, int32_t *indices, void *K_out, void *V_out,
                          void *hip_stream) {
  SeqTab st; Dims dm;
  int rc = build_tables(L, st, dm);
  if (rc != ADAKV_OK) return rc;
  if (workspace_for(st, dm, L) > (size_t)ADAKV_STATIC_SCRATCH_BYTES) return ADAKV_ESCRATCH;
  void *ws = static_scratch();
  if (!ws) return ADAKV_EHIP;
  return adakv_compress(L, q_window, K, V, row_lse, scores, budgets, cu_seqlens, indices, K_out,
                        V_out, ws, ADAKV_STATIC_SCRATCH_BYTES, hip_stream);
}

// ---- decode side ------------------------------------------------------------------------------
static int check_headroom(const SeqTab &st, const Dims &dm, int32_t headroom) {
  if (headroom < 0) return ADAKV_EINVAL;
  const long long rows = (long long)st.out_off[st.batch] + (long long)st.batch * dm.h_kv * headroom;
  return rows < (1ll << 31) ? ADAKV_OK : ADAKV_EUNSUPPORTED;
}

int adakv_cache_build(const adakv_layer *L, const void *K, const void *V, const int32_t *indices,
                      const int32_t *cu_seqlens, int32_t headroom, void *K_cache, void *V_cache,
                      int32_t *seg_len, void *hip_stream) {
  SeqTab st; Dims dm;
  int rc = build_tables(L, st, dm);
  if (rc != ADAKV_OK) return rc;
  if ((rc = check_headroom(st, dm, headroom)) != ADAKV_OK) return rc;
  if (!K || !V || !indices || !cu_seqlens || !K_cache || !V_cache || !seg_len) return ADAKV_EINVAL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(K_cache) || !aligned16(V_cache))
    return ADAKV_EUNSUPPORTED;
  hipError_t e = launch_compact(st, dm, L->dtype, K, V, indices, cu_seqlens, K_cache, V_cache,
                                headroom, seg_len, (hipStream_t)hip_stream);
  return e == hipSuccess ? ADAKV_OK : ADAKV_EHIP;
}

int adakv_append(const adakv_layer *L, const void *k_new, const void *v_new,
                 const int32_t *cu_seqlens, int32_t headroom, void *K_cache, void *V_cache,
                 int32_t *seg_len, int32_t *overflow, void *hip_stream) {
  SeqTab st; Dims dm;
  int rc = build_tables(L, st, dm);
  if (rc != ADAKV_OK) return rc;
  if ((rc = check_headroom(st, dm, headroom)) != ADAKV_OK) return rc;
  if (!k_new || !v_new || !cu_seqlens || !K_cache || !V_cache || !seg_len) return ADAKV_EINVAL;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(K_cache) || !aligned16(V_cache))
    return ADAKV_EUNSUPPORTED;
  hipError_t e = launch_append(st, dm, L->dtype, headroom, k_new, v_new, cu_seqlens, K_cache,
                               V_cache, seg_len, overflow, (hipStream_t)hip_stream);
  return e == hipSuccess ? ADAKV_OK : ADAKV_EHIP;
}

size_t adakv_decode_workspace_bytes(const adakv_layer *L, int32_t headroom) {
  SeqTab st; Dims dm;
  if (build_tables(L, st, dm) != ADAKV_OK || check_headroom(st, dm, headroom) != ADAKV_OK) return 0;
  if (!decode_supported(dm)) return 0;
  return plan_decode(st, dm, headroom).total + 256;
}

int adakv_decode_attn(const adakv_layer *L, const void *q_new, const int32_t *cu_seqlens,
                      int32_t headroom, const void *K_cache, const void *V_cache,
                      const int32_t *seg_len, float *out, float *lse, void *ws, size_t ws_bytes,
                      void *hip_stream) {
  SeqTab st; Dims dm;
  int rc = build_tables(L, st, dm);
  if (rc != ADAKV_OK) return rc;
  if ((rc = check_headroom(st, dm, headroom)) != ADAKV_OK) return rc;
  if (!q_new || !cu_seqlens || !K_cache || !V_cache || !seg_len || !out) return ADAKV_EINVAL;
  if (!decode_supported(dm)) return ADAKV_EUNSUPPORTED;
  if (!aligned16(q_new) || !aligned16(K_cache) || !aligned16(V_cache)) return ADAKV_EUNSUPPORTED;
  if (!ws || ws_bytes < plan_decode(st, dm, headroom).total + 256) return ADAKV_EWORKSPACE;
  char *wsp = (char *)(((uintptr_t)ws + 255) & ~(uintptr_t)255);
  hipError_t e = launch_decode_attn(st, dm, L->dtype, headroom, q_new, nullptr, nullptr,
                                    cu_seqlens, (void *)K_cache, (void *)V_cache,
                                    (int *)seg_len, nullptr, out, lse, wsp,
                                    (hipStream_t)hip_stream);
  return e == hipSuccess ? ADAKV_OK : ADAKV_EHIP;
}

int adakv_decode_step(const adakv_layer *L, const void *q_new, const void *k_new,
                      const void *v_new, const int32_t *cu_seqlens, int32_t headroom,
                      void *K_cache, void *V_cache, int32_t *seg_len, int32_t *overflow,
                      float *out, float *lse, void *ws, size_t ws_bytes, void *hip_stream) {
  SeqTab st; Dims dm;
  int rc = build_tables(L, st, dm);
  if (rc != ADAKV_OK) return rc;
  if ((rc = check_headroom(st, dm, headroom)) != ADAKV_OK) return rc;
  if (!q_new || !k_new || !v_new || !cu_seqlens || !K_cache || !V_cache || !seg_len || !out)
    return ADAKV_EINVAL;
  if (!decode_supported(dm)) return ADAKV_EUNSUPPORTED;
  if (!aligned16(q_new) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(K_cache) ||
      !aligned16(V_cache))
    return ADAKV_EUNSUPPORTED;
  if (!ws || ws_bytes < plan_decode(st, dm, headroom).total + 256) return ADAKV_EWORKSPACE;
  char *wsp = (char *)(((uintptr_t)ws + 255) & ~(uintptr_t)255);
  hipError_t e = launch_decode_attn(st, dm, L->dtype, headroom, q_new, k_new, v_new, cu_seqlens,
                                    K_cache, V_cache, seg_len, overflow, out, lse, wsp,
                                    (hipStream_t)hip_stream);
  return e == hipSuccess ? ADAKV_OK : ADAKV_EHIP;
}

int adakv_describe(const adakv_layer *L, int have_row_lse, char *out, size_t out_bytes) {
  SeqTab st; Dims dm;
  int rc = build_tables(L, st, dm);
  if (rc != ADAKV_OK) return rc;
  if (!out || out_bytes == 0) return ADAKV_EINVAL;
  if (pool_first(L) && dm.pool_k / 2 > 100) return ADAKV_EUNSUPPORTED;
  const char *dt = L->dtype == ADAKV_FP32 ? "fp32" : L->dtype == ADAKV_FP16 ? "fp16" : "bf16";
  const char *topk = pipeline_mode(L, dm) ? "carried" : "separate";
  const char *stats = have_row_lse ? "caller" : "sweep";
  int len;
  if (on_mfma(dm, L)) {
    const MfmaVariant v = choose_mfma_variant(st, dm);
    len = snprintf(out, out_bytes,
                   "score=%s dtype=%s d=%d rows=%d mb=%d rs=%d kg=%d chunk=%d stats=%s lse=%s pool=%s topk=%s",
                   pool_first(L) ? "mfma-pool-first" : "mfma", dt, dm.d, dm.g * dm.w, v.mb, v.rs, v.kg,
                   v.chunk, stats, have_row_lse ? "caller" : v.fuse_lse ? "fused" : "kernel",
                   pool_first(L) ? "rows" : v.fuse_pool ? "fused" : "kernel", topk);
  } else {
    len = snprintf(out, out_bytes, "score=%s dtype=%s d=%d rows=%d stats=%s lse=%s pool=kernel topk=%s",
                   pool_first(L) ? "fma-pool-first" : "fma", dt, dm.d, dm.g * dm.w, stats,
                   have_row_lse ? "caller" : "kernel", topk);
  }
  return (len < 0 || (size_t)len >= out_bytes) ? ADAKV_EINVAL : ADAKV_OK;
}

int adakv_probe_read(const void *src, size_t bytes, void *sink, void *hip_stream) {
  if ((!src && bytes > 0) || !sink || bytes % 16 != 0) return ADAKV_EINVAL;
  if (!aligned16(src) || !aligned16(sink)) return ADAKV_EUNSUPPORTED;
  static_assert(ADAKV_PROBE_SINK_BYTES == ADAKV_PROBE_BLOCKS * 4 * 16, "one word per wave");
  if (probe_waves_per_block() != 4) return ADAKV_EHIP;
  hipError_t e = launch_probe_read(src, (long long)(bytes / 16), sink, ADAKV_PROBE_BLOCKS,
                                   (hipStream_t)hip_stream);
  return e == hipSuccess ? ADAKV_OK : ADAKV_EHIP;
}

}  // extern "C"
