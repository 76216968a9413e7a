/*
 * adakv.h -- C ABI of the MI355X (gfx950) Ada-KV per-layer cache compression library.
 *
 * The library runs the compression step the paper performs on every attention layer at the
 * end of prefill (Section 4.1, "Parameters"): Algorithm 2 ("Ada-SnapKV/Ada-Pyramid in One
 * Layer") with Algorithm 1 ("Adaptive Budget Allocation") inside it, as four calls:
 *
 *     adakv_score     Alg. 2 lines 1-5   observation-window attention scores of every prefix key
 *     adakv_allocate  Alg. 2 lines 6-8   layer-wide Top-B' -> per-head budgets (Alg. 1) + safeguard
 *     adakv_select    Alg. 2 line 9      per-head Top-B_i eviction decision, as index lists
 *     adakv_compact   Alg. 2 lines 10-11 gather of the retained K/V rows into the flattened
 *                                        variable-length per-head cache (Section 3.5)
 *
 * Notation (paper's where it has one):
 *     n      cache elements OUTSIDE the observation window = eviction candidates of a sequence
 *     w      observation window size; a sequence owns N = n + w rows of q/K/V, window last
 *     h_kv   KV heads; h_q query heads, g = h_q / h_kv of them share a KV head.  Scores,
 *            budgets and outputs are per KV head (Section 3.5: group-mean criterion)
 *     B      layer budget of a sequence INCLUDING its w window rows per head (Alg. 2 l.6)
 *     B'     B - w*h_kv, the part Algorithm 1 distributes
 *     alpha  safeguard hyper-parameter: share of B' handed out uniformly.  alpha = 1 is the
 *            uniform allocation B'/h of Section 3.2, alpha = 0 is Algorithm 1 unmodified
 *     k      max-pool kernel (Section 4.1: 7)
 *
 * General rules
 *   - Every pointer marked (device) is device memory on the current HIP device; (host) is
 *     ordinary host memory that is read during the call and may be reused on return.
 *   - The caller owns every buffer.  The library allocates nothing, frees nothing and keeps
 *     no state between calls; scratch memory comes in through `ws` (size from
 *     adakv_workspace_bytes; its contents need not survive from one call to the next unless
 *     the caller asks for that with ADAKV_FLAG_PIPELINE).  Two stated exceptions, neither on
 *     the path of the method's calls: adakv_compress_static uses a built-in device array as its
 *     scratch and remembers that array's address per GPU, and the measurement aid
 *     adakv_trace_arm keeps the armed event list per calling host thread until
 *     adakv_trace_disarm.
 *   - Every call only enqueues kernels on `hip_stream` (a hipStream_t, NULL = default stream)
 *     and returns; nothing synchronises with the host.  The number of output rows, sum_b B_b,
 *     is known before the call, so outputs are pre-sized by the caller.
 *   - Return value: ADAKV_OK or a negative adakv_status.  On ADAKV_EINVAL, ADAKV_EUNSUPPORTED
 *     and ADAKV_EWORKSPACE nothing was launched and outputs are untouched.
 *   - Calls that share a workspace or an output buffer must be ordered on one stream.
 */
#ifndef ADAKV_H
#define ADAKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { ADAKV_BF16 = 0, ADAKV_FP32 = 1, ADAKV_FP16 = 2 } adakv_dtype;

typedef enum {
  ADAKV_OK = 0,
  ADAKV_EINVAL = -1,       /* NULL required pointer, or a parameter outside its domain      */
  ADAKV_EUNSUPPORTED = -2, /* valid problem, but a shape/dtype this build has no kernel for  */
  ADAKV_EWORKSPACE = -3,   /* ws == NULL or ws_bytes < adakv_workspace_bytes(L)              */
  ADAKV_EHIP = -4,         /* a HIP runtime call failed (kernel launch)                      */
  ADAKV_ESCRATCH = -5      /* adakv_compress_static: the layer needs more scratch memory than
                              the library's built-in array holds (ADAKV_STATIC_SCRATCH_BYTES)  */
} adakv_status;

#define ADAKV_MAX_BATCH 64          /* sequences per call                                    */
#define ADAKV_FLAG_ROW_LSE 1u       /* bit 0 of flags: informational, set by callers that
                                       pass row_lse to adakv_score                           */
#define ADAKV_FLAG_PIPELINE 2u      /* bit 1 of flags: a promise by the caller that adakv_score,
                                       adakv_allocate and adakv_select are issued in this order
                                       on one stream, for this layer, with the same ws and the
                                       same scores buffer, and that nothing else touches ws in
                                       between.  The library may then carry intermediate results
                                       in ws from one call to the next (the scoring call clears
                                       the Top-k histograms and counts the first radix digit of
                                       every score while it still holds it), which removes four
                                       kernel launches.  Results are identical with and without
                                       the flag; breaking the promise gives undefined budgets and
                                       indices (no out-of-bounds access).                      */

#define ADAKV_FLAG_POOL_THEN_MEAN 4u /* bit 2 of flags: adakv_score max-pools every window row along
                                       the keys first and averages the g*w rows afterwards (Alg. 2
                                       l.4 as printed) instead of averaging first (Section 3.4's
                                       prose, the default).  On the matrix cores for pool_k/2 <= 7
                                       (the pool is a sliding maximum across lanes, tiles overlap by
                                       the radius), on the plain-FMA kernels up to pool_k/2 <= 100. */

/*
 * One attention layer's compression problem, for `batch` independent sequences (Algorithm 1
 * acts "within a single layer" of one sequence, so budgets never move between sequences).
 *
 * Domain (else ADAKV_EINVAL): h_q % h_kv == 0; w >= 1; pool_k odd >= 1; 0 <= alpha <= 1;
 * 1 <= batch <= ADAKV_MAX_BATCH; n[b] >= 1; w*h_kv <= B[b] <= w*h_kv + h_kv*n[b];
 * tok_off non-decreasing with tok_off[b+1] - tok_off[b] >= n[b] + w.
 * Supported (else ADAKV_EUNSUPPORTED): d in {64, 128}; dtype bf16, fp16 or fp32; sum_b h_kv*n[b]
 * and sum_b B[b] below 2^31.
 */
typedef struct {
  int32_t dtype;            /* adakv_dtype of q_window, K, V, K_out, V_out (and the caches)  */
  int32_t h_q, h_kv, d;     /* query head hq belongs to KV head hq / (h_q / h_kv)           */
  int32_t w, pool_k;
  float alpha;
  float scale;              /* logit scale; 0 means 1/sqrt(d)                               */
  int32_t batch;
  const int32_t *n;         /* (host) [batch]  prefix length per sequence                   */
  const int32_t *B;         /* (host) [batch]  layer budget per sequence, window included   */
  const int64_t *tok_off;   /* (host) [batch+1] first K/V row of each sequence; NULL means
                               batch == 1 at row 0                                          */
  int64_t k_stride_tok, k_stride_head; /* K element strides; the d axis is contiguous       */
  int64_t v_stride_tok, v_stride_head; /* same for V                                        */
  uint32_t flags;
} adakv_layer;

/* Scratch bytes that any of the four calls may need for this problem (0 on invalid L). */
size_t adakv_workspace_bytes(const adakv_layer *L);

/* Static, never NULL. */
const char *adakv_strerror(int status);

/*
 * Alg. 2 lines 1-5 and Section 3.5.  For every sequence b, KV head c and prefix position j:
 *
 *   scores[off_b + c*n_b + j] = max over |j' - j| <= k/2, 0 <= j' < n_b of
 *        (1/(g*w)) * sum over the g query heads hq of c and the w window rows r of
 *        exp(scale * q_window[b][hq][r] . K[tok_off[b] + j'][c]  -  lse[b][hq][r])
 *
 * with off_b = h_kv * sum_{b'<b} n_b'.  lse[b][hq][r] is row_lse if given; otherwise it is
 * the natural log of the sum over the n_b prefix keys of exp(scaled logit), i.e. the softmax
 * of Alg. 2 l.3 runs over the cache outside the window.  A caller that passes the prefill
 * attention's own log-sum-exp gets the normalisation over every visible key instead.
 * Logits are accumulated in fp32, softmax and reductions are fp32, the mean is taken before
 * the pool (unless ADAKV_FLAG_POOL_THEN_MEAN asks for the other order: the max over j' then
 * moves inside the sum over rows), and the pool is stride 1, same length, clipped at both ends.
 *
 *   q_window (device) [batch][h_q][w][d], contiguous, L->dtype
 *   K        (device) rows tok_off[b] .. tok_off[b]+n_b-1 are read, element (row, c, e) at
 *                     row*k_stride_tok + c*k_stride_head + e; rows must be 16-byte aligned
 *   row_lse  (device) [batch][h_q][w] fp32, or NULL
 *   scores   (device) [sum_b h_kv*n_b] fp32, written
 */
int adakv_score(const adakv_layer *L, const void *q_window, const void *K, const float *row_lse,
                float *scores, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Alg. 2 lines 6-8 with Algorithm 1.  Per sequence: B' = B - w*h_kv; the B' largest of the
 * h_kv*n scores are found (ties: lower flat index c*n + j first) and counted per head, f_c;
 * the safeguard mixes in the uniform share, x_c = (1-alpha) f_c + alpha B'/h_kv, in exact
 * integer arithmetic with alpha rounded to 16 fractional bits:
 *     num_c = (65536-a) h_kv f_c + a B',  den = 65536 h_kv,  budgets[c] = floor(num_c/den),
 * and the B' - sum floor units left go to the heads with the largest num_c % den (ties: lower
 * c), so sum_c budgets[c] = B' exactly.  Scores must be >= 0 and not NaN.
 *
 *   scores     (device) as written by adakv_score
 *   budgets    (device) [batch*h_kv] int32, written: prefix rows kept per (b, c)
 *   cu_seqlens (device) [batch*h_kv+1] int32, written: cu[0] = 0,
 *                       cu[s+1] = cu[s] + budgets[s] + w, segment s = b*h_kv + c
 */
int adakv_allocate(const adakv_layer *L, const float *scores, int32_t *budgets,
                   int32_t *cu_seqlens, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Alg. 2 line 9 (the Top-k eviction decision of Section 3.2) as index lists.  Segment
 * s = (b, c) of `indices` starts at cu_seqlens[s] and holds the budgets[s] prefix positions
 * of head c with the largest scores (ties: lower position first) in ascending order, followed
 * by the window positions n_b .. n_b+w-1.  Positions count from the sequence's first row.
 *
 *   scores, budgets, cu_seqlens (device) as above; budgets[s] <= n_b and cu_seqlens must be
 *                               the running sum of budgets + w (not checked)
 *   indices (device) [sum_b B_b] int32, written
 */
int adakv_select(const adakv_layer *L, const float *scores, const int32_t *budgets,
                 const int32_t *cu_seqlens, int32_t *indices, void *ws, size_t ws_bytes,
                 void *hip_stream);

/*
 * Alg. 2 lines 10-11 into the flattened layout of Section 3.5: for segment s = (b, c) and
 * cu_seqlens[s] <= t < cu_seqlens[s+1],
 *     K_out[t][:] = K[tok_off[b] + indices[t]][c][:],   V_out likewise.
 * Pure byte copy.
 *
 *   K, V           (device) strided as in the layer; rows 16-byte aligned
 *   indices        (device) [sum_b B_b] int32, each in [0, n_b + w)  (values outside are clamped)
 *   cu_seqlens     (device) [batch*h_kv+1] int32 with cu[last] = sum_b B_b
 *   K_out, V_out   (device) [sum_b B_b][d] contiguous, L->dtype, written; 16-byte aligned
 */
int adakv_compact(const adakv_layer *L, const void *K, const void *V, const int32_t *indices,
                  const int32_t *cu_seqlens, void *K_out, void *V_out, void *hip_stream);

/*
 * The whole step of Algorithm 2 in one call: adakv_score, adakv_allocate, adakv_select and
 * adakv_compact back to back on `hip_stream`, in pipeline mode (the promise ADAKV_FLAG_PIPELINE
 * asks for is kept by construction, whatever L->flags says about it).  Arguments and outputs as
 * for the four calls; every output buffer is required.  Nothing is launched if any check fails.
 */
int adakv_compress(const adakv_layer *L, const void *q_window, const void *K, const void *V,
                   const float *row_lse, float *scores, int32_t *budgets, int32_t *cu_seqlens,
                   int32_t *indices, void *K_out, void *V_out, void *ws, size_t ws_bytes,
                   void *hip_stream);

/*
 * adakv_compress for callers that cannot allocate device memory and have no workspace to hand
 * over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments minus `ws`, same kernels, same results bit for bit; the scratch memory is a
 * built-in device array of ADAKV_STATIC_SCRATCH_BYTES that lives in the library's code object
 * (every GPU the library runs on holds its own copy until the process ends).  The call allocates
 * and frees nothing; the first call on a device looks the array's address up once.
 *
 *   - the HIP device current at the call must be the one `hip_stream` and all buffers belong to
 *   - a layer with adakv_workspace_bytes(L) > ADAKV_STATIC_SCRATCH_BYTES is rejected with
 *     ADAKV_ESCRATCH before anything is launched (every named workload of this build fits)
 *   - all calls on one GPU share the one array: it keeps the previous call's contents (the
 *     kernels clear what they need cleared), and two calls that overlap on one GPU (different
 *     streams or threads) race on it.  Order them on one stream.
 */
#define ADAKV_STATIC_SCRATCH_BYTES (24u << 20)
int adakv_compress_static(const adakv_layer *L, const void *q_window, const void *K, const void *V,
                          const float *row_lse, float *scores, int32_t *budgets,
                          int32_t *cu_seqlens, int32_t *indices, void *K_out, void *V_out,
                          void *hip_stream);

/*
 * ---- Decode side of the flattened layout (Section 3.5; Section 3.1, Eqs. 1-2) --------------
 *
 * After compression every (sequence, KV head) segment s = b*h_kv + c has its own length.  The
 * decode-side cache keeps the flattened layout and leaves `headroom` spare rows behind every
 * segment for the tokens generated afterwards:
 *
 *     start_s = cu_seqlens[s] + s*headroom      first row of segment s in K_cache / V_cache
 *     cap_s   = cu_seqlens[s+1] - cu_seqlens[s] + headroom
 *     seg_len[s]                                rows currently held, device resident
 *
 * cu_seqlens stays as adakv_allocate wrote it for the whole life of the cache; only seg_len
 * changes.  K_cache and V_cache are [sum_b B_b + batch*h_kv*headroom][d], contiguous, L->dtype,
 * 16-byte aligned.  0 <= headroom, and the row count must stay below 2^31.
 * Of L these calls use dtype, h_q, h_kv, d, w, batch, n, B, scale (B only to size the cache).
 */

/*
 * adakv_compact with the head-room layout: for segment s = (b, c) and 0 <= t < cu[s+1]-cu[s]
 *     K_cache[start_s + t][:] = K[tok_off[b] + indices[cu[s] + t]][c][:],   V_cache likewise,
 * and seg_len[s] = cu[s+1] - cu[s].  Spare rows are not written.
 *
 *   K, V, indices, cu_seqlens   as for adakv_compact
 *   seg_len (device) [batch*h_kv] int32, written
 */
int adakv_cache_build(const adakv_layer *L, const void *K, const void *V, const int32_t *indices,
                      const int32_t *cu_seqlens, int32_t headroom, void *K_cache, void *V_cache,
                      int32_t *seg_len, void *hip_stream);

/*
 * The cache update of Eq. (1), K_i = Cat[K_i : k_i] and V_i likewise, for every segment at
 * once: row k_new[b][c] is stored at start_s + seg_len[s] and seg_len[s] grows by one.  A
 * segment that is already full (seg_len[s] == cap_s) is left as it is and *overflow is set
 * to 1 (it is never cleared by the library).
 *
 *   k_new, v_new (device) [batch][h_kv][d] contiguous, L->dtype, 16-byte aligned
 *   seg_len      (device) [batch*h_kv] int32, read and written
 *   overflow     (device) one int32, or NULL
 */
int adakv_append(const adakv_layer *L, const void *k_new, const void *v_new,
                 const int32_t *cu_seqlens, int32_t headroom, void *K_cache, void *V_cache,
                 int32_t *seg_len, int32_t *overflow, void *hip_stream);

/* Scratch bytes adakv_decode_attn needs for this layer and head-room (0 on invalid input). */
size_t adakv_decode_workspace_bytes(const adakv_layer *L, int32_t headroom);

/*
 * One decoding step of Eq. (2) per query head over segments of different lengths (the
 * variable-length attention of Section 3.5): for sequence b and query head i, with
 * s = b*h_kv + i/g and the seg_len[s] rows of that segment,
 *
 *     out[b][i][:] = sum_t softmax_t(scale * q_new[b][i] . K_cache[start_s + t]) V_cache[start_s + t][:]
 *     lse[b][i]    = ln sum_t exp(scale * q_new[b][i] . K_cache[start_s + t])
 *
 * Logits, the softmax and the weighted sum are accumulated in fp32.  A segment of length 0
 * gives a zero row and lse = -inf.  The projection by W^O is not part of this call.
 *
 *   q_new (device) [batch][h_q][d] contiguous, L->dtype, 16-byte aligned
 *   out   (device) [batch][h_q][d] fp32, written
 *   lse   (device) [batch][h_q] fp32, written; may be NULL
 *   ws    (device) adakv_decode_workspace_bytes(L, headroom) bytes
 * Supported (else ADAKV_EUNSUPPORTED): g = h_q/h_kv in {1, 2, 4, 8}; d in {64, 128}.
 */
int adakv_decode_attn(const adakv_layer *L, const void *q_new, const int32_t *cu_seqlens,
                      int32_t headroom, const void *K_cache, const void *V_cache,
                      const int32_t *seg_len, float *out, float *lse, void *ws, size_t ws_bytes,
                      void *hip_stream);

/*
 * adakv_append followed by adakv_decode_attn in one call (one kernel launch fewer per decoding
 * step, and the new row is not read back from memory): every segment with room takes
 * k_new[b][c], v_new[b][c] as its next row, attention runs over the rows including it, and
 * seg_len[s] grows by one when the call's last kernel ends.  A full segment is attended as it
 * is, keeps its length, and sets *overflow to 1.  Arguments as for the two calls.
 */
int adakv_decode_step(const adakv_layer *L, const void *q_new, const void *k_new,
                      const void *v_new, const int32_t *cu_seqlens, int32_t headroom,
                      void *K_cache, void *V_cache, int32_t *seg_len, int32_t *overflow,
                      float *out, float *lse, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Layer budgets for the pyramidal variant (Section 3.4: Ada-Pyramid differs from Ada-SnapKV only
 * in how the total budget is spread over the layers, "via pre-set hyper-parameters" that the
 * paper does not give; inside a layer the algorithm is the same).  Host arithmetic only.  The
 * schedule chosen here is linear in depth, largest at layer 0:
 *     real_l = B_max - (B_max - B_min) * l / (n_layers - 1),  B_max = ratio * B_min,
 *     B_min = 2 * avg_budget / (1 + ratio),  so that the mean over the layers is avg_budget;
 * out[l] = floor(real_l) and the units still missing from n_layers * avg_budget go one each to
 * the first layers.  ratio = 1 gives avg_budget everywhere.
 *
 *   out (host) [n_layers] int64, written; sum = n_layers * avg_budget, non-increasing
 * The arithmetic is exact (the double `ratio` is taken as the binary fraction it is, everything
 * else is integer), so out[l] is the floor of the real value in every case.
 * Returns ADAKV_EINVAL for n_layers < 1, avg_budget < 0, ratio < 1 or not finite, out == NULL;
 * ADAKV_EUNSUPPORTED for avg_budget > 2^40, n_layers > 2^24 or ratio > 2^20.
 */
int adakv_pyramid_budgets(int32_t n_layers, int64_t avg_budget, double ratio, int64_t *out);

/*
 * Profiling aid for benchmarks (no part of the method).  While armed, on the arming host thread,
 * every kernel the library launches carries two of the caller's events, taken from the array in
 * order: events 2i and 2i+1 receive the start and the end timestamp of the i-th kernel itself
 * (hipEventElapsedTime between them is that kernel's run time, without launch gaps), and
 * adakv_trace_name(2i) names it.  When fewer than two events are left, further kernels are
 * launched plainly.  Dispatches that carry events are ordered more strictly by the runtime, so
 * throughput is measured unarmed.
 *
 *   events (host) array of n_events hipEvent_t handles created by the caller, which must stay
 *          alive until adakv_trace_disarm; 2 <= n_events <= ADAKV_TRACE_MAX
 * adakv_trace_disarm returns how many events were used; adakv_trace_name(i) is valid until
 * the next adakv_trace_arm on the same thread.
 */
#define ADAKV_TRACE_MAX 256
int adakv_trace_arm(void *const *events, int n_events);
int adakv_trace_disarm(void);
const char *adakv_trace_name(int i);

/*
 * Diagnostic (host only, launches nothing): which kernels a layer of this shape is scored and
 * selected with, as one line of "key=value" words, e.g.
 *   score=mfma dtype=bf16 d=128 rows=128 mb=2 rs=2 kg=2 chunk=2048 stats=sweep lse=fused pool=fused topk=carried
 * score: mfma (matrix cores) | fma (plain FMA path) | fma-pool-first (ADAKV_FLAG_POOL_THEN_MEAN);
 * rows = g*w window rows per KV head; mb/rs/kg/chunk: 32-row blocks per wavefront, wavefronts
 * along rows and along keys, keys per workgroup; stats: sweep (the statistics sweep runs) |
 * caller (row_lse given); lse / pool: fused into the weights sweep | a kernel of their own;
 * topk: carried (ADAKV_FLAG_PIPELINE in effect) | separate.  The tests use it to check that
 * every variant is exercised.
 *
 *   have_row_lse  non-zero: describe a call that passes row_lse
 *   out (host)    out_bytes bytes, written, NUL-terminated
 * Returns what adakv_score would return for the layer's validity, ADAKV_EINVAL if the text
 * does not fit.
 */
int adakv_describe(const adakv_layer *L, int have_row_lse, char *out, size_t out_bytes);

/*
 * Measurement aid for benchmarks (no part of the method): a plain streaming read of a device
 * buffer, 16 bytes per lane, by ADAKV_PROBE_BLOCKS long-running workgroups.  Its rate on the K
 * buffers is the figure a scoring sweep, which has to read K once, is compared with.
 *
 *   src  (device) bytes bytes, 16-byte aligned, read once; bytes must be a multiple of 16
 *                 (0 is allowed, src may then be NULL: the sink is all zero afterwards)
 *   sink (device) ADAKV_PROBE_SINK_BYTES bytes, 16-byte aligned, written: one 16-byte word per
 *                 wave, the XOR of the words that wave read (the XOR of all of them is the XOR
 *                 of the buffer's 16-byte words, which is what makes the reads observable)
 * Returns ADAKV_EINVAL for a NULL sink, a NULL src with bytes > 0 or bytes % 16 != 0,
 * ADAKV_EUNSUPPORTED for a misaligned pointer, ADAKV_EHIP if the launch failed.  Enqueues one
 * kernel on hip_stream.
 */
#define ADAKV_PROBE_BLOCKS 2048
#define ADAKV_PROBE_SINK_BYTES (ADAKV_PROBE_BLOCKS * 4 * 16)
int adakv_probe_read(const void *src, size_t bytes, void *sink, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ADAKV_H */
