/* xsv — per-frame streaming step of XStreamVGGT on MI355X (gfx950), C ABI.
 *
 * One global-attention layer of the streaming model keeps a KV cache per layer (paper Sec. 3.1).
 * For every incoming frame the layer (1) attends the frame's queries over [cache ; frame],
 * (2) once the cache would exceed its token budget, scores the prunable middle with pooled
 * queries and keeps the top-k (Sec. 3.2), and (3) re-quantizes the retained cache, keys per
 * channel and values per token (Sec. 3.3).  This library is exactly that path; every step runs
 * in HIP kernels on the stream given at creation.
 *
 * Conventions
 *   - All functions return 0 (XSV_OK) or a negative error code; they never throw, abort or exit.
 *     Argument errors are detected on the host before anything is launched.
 *   - "DEVICE" pointers are HIP device memory owned by the caller and must stay valid until the
 *     stream has passed the call.  "HOST" pointers are ordinary host memory.
 *   - Q/K/V are bf16 (raw 16-bit patterns), channel-contiguous, described by xsv_tensor with
 *     strides in ELEMENTS; row r of head h starts at ptr + h*stride_head + r*stride_token.
 *     The first n_special rows of a frame are its camera/register tokens, the rest patch tokens.
 *   - A context owns all cache and workspace memory, is bound to one stream and is not
 *     thread-safe.  Calls are asynchronous on that stream unless stated otherwise.
 *   - Per layer and frame the order is attend → score_prune → quantize (xsv_step does the three);
 *     any other order returns XSV_ERR_STATE.
 */
#ifndef XSV_H
#define XSV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  XSV_OK = 0,
  XSV_ERR_ARG = -1,         /* NULL pointer, out-of-range value, inconsistent sizes        */
  XSV_ERR_UNSUPPORTED = -2, /* valid in the method, not built (e.g. head_dim != 64)        */
  XSV_ERR_OOM = -3,         /* device allocation failed                                     */
  XSV_ERR_STATE = -4,       /* call order violated, or layers out of step for a batched call */
  XSV_ERR_HIP = -5          /* a HIP call failed; the context can only be destroyed          */
};

typedef struct xsv_ctx xsv_ctx; /* opaque */

typedef struct {
  int32_t n_layers;         /* L >= 1                                                          */
  int32_t n_heads;          /* H >= 1                                                          */
  int32_t head_dim;         /* d; must be 64                                                   */
  int32_t tokens_per_frame; /* n = n_special + patches                                         */
  int32_t n_special;        /* camera + register tokens, first rows of each frame (Sec. 3.1)  */
  int32_t budget;           /* L_max, tokens per head per layer (Sec. 3.2); 0 = unbounded      */
  int32_t kv_bits;          /* 2 | 4 = quantized cache (Sec. 3.3); 16 = bf16 cache, no quantizer */
  int32_t group_size;       /* G: 32 | 64; keys: tokens per group, values: channels per group  */
  int32_t pool_size;        /* g of the pooled query (Sec. 3.2), >= 1                           */
  int32_t score_mode;       /* 0: the paper's score (Sec. 3.2): queries and keys averaged over the heads,
                               one retained index set per layer shared by all heads.
                               1: a variant: no averages over heads, every head scores its own keys with
                               its own pooled queries and keeps its own top-k (same count for all heads) */
  float softmax_scale;      /* 0 → 1/sqrt(head_dim)                                            */
  int32_t max_frames;       /* only for budget == 0: frames the cache must be able to hold     */
  int32_t value_mode;       /* 0: the whole retained cache is quantized anew every step (Sec. 3.3 applied to the
                               final cache, history through its dequantized view).
                               1: a variant, "quantize once" for the values: a value row is quantized when its
                               frame is appended and keeps those codes, its scale and its zero point while it is
                               retained (its groups are its own channels).  Keys are quantized anew either way:
                               their groups are runs of retained tokens.  No effect with kv_bits == 16. */
} xsv_config;

typedef struct {
  const void* ptr;      /* DEVICE, bf16, 16-byte aligned */
  int64_t stride_head;  /* elements, >= 0, a multiple of 8 */
  int64_t stride_token; /* elements, a multiple of 8, >= head_dim and <= 2^24; for K and V the rows
                           of one head of a frame must lie within 2 GiB,
                           ((tokens_per_frame - 1) * stride_token + head_dim) * 2 <= 2^31 (they are
                           fetched in 16-byte pieces through 32-bit byte offsets); anything else
                           is XSV_ERR_ARG */
} xsv_tensor;

/* ---- life cycle ------------------------------------------------------------------------------- */

/* Validates cfg, allocates the double-buffered packed caches and all workspaces for every layer
 * on the current device, launches nothing that computes.  hip_stream is a hipStream_t (NULL = the
 * default stream).  On success *out owns the memory until xsv_destroy. */
int xsv_create(const xsv_config* cfg, void* hip_stream, xsv_ctx** out);
/* Synchronizes the stream and frees everything.  NULL is allowed. */
int xsv_destroy(xsv_ctx* ctx);
/* Starts a new stream: every layer's cache length and frame count return to 0. */
int xsv_reset(xsv_ctx* ctx);

/* ---- the hot path (asynchronous, no host synchronization) --------------------------------------- */

/* Sec. 3.1 temporal attention with Sec. 3.3 dequantization fused in:
 *   out = softmax(scale * q [K~ ; k_new]^T) [V~ ; v_new],   K~, V~ = (code - zero) * scale per group,
 * for the n queries of the current frame over the layer's T cached tokens plus the frame's own
 * n tokens; nothing is masked inside a step (every key belongs to a frame <= the current one).
 * q, k_new, v_new: bf16 [H][n][64] via strides.  out: DEVICE bf16 [H][n][64] contiguous. */
int xsv_dequant_attend(xsv_ctx* ctx, int layer, xsv_tensor q, xsv_tensor k_new, xsv_tensor v_new, void* out);

/* The frame-wise attention of the alternating-attention backbone (Sec. 3.1: the layers alternate between
 * attention inside each frame and global attention across frames): out = softmax(scale * q k^T) v over
 * the frame's own n tokens only, no cache involved and no state touched (any phase, any layer count).
 * Same kernel as xsv_dequant_attend with an empty cache.  q, k, v: bf16 [H][n][64] via strides;
 * out: DEVICE bf16 [H][n][64] contiguous. */
int xsv_frame_attend(xsv_ctx* ctx, xsv_tensor q, xsv_tensor k, xsv_tensor v, void* out);

/* Sec. 3.2 after the append (T = T_cache + n).  If budget == 0, T <= budget, or this is the first
 * frame, everything is kept.  Otherwise, with T_first = T_cur = n, P = T - T_first - T_cur and
 * k = min(max(0, budget - T_first - T_cur), P): the importance of every middle token j is
 *   S_j = mean_i (Qbar Kbar^T)[i][j],  Qbar = head-mean of [special rows ; patch rows averaged in
 *   consecutive groups of pool_size (a short last group over its real size)],
 *   Kbar = head-mean of the dequantized cached keys of the middle,
 * and the keep list is first frame ∪ top-k middle (equal scores: smaller position first) ∪ current
 * frame, in ascending position.  One list per layer, shared by all heads and by K and V (score_mode 1:
 * the head-means are left out, head h scores its own keys with its own pooled queries, and there is one
 * list per head).  Writes context-owned scores and keep list(s); frame-t keys themselves are never scored. */
int xsv_score_prune(xsv_ctx* ctx, int layer, xsv_tensor q);

/* Sec. 3.3 on the final cache of the step: gathers the kept rows (cached rows through their
 * dequantized bf16 view (code - zero) * scale, frame rows as given) and quantizes all of them:
 *   s = (max - min) / (2^b - 1)  (s = 1 if max == min),  zero = round(-min / s),
 *   code = clamp(round(x / s) + zero, 0, 2^b - 1),   round = nearest-even, x / s the IEEE fp32 quotient,
 * keys per (head, channel) over groups of G consecutive kept tokens (short last group on its own),
 * values per (head, token) over groups of G consecutive channels.  With kv_bits == 16 the rows are
 * stored as bf16 unchanged.  The result is the layer's cache; cache length becomes the keep length.
 * (A budgeted cache is written into the layer's second buffer and the two swap; a cache with
 * budget 0 never moves a row and is rewritten in place in its single buffer.  A block of 64 cached
 * tokens that keeps its place and that one re-quantization reproduced bit for bit is not
 * recomputed again - its result is the same bytes either way.) */
int xsv_quantize(xsv_ctx* ctx, int layer, xsv_tensor k_new, xsv_tensor v_new);

/* The three calls above for one layer.  Attention runs on the context's stream while score, select
 * and re-quantization run concurrently on a stream owned by the context (they read the same inputs
 * and write the layer's other cache buffer).  In the default overlap mode (1) the context's stream is
 * ordered after both when the call returns, so the usual "valid until the stream has passed the
 * call" rule holds; see xsv_set_overlap for the mode that defers this join. */
int xsv_step(xsv_ctx* ctx, int layer, xsv_tensor q, xsv_tensor k_new, xsv_tensor v_new, void* out);

/* One frame through ALL layers with layer-batched launches (arrays of n_layers entries; every
 * layer must be at the same frame, else XSV_ERR_STATE; all q share strides, likewise k, v;
 * n_layers <= 32, else XSV_ERR_UNSUPPORTED).  Same results as n_layers calls of xsv_step.  Only
 * meaningful when the layers' inputs do not depend on each other's outputs (synthetic streams). */
int xsv_step_all_layers(xsv_ctx* ctx, const xsv_tensor* q, const xsv_tensor* k_new, const xsv_tensor* v_new,
                        void* const* out);

/* How xsv_step / xsv_step_all_layers order the score/select/re-quantize chain:
 *   0  everything on the context's stream, in order;
 *   1  (default) the chain overlaps the attention kernel on the context's side stream and the
 *      context's stream waits for it before the call returns;
 *   2  as 1, but the wait is deferred: the context's stream waits for the chain of a layer only
 *      before the next call that touches that layer, or in xsv_join.  A cross-stream wait costs
 *      more than most of these kernels run, and the next LAYER's attention does not depend on this
 *      layer's chain — only this layer's next FRAME does.  In this mode q, k_new and v_new of a step
 *      must stay valid and unchanged until the context's stream has passed the next call for that
 *      layer or an xsv_join; `out` follows the usual rule.
 * Switching the mode joins first. */
int xsv_set_overlap(xsv_ctx* ctx, int mode);
/* Orders the context's stream after all side-stream work enqueued so far (no host wait).  A no-op
 * unless overlap mode 2 has steps outstanding. */
int xsv_join(xsv_ctx* ctx);
/* ---- introspection, synchronous, HOST buffers, canonical unpacked layout ------------------------ */

/* Cache length T of a layer (tokens per head). */
int xsv_cache_len(xsv_ctx* ctx, int layer, int32_t* T);

/* Copies a layer's cache out.  Any pointer may be NULL.  With T = cache length, H, d = 64, G:
 *   k_codes, v_codes  uint8 [H][T][d], one code per byte            (kv_bits 2|4 only)
 *   k_scale, k_zero   float [H][ceil(T/G)][d]                        (kv_bits 2|4 only)
 *   v_scale, v_zero   float [H][T][d/G]                              (kv_bits 2|4 only)
 *   k_bf16, v_bf16    uint16 [H][T][d]: the dequantized view (kv_bits 2|4) or the stored rows (16)
 *   token_frame, token_index int32 [T]: which frame / row each cached token came from
 *                     (score_mode 1: [H][T], every head has its own retained set). */
int xsv_cache_export(xsv_ctx* ctx, int layer, uint8_t* k_codes, float* k_scale, float* k_zero, uint8_t* v_codes,
                     float* v_scale, float* v_zero, uint16_t* k_bf16, uint16_t* v_bf16, int32_t* token_frame,
                     int32_t* token_index);

/* Replaces a layer's cache (same arrays as the export; codes/scales for kv_bits 2|4, bf16 rows for
 * 16).  frames_seen becomes the layer's frame count (>= 1 when T > 0); the first frame is taken to
 * be the first tokens_per_frame tokens. */
int xsv_cache_import(xsv_ctx* ctx, int layer, int32_t T, int32_t frames_seen, const uint8_t* k_codes,
                     const float* k_scale, const float* k_zero, const uint8_t* v_codes, const float* v_scale,
                     const float* v_zero, const uint16_t* k_bf16, const uint16_t* v_bf16,
                     const int32_t* token_frame, const int32_t* token_index);

/* What the last xsv_score_prune of this layer decided: n_scores = P if scores were computed (else
 * 0), n_keep = length of the keep list (positions in [cache ; frame]).  Buffers may be NULL to query
 * sizes only; otherwise they must hold n_scores floats / n_keep ints (score_mode 1: H lists of that
 * length each, [H][n_scores] and [H][n_keep]). */
int xsv_last_selection(xsv_ctx* ctx, int layer, int32_t* n_scores, float* scores, int32_t* n_keep, int32_t* keep);

/* ---- stateless kernels (DEVICE pointers; synchronous: they allocate temporaries and wait) ------- */

/* Sec. 3.3 quantizers on a plain bf16 tensor [H][T][64] (contiguous).  Outputs canonical:
 * codes uint8 [H][T][64]; keys: scale, zero float [H][ceil(T/G)][64]; values: [H][T][64/G]. */
int xsv_quantize_k(void* hip_stream, const void* k_bf16, int H, int T, int d, int bits, int G, void* codes_u8,
                   float* scale, float* zero);
int xsv_quantize_v(void* hip_stream, const void* v_bf16, int H, int T, int d, int bits, int G, void* codes_u8,
                   float* scale, float* zero);
/* Sec. 3.2 importance of P keys k_mid (bf16 [H][P][64] contiguous) for the frame's queries q
 * (n rows, first n_s special, pooling size g).  scores: float [P]. */
int xsv_score(void* hip_stream, xsv_tensor q, const void* k_mid_bf16, int H, int n, int n_s, int P, int d, int g,
              float* scores);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): xsv_score with its one temporary - the per-head partial sums of the pooled query - in
 * a fixed device array of the library instead of a hipMalloc'ed buffer.  Same arguments, same kernels, same
 * scores as xsv_score.  Differences: it calls no hipMalloc / hipFree and does not wait - it only enqueues on
 * hip_stream, so `scores` is valid once the stream has passed the call; H is limited to
 * XSV_NOALLOC_MAX_HEADS (more: XSV_ERR_UNSUPPORTED, nothing launched); the array (16 KB) stays allocated on
 * every device the call ran on until the process ends.  All calls on one device share that array: calls
 * whose kernels could overlap on one device (different streams, no ordering between them) race; order them. */
#define XSV_NOALLOC_MAX_HEADS 64
int xsv_score_noalloc(void* hip_stream, xsv_tensor q, const void* k_mid_bf16, int H, int n, int n_s, int P, int d, int g,
                      float* scores);
/* Sec. 3.2 keep list from scores [P]: [0,T_first) ∪ (T_first + top-k) ∪ [T_first+P, T_first+P+T_cur),
 * ascending; keep: int32 [T_first + k + T_cur]. */
int xsv_topk_keep(void* hip_stream, const float* scores, int P, int k, int T_first, int T_cur, int32_t* keep);

const char* xsv_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* XSV_H */
