/* linear_kv.h -- C ABI of the LineAR decode path for one MI355X (gfx950).
 *
 * The library keeps, per layer, a line-structured visual KV cache
 *     [ C conditional | N_init anchor | mid survivors | r recent lines | line being written ]
 * compact and contiguous per (sequence, head), and runs on it
 *   - single-query decode attention with the append of the new (k, v)   (paper Eq. 2-4),
 *   - accumulation of the saliency of the mid tokens under the queries of the
 *     line being generated                                                (Eq. 8-9),
 *   - at the end of a raster line, BottomK selection of n mid tokens per
 *     head and the order-preserving compaction of K, V and the survivors' positions
 *                                                                        (Eq. 5-7, 10).
 * Symbols are the paper's (Sec. 3.1, 3.3): C, n (tokens per raster line, an
 * end-of-line token counts), h lines, N = h n, budget B (n divides B),
 * rho = B/N, N_init, r.
 *
 * Conventions for every entry point
 *   - Pointers marked DEVICE are device memory owned by the caller for as long as
 *     the handle lives; the library never allocates or frees device memory.
 *     Pointers marked HOST are ordinary host memory read or written during the call.
 *   - All DEVICE pointers must be 16-byte aligned (LINEAR_EALIGN otherwise).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work: none synchronises, none reads device memory back.
 *     All calls on one handle must be issued in stream order on one stream.
 *   - Return value: LINEAR_OK (0) or a negative LINEAR_E* code; on error the
 *     handle's state is unchanged and nothing was enqueued.
 *   - Tensors are dense row-major with the listed shape.  "elem" is the
 *     storage type selected by cfg.dtype (float or bfloat16).  Bz = batch,
 *     H = n_heads, d = head_dim.
 */
#ifndef LINEAR_KV_H
#define LINEAR_KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LINEAR_API __attribute__((visibility("default")))

#define LINEAR_OK 0
#define LINEAR_EINVAL (-1) /* bad configuration or argument value            */
#define LINEAR_ESTATE (-2) /* call not allowed in the layer's current state  */
#define LINEAR_ENULL (-3)  /* required pointer is NULL                       */
#define LINEAR_EALIGN (-4) /* device pointer not 16-byte aligned             */
#define LINEAR_EHIP (-5)   /* a HIP call failed: see linear_last_hip_error() */
#define LINEAR_ECAPACITY (-6) /* decode_step_static: the step needs more scratch than the library holds */

#define LINEAR_F32 0
#define LINEAR_BF16 1

#define LINEAR_OUT_F32 0
#define LINEAR_OUT_ELEM 1

#define LINEAR_QUEUE_AUTO 0
#define LINEAR_QUEUE_LOGITS 1
#define LINEAR_QUEUE_QUERIES 2

typedef struct linear_kv linear_kv_t; /* opaque; host-side bookkeeping only */

typedef struct {
  int32_t n_layers;
  int32_t batch;          /* Bz: independent sequences (CFG halves are just sequences) */
  int32_t n_heads;        /* H; keys/values have the same number of heads             */
  int32_t head_dim;       /* d: 64 or 128                                             */
  int32_t n_cond;         /* C >= 0: never evicted, never scored, outside the budget  */
  int32_t line_len;       /* n <= 4096                                                */
  int32_t n_lines;        /* h                                                        */
  int32_t budget;         /* B: multiple of n, n <= B <= h n; B == h n never evicts   */
  int32_t n_init;         /* N_init visual anchor tokens, 0 <= N_init <= B            */
  int32_t n_recent_lines; /* r, 1 <= r <= h; needs N_init + (r+1) n <= B when B < h n, and the
                             mid region B - N_init - r n must not exceed 2048 tokens  */
  int32_t dtype;          /* LINEAR_F32 or LINEAR_BF16: q, k, v and both caches       */
  int32_t score_mode;     /* 0: Eq. 9 as printed, softmax over the mid tokens only;
                             1: each query's decode-time probabilities (softmax over
                                everything it attends to) restricted to mid;
                             2: accumulated attention (the paper's AttAcc ablation, Table 6):
                                every token behind the anchor carries the sum of the
                                decode-time probabilities it received from every query since
                                it was appended, never reset; needs B - N_init <= 7680;
                             3: random eviction inside the same pipeline (the paper's Random baseline,
                                Sec. 4.2 / Table 3, restricted to the mid region): a candidate's score is
                                a 24-bit integer hash of (seed, layer, sequence, head, line, original
                                position) -- h = mix(seed ^ 0x9e3779b9), then h = mix(h + x) for each of
                                the five counters in that order, score = h >> 8, where mix(x) is
                                x ^= x >> 16, x *= 0x7feb352d, x ^= x >> 15, x *= 0x846ca68b, x ^= x >> 16
                                in 32-bit arithmetic; line counts from 1, positions as kv_gather
                                reports them.  No guide queue is kept and the decode step scores nothing */
  int32_t guide_queue;    /* what the line's guide queue holds (Eq. 8):
                             LINEAR_QUEUE_QUERIES: the queries themselves, as Eq. 8 prints it;
                                Eq. 9 is evaluated at the end of the line as the matrix
                                product Q_guide K_mid^T on the matrix cores.  score_mode 0 only;
                             LINEAR_QUEUE_LOGITS: every query's logits on the scored keys, taken
                                from the decode step's own q.k (Eq. 9 then needs no product);
                             LINEAR_QUEUE_AUTO: queries with score_mode 0 (measured faster on
                                every benchmark workload), logits with score_mode 1 and 2;
                                score_mode 3 keeps no queue and accepts only this value      */
  float scale;            /* logit scale; 0 selects 1/sqrt(d) (Eq. 2)                 */
  uint32_t seed;          /* score_mode 3: seed of the random draws; ignored otherwise */
  int32_t out_dtype;      /* type of decode_step's `out`: LINEAR_OUT_F32 (float), or LINEAR_OUT_ELEM
                             (the storage type, rounded to nearest even: what the output projection
                             that follows attention takes as its input)                      */
} linear_cfg_t;

/* Sizes the caller must allocate (Sec. 3.3: at most C + B pairs per head are cached).
 *   *cache_bytes_per_layer : bytes of EACH of the K and the V cache of one layer,
 *                            laid out [Bz, H, C + B, d] elem;
 *   *scratch_bytes         : bytes of the one scratch buffer shared by all layers
 *                            (guide queues, survivor position maps, attention accumulators,
 *                            split partials).
 * HOST pointers.  LINEAR_EINVAL if the configuration is not valid. */
LINEAR_API int linear_workspace_bytes(const linear_cfg_t* cfg, size_t* cache_bytes_per_layer,
                           size_t* scratch_bytes);

/* Start an image (Sec. 3.1, prefill result): creates the handle, copies the conditional
 * K/V into rows [0, C) of every layer's cache and clears the saliency accumulators.
 *   k_cache, v_cache : HOST arrays of n_layers DEVICE pointers, each
 *                      cache_bytes_per_layer big; contents need no initialisation;
 *   scratch          : DEVICE, scratch_bytes big;
 *   k_cond, v_cond   : HOST arrays of n_layers DEVICE pointers to [Bz, H, C, d] elem
 *                      (may be NULL when C == 0); read during the enqueued copy only;
 *   *out             : receives the handle (release with kv_free). */
LINEAR_API int kv_init(const linear_cfg_t* cfg, void* const* k_cache, void* const* v_cache, void* scratch,
            const void* const* k_cond, const void* const* v_cond, void* stream,
            linear_kv_t** out);

/* One decode step of one layer (Eq. 2-4, and the per-query term of Eq. 9 on lines that
 * end in an eviction): appends (k, v) as visual token i at original position C + i - 1
 * and writes out = Softmax(q K^T * scale) V over every cached key including the new one.
 *   q, k, v : DEVICE [Bz, H, d] elem, already rotated if the model uses RoPE;
 *   out     : DEVICE [Bz, H, d] float (elem with cfg.out_dtype = LINEAR_OUT_ELEM).  Dense row-major,
 *             so it is at the same time [Bz, H d]: one row per sequence with its heads side by
 *             side, the left operand of the output projection, with no transpose in between.
 * LINEAR_ESTATE if the layer's line is complete (end_of_line_evict is due) or the image
 * is complete. */
LINEAR_API int decode_step(linear_kv_t* kv, int32_t layer, const void* q, const void* k, const void* v,
                void* out, void* stream);

/* The same step for `count` consecutive layers whose inputs are already resident (a
 * benchmark, or a runtime that pipelines layers): exactly decode_step(kv, first_layer + i,
 * q + i*qkv_stride, k + i*qkv_stride, v + i*qkv_stride, out + i*out_stride, stream) for
 * i = 0 .. count-1 (strides in bytes, multiples of 16), enqueued back to back.  Stops at the
 * first error and returns it; layers before it have been enqueued and advanced. */
LINEAR_API int decode_step_layers(linear_kv_t* kv, int32_t first_layer, int32_t count, const void* q,
                       const void* k, const void* v, void* out, size_t qkv_stride,
                       size_t out_stride, void* stream);

/* decode_step with the rotary position embedding of the new token fused in (the producer side
 * of Eq. 2-4: the paper's models rotate q and k before attention).  q and k arrive as the
 * projection leaves them, NOT rotated; the step rotates both in fp32 (element t paired with
 * t + d/2: x'_t = x_t cos_t - x_(t+d/2) sin_t, x'_(t+d/2) = x_t sin_t + x_(t+d/2) cos_t, every
 * product and sum rounded separately), rounds to the storage type, attends with the rotated q
 * and appends the rotated k; v is used as is.
 *   cos_sin : DEVICE [d] float, 16-byte aligned: the d/2 cosines, then the d/2 sines, of the
 *             pair angles at the new token's position; read during the step only.
 * Everything else as decode_step. */
LINEAR_API int decode_step_rope(linear_kv_t* kv, int32_t layer, const void* q, const void* k, const void* v,
                     const float* cos_sin, void* out, void* stream);

/* decode_step_rope for `count` consecutive layers (one position, so one cos_sin row); strides
 * and error behaviour as decode_step_layers. */
LINEAR_API int decode_step_rope_layers(linear_kv_t* kv, int32_t first_layer, int32_t count, const void* q,
                            const void* k, const void* v, const float* cos_sin, void* out,
                            size_t qkv_stride, size_t out_stride, void* stream);

/* End of a raster line of one layer (Sec. 3.3; Eq. 5-7 and 10).  Must follow exactly n
 * decode_step calls.  On lines B/n .. h-1 it evicts, independently per (sequence, head),
 * the n mid tokens with the smallest saliency (ties: older token first) and compacts K, V and
 * the position map in place keeping ascending original position; on other lines it only
 * advances the line counter (with score_mode 2 it also folds the line's attention into the
 * per-token accumulators).
 * LINEAR_ESTATE in the middle of a line. */
LINEAR_API int end_of_line_evict(linear_kv_t* kv, int32_t layer, void* stream);

/* end_of_line_evict for layers first_layer .. first_layer + count - 1.  The evictions of
 * different layers do not depend on one another, so layers that are in the same state (the
 * usual case: every layer has just finished the same line) share kernel launches, up to 48
 * layers each; otherwise the calls are enqueued one by one, stopping at the first error. */
LINEAR_API int end_of_line_evict_layers(linear_kv_t* kv, int32_t first_layer, int32_t count, void* stream);

/* Saliency of the current line so far (Eq. 9): S[j] for the mid candidates, averaged over
 * the n queries of the line (meaningful after the n-th decode_step of an evicting line,
 * before end_of_line_evict); with score_mode 2 the attention accumulated so far; with
 * score_mode 3 the candidates' random keys for this line.  out: DEVICE [Bz, H, mid] float with
 * mid = B - N_init - r n; *mid_out (HOST, may be NULL) receives mid.
 * LINEAR_ESTATE if the layer's current line does not evict. */
LINEAR_API int kv_scores(linear_kv_t* kv, int32_t layer, float* out, int32_t* mid_out, void* stream);

/* Export the retained cache of one layer (Sec. 3.3: what Eq. 5-6 leave after the evictions so
 * far -- conditional tokens, anchor, the mid tokens that survived, the recent lines -- plus the
 * line being written) in canonical order: conditional tokens, then visual tokens in ascending
 * original position.
 *   k_out, v_out : DEVICE [Bz, H, len, d] elem (either may be NULL to skip);
 *   pos_out      : DEVICE [Bz, H, len] int32 original positions (cond 0..C-1, visual
 *                  token i at C + i - 1); may be NULL;
 *   *len_out     : HOST, receives len = C + cached visual tokens (known on the host:
 *                  the eviction schedule does not depend on the data). */
LINEAR_API int kv_gather(linear_kv_t* kv, int32_t layer, void* k_out, void* v_out, int32_t* pos_out,
              int32_t* len_out, void* stream);

/* decode_step for callers that cannot allocate device memory and have no workspace to hand
 * over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * One stateless step on a cache the caller lays out itself: appends (k, v) as row
 * `cached_keys` of every pair's K and V and writes out = Softmax(q K^T * scale) V over the
 * cached_keys + 1 rows, exactly as decode_step does (same kernels).  When the keys of a pair
 * are split over several workgroups, the split partials -- which decode_step keeps in the
 * caller's workspace -- live in a device array inside the library: 4 MiB per GPU, held from
 * the first call on that GPU until the process ends, its address looked up on that first call
 * (make it, or a call of linear_static_scratch_bytes, outside graph capture).  The call
 * allocates and frees nothing, on the host or on the device.
 *   dtype, head_dim        : as in linear_cfg_t;
 *   n_pairs                : (sequence, head) pairs, >= 1;
 *   cached_keys            : rows already in the cache, >= 0;
 *   cache_pitch            : rows between consecutive pairs in k_cache / v_cache, > cached_keys;
 *   k_cache, v_cache       : DEVICE [n_pairs, cache_pitch, d] elem, rows [0, cached_keys) valid;
 *   q, k, v                : DEVICE [n_pairs, d] elem;   out : DEVICE [n_pairs, d] float;
 *   scale                  : logit scale, 0 selects 1/sqrt(d);
 *   n_split                : workgroups per pair, 1..64, or 0 = chosen as decode_step chooses it.
 * LINEAR_ECAPACITY when n_pairs * splits * (d + 2) floats exceed the 4 MiB (nothing enqueued);
 * other errors as decode_step.  All calls on one GPU share that GPU's array, which keeps the
 * last call's contents (nothing in it has to start at zero: every partial is written before it
 * is read): calls that may overlap on one GPU, on different streams or threads, race. */
LINEAR_API int decode_step_static(int32_t dtype, int32_t head_dim, int32_t n_pairs, int32_t cached_keys,
                       int32_t cache_pitch, void* k_cache, void* v_cache, const void* q, const void* k,
                       const void* v, float scale, int32_t n_split, void* out, void* stream);

/* Capacity in bytes of the array decode_step_static keeps its partials in; also performs the
 * one-time address lookup for the current device.  *bytes: HOST. */
LINEAR_API int linear_static_scratch_bytes(size_t* bytes);

/* Host-side queries (no device work). */
LINEAR_API int kv_length(const linear_kv_t* kv, int32_t layer, int32_t* cached_tokens,
              int32_t* tokens_in_line, int32_t* lines_done);

/* Releases the handle (host memory only). */
LINEAR_API int kv_free(linear_kv_t* kv);

LINEAR_API const char* linear_strerror(int code);
/* hipError_t of the most recent LINEAR_EHIP on the calling thread, as int. */
LINEAR_API int linear_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LINEAR_KV_H */
