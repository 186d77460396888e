/*
 * kvx -- compressed-KV streaming attention step for frame-wise causal global
 * attention (XStreamVGGT, arxiv 2601.01204), hand-written HIP for gfx950.
 *
 * One kv_step() is one frame on one per-layer cache:
 *   1. attention of the frame's queries over [de-quantised cache ; the frame's own
 *      K/V at input precision]                       (paper Sec. 3.1 Eq. 1, Sec. 3.3 Eq. 10)
 *   2. append the frame; if the length now exceeds the budget L_max, score the
 *      middle tokens with the pooled query           (Sec. 3.2 Eq. 2-6)
 *   3. keep first frame + top-k middle + current frame, k = L_max - 2n, in
 *      ascending position order                      (Sec. 3.2, keep set)
 *   4. quantise the final cache: keys per channel over groups of k_group
 *      consecutive cache tokens, values per token over groups of v_group
 *      channels, asymmetric uniform, round-to-nearest-even   (Sec. 3.3 Eq. 7-9)
 *
 * All pointers named "device" are HIP device pointers on the current device;
 * "host" pointers are ordinary host memory.  The library owns the cache, the
 * caller owns q/k/v/out.  No call throws or aborts; every call returns a
 * kv_status (0 = ok, negative = error) and kv_last_error() gives the text.
 * A handle is not thread-safe.  All kv_step / kv_step_batched calls on one handle must be
 * stream-ordered with each other, whatever caches they name: the partial-result buffers of
 * the attention kernel and the library's second stream belong to the handle, not to a cache.
 * Callers that want two caches to progress on two HIP streams at once use two handles.
 */
#ifndef KVX_H
#define KVX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum kv_status {
  KV_OK = 0,
  KV_E_INVAL = -1,   /* bad argument or configuration                     */
  KV_E_NOMEM = -2,   /* device or host allocation failed                  */
  KV_E_RANGE = -3,   /* stream / layer / size out of range                */
  KV_E_STATE = -4,   /* call not valid in the handle's current state      */
  KV_E_HIP = -5      /* a HIP runtime call failed                         */
};

enum kv_dtype { KV_BF16 = 0, KV_F32 = 1 };

enum kv_meta_format {
  KV_META_F32 = 0,  /* per group an fp32 scale and an int32 zero-point (8 bytes): the stored values are    */
                    /* exactly those of Eq. 8                                                              */
  KV_META_F16 = 1   /* 16-bit scale and 16-bit zero-point (4 bytes per group; INT4 with groups of 64 goes  */
                    /* from 5.0 to 4.5 bits per element).  The scale is rounded UP to its storage format   */
                    /* before the zero-point and the codes are computed from it, so the group's range      */
                    /* stays covered and the s/2 bound of Eq. 7-8 holds for the stored scale.  Keys store  */
                    /* the scale in the logit domain, a = s * softmax_scale * log2(e), with 7 significant  */
                    /* bits inside [2^-14, 2048]; Eq. 7 and Eq. 10 use s = a * fp32(1 / (softmax_scale *   */
                    /* log2 e)).  With 7 bits a * (code - z) is exact in half precision for 2- and 4-bit   */
                    /* codes, so Eq. 1 needs one matrix instruction per key tile instead of two.  Values   */
                    /* store s as a half inside [2^-14, 2048].  Zero-points are kept in [-1024, 1023].     */
                    /* Needs k_bits of 2 or 4 and in_dtype KV_BF16; keys with |k * softmax_scale * log2 e| */
                    /* >= 65504 are outside its domain.                                                    */
};

enum kv_order {
  KV_ATTEND_THEN_PRUNE = 0, /* Eq. 1 over [cache before the step ; the new frames at input precision], then the */
                            /* cache update (Sec. 3.1: "after attention computation ... appended")              */
  KV_PRUNE_THEN_ATTEND = 1  /* the other reading of Fig. 2's order: append, score, prune and quantise first,    */
                            /* then Eq. 1 over the compressed cache (at most L_max keys, the current frame in   */
                            /* codes like every other token).  One frame per call.                              */
};

enum kv_layout {
  KV_LAYOUT_COMPACT = 0,    /* survivors are compacted in ascending position order into the other half of a   */
                            /* double buffer; every key group behind the first dropped token changes members   */
                            /* and is re-quantised (Sec. 3.3: quantisation applied to the final cache)         */
  KV_LAYOUT_SLOTS = 1       /* tokens never move: a pruned token frees its slot, the call's new tokens fill    */
                            /* the freed slots in ascending order (then the never-used tail); one buffer, in   */
                            /* place; values and ids of survivors are not touched; a key group, k_group        */
                            /* consecutive slots, is re-quantised by Eq. 7-8 only when it received a new       */
                            /* member, every other group keeps codes, scale and zero-point bit for bit.  The   */
                            /* keep set of Sec. 3.2 is the same rule (ties keep the lower slot).  kv_export    */
                            /* returns ids in slot order.                                                      */
};

enum kv_mode {
  KV_COMPRESSED = 0,        /* pruned + quantised cache (the paper's method)                */
  KV_UNCOMPRESSED_BF16 = 1  /* baseline: bf16 cache that grows by n tokens per frame,       */
                            /* no pruning, no quantisation (what the paper compares against) */
};

typedef struct kv_config {
  int32_t n_streams;        /* independent caches: n_streams x n_layers                        */
  int32_t n_layers;
  int32_t n_heads;          /* H                                                               */
  int32_t head_dim;         /* d; must be 64                                                   */
  int32_t tokens_per_frame; /* n = 1 + R + N, special tokens first (Sec. 3.1)                  */
  int32_t n_special;        /* 1 + R camera/register tokens, not pooled (Sec. 3.2 Eq. 2)       */
  int32_t pool_group;       /* g, patch tokens averaged per pooled query row; paper: 16        */
  int32_t budget_tokens;    /* L_max; must be >= 2 * tokens_per_frame                          */
  int32_t k_bits;           /* 2, 4 or 8                                                       */
  int32_t k_group;          /* tokens per per-channel key group: 32 or 64                      */
  int32_t v_bits;           /* 2, 4 or 8                                                       */
  int32_t v_group;          /* channels per per-token value group: 32 or 64                    */
  int32_t in_dtype;         /* kv_dtype of q, k and v                                          */
  int32_t out_dtype;        /* kv_dtype of out (fp32 keeps the full result of the fp32         */
                            /* accumulation; bf16 rounds it to nearest-even on the store)      */
  int32_t mode;             /* kv_mode                                                         */
  int32_t max_frames;       /* KV_UNCOMPRESSED_BF16 only: frames the cache is sized for        */
  float softmax_scale;      /* 0 -> 1/sqrt(head_dim)                                           */
  int32_t meta_format;      /* kv_meta_format of the quantiser's scales and zero-points        */
  int32_t max_frames_per_step; /* most frames one kv_step_frames call may carry (0 or 1: one); */
                            /* budget_tokens must be >= (1 + max_frames_per_step) * tokens_per_frame */
  int32_t order;            /* kv_order                                                        */
  int32_t layout;           /* kv_layout                                                       */
} kv_config;

typedef struct kv_handle kv_handle;

/* One frame for one cache in a batched call. q, k, v, out: device, [n, H, d] with the
 * strides given to kv_step_batched. */
typedef struct kv_step_item {
  int32_t stream;
  int32_t layer;
  const void* q;
  const void* k;
  const void* v;
  void* out;
} kv_step_item;

typedef struct kv_stats_t {
  int64_t bytes_allocated;       /* device bytes held by the handle; constant after kv_init      */
  int64_t bytes_k_codes;         /* of which: key codes (both halves of the double buffer)       */
  int64_t bytes_k_meta;          /*           key scales and zero-points                         */
  int64_t bytes_v_codes;
  int64_t bytes_v_meta;
  int64_t bytes_ids;
  int64_t bytes_scratch;         /* attention partials, scores, keep lists                       */
  int64_t bytes_live_per_cache;  /* codes + metadata of one cache at its current maximum length  */
  int64_t frames_seen_total;     /* sum over caches                                              */
  int64_t tokens_dropped_total;  /* sum over caches                                              */
  int64_t k_groups_rebuilt_total;/* key groups written by the re-quantiser, sum over caches      */
  int32_t cache_len_min;         /* over caches                                                  */
  int32_t cache_len_max;
  int32_t n_caches;
  int32_t nonfinite_flag;        /* 1 if a step with "debug_checks" on met an infinity or NaN in  */
                                 /* q, k or v since kv_init (the step itself ran unchanged)       */
  int64_t zp_range_warnings;     /* quantisation groups written since kv_init whose zero-point    */
                                 /* lies beyond +-2^20: their values sit so far from zero,        */
                                 /* measured in quantisation steps, that Eq. 10 cancels most bits */
                                 /* (KV_META_F16: groups whose scale or zero-point had to be      */
                                 /* brought into the 16-bit format's range)                       */
} kv_stats_t;

/* Host buffers for kv_export; any pointer may be NULL to skip that part. Sizes are in
 * elements, for T = cache length, H heads, d head_dim. */
typedef struct kv_export_t {
  int32_t cache_len;     /* out: T                                                            */
  int32_t frames_seen;   /* out                                                               */
  int32_t last_keep_len; /* out: length of the last keep list (0 if the last step kept all)   */
  int32_t last_scores_len; /* out: number of middle tokens scored in the last step            */
  int32_t* ids;          /* [T] token ids (frame * n + index) in cache order                  */
  uint8_t* k_codes;      /* [H, T, d] one code per byte                                       */
  float* k_scale;        /* [H, ceil(T / k_group), d]                                         */
  int32_t* k_zero;       /* [H, ceil(T / k_group), d]                                         */
  uint8_t* v_codes;      /* [H, T, d]                                                         */
  float* v_scale;        /* [H, T, d / v_group]                                               */
  int32_t* v_zero;       /* [H, T, d / v_group]                                               */
  int32_t* last_keep;    /* [budget] positions kept by the last pruning step, ascending,      */
                         /* indexing the pre-prune sequence [cache ; current frame]           */
  float* last_scores;    /* [last_scores_len] importance scores of the middle tokens          */
  int32_t capacity_tokens; /* in: capacity of the buffers above in tokens (>= T)              */
} kv_export_t;

/* Validate the configuration and allocate every device buffer the handle will ever use
 * (Sec. 3.2: the cache is bounded by L_max, so the footprint is fixed here).
 * cfg: host. out: host, receives the handle. */
int kv_init(const kv_config* cfg, kv_handle** out);

/* One frame on cache (stream, layer): Eq. 1 with Eq. 10 inside, then Eq. 2-9 to update
 * the cache.  q, k, v: device, [n, H, d], element (i, h, c) at i * tok_stride +
 * h * head_stride + c (strides in elements; the innermost d elements contiguous, every
 * row 16-byte aligned).  out: device, same layout with the same element strides, in the
 * configured out_dtype, receives the attention
 * output defined by the cache as it was before this step's pruning.  Work is enqueued on
 * hip_stream (a hipStream_t, NULL = default stream); the call never synchronises.  All
 * validation precedes the first launch, so a failed call leaves the cache unchanged. */
int kv_step(kv_handle* h, int32_t stream, int32_t layer, const void* q, const void* k, const void* v,
            int64_t tok_stride, int64_t head_stride, void* out, void* hip_stream);

/* A chunk of n_frames consecutive frames of one stream in one call (1 <= n_frames <= max_frames_per_step).
 * q, k, v, out: device, [n_frames * n, H, d], frame after frame, strides as in kv_step.  Attention is the
 * frame-wise causal one of Sec. 3.1 Eq. 1: a query of the chunk's frame a sees the cache as it was before
 * the call and the chunk's frames 0..a at input precision, nothing of the frames after its own.  The cache is
 * then updated once with the whole chunk as the current tokens of Sec. 3.2: T_current = n_frames * n,
 * k = L_max - T_first - T_current, the pooled query of Eq. 2-3 taken over the rows of all the chunk's frames;
 * the chunk's keys and values are quantised by Eq. 7-9 as in kv_step.  n_frames = 1 is kv_step.
 * KV_E_RANGE for n_frames outside [1, max_frames_per_step]; KV_E_INVAL with KV_PRUNE_THEN_ATTEND and
 * n_frames > 1. */
int kv_step_frames(kv_handle* h, int32_t stream, int32_t layer, int32_t n_frames, const void* q, const void* k,
                   const void* v, int64_t tok_stride, int64_t head_stride, void* out, void* hip_stream);

/* kv_step for callers that cannot allocate device memory or let a library do so around the call:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same results as kv_step (same kernels, same cache update), but the attention
 * kernel's key-range splits leave their partial results in a static device array of
 * KV_STATIC_SCRATCH_BYTES bytes that is part of the library's code object (each GPU the library
 * runs on holds its own copy until the process ends) instead of in the buffers kv_init
 * allocated, and the call makes no hipMalloc / hipFree / event-creation call of its own (launch
 * timing of kv_set_timing is not recorded for it).  Fewer splits are used when the array holds
 * fewer than kv_step would choose; KV_E_RANGE, with nothing launched, when the partial results
 * of two splits, 2 * n_heads * (tokens_per_frame rounded up to the query tiling) * 264 bytes,
 * exceed the array.  Every call on a GPU shares that GPU's array: nothing in it has to start at
 * zero (each call overwrites what it reads), but two calls that overlap in time on one GPU,
 * from any handles or streams, race on it; order them on one stream. */
#define KV_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
int kv_step_static(kv_handle* h, int32_t stream, int32_t layer, const void* q, const void* k, const void* v,
                   int64_t tok_stride, int64_t head_stride, void* out, void* hip_stream);

/* The same for n_items distinct caches in one set of launches.  Sec. 3.1 gives every layer
 * its own cache (the layer superscript of Eq. 1) and Sec. 3.2 / 3.3 prune and quantise each
 * layer's cache from that layer's own queries and keys, so the caches of one call are
 * independent: streams of different videos, or the layers of a synthetic stack whose inputs
 * do not depend on each other.  items: host array of n_items records (a cache may appear
 * once); strides as in kv_step, shared by all items.  More than 48 items are issued as
 * several launch sets.  KV_E_INVAL / KV_E_RANGE before anything is launched. */
int kv_step_batched(kv_handle* h, int32_t n_items, const kv_step_item* items, int64_t tok_stride,
                    int64_t head_stride, void* hip_stream);

/* Counters and footprint.  Sec. 3.2 bounds every cache by L_max (cache_len_max never
 * exceeds budget_tokens; tokens_dropped_total counts what the top-k of Sec. 3.2 removed),
 * and Sec. 3.3's codes and (s, z) are what bytes_live_per_cache adds up, the figure behind
 * the paper's memory comparison (Sec. 4, efficiency analysis).  stats: host, overwritten.
 * Synchronises the device. */
int kv_stats(kv_handle* h, kv_stats_t* stats);

/* Copy one cache to host buffers: the stored state of Sec. 3.3 (codes of Eq. 7, scales and
 * zero-points of Eq. 8, keys grouped per channel and values per token as in Eq. 9), the token
 * ids in cache order, and the last step's keep set and importance scores (Sec. 3.2, Eq. 6).
 * Codes are unpacked to one per byte.  Used by parity checks and as a checkpoint.
 * Synchronises the device.  bufs: host struct of host pointers, capacity_tokens set by the
 * caller; KV_E_RANGE if it is below the cache length. */
int kv_export(kv_handle* h, int32_t stream, int32_t layer, kv_export_t* bufs);

/* Frames of another size for one stream: Sec. 4 feeds images with a maximum edge of 518 pixels, so the token
 * count n = 1 + R + N of a frame follows the video's aspect ratio (518 x 392 gives 1041, 518 x 294 gives 782) and
 * is a property of the stream.  tokens_per_frame: n of this stream, n_special <= n <= kv_config.tokens_per_frame
 * (which sizes every buffer).  Every quantity of Sec. 3.2 follows the stream's n: T_first = T_current = n,
 * k = L_max - 2 n, N_pooled = n_special + ceil((n - n_special) / g).  Allowed only while the stream's caches are
 * empty (KV_E_STATE otherwise; kv_reset first).  A kv_step_batched call carries streams of one frame size
 * (KV_E_INVAL otherwise).  Host bookkeeping only. */
int kv_set_stream_tokens(kv_handle* h, int32_t stream, int32_t tokens_per_frame);

/* Forget the contents of one cache (stream, layer), or of all with stream = layer = -1: the
 * next frame is again the first frame of its stream, the one Sec. 3.2 never prunes.  Host
 * bookkeeping only; the caller orders it after the steps already enqueued on that cache. */
int kv_reset(kv_handle* h, int32_t stream, int32_t layer);

/* Load a cache from host buffers laid out as kv_export writes them (the checkpoint of a
 * stream: Sec. 3.2 bounds the state by L_max tokens, so this is all a stream needs to resume).
 * bufs: host; cache_len, frames_seen, ids, k_codes, k_scale, k_zero, v_codes, v_scale and
 * v_zero must be set, with cache_len = min(frames_seen * tokens_per_frame, budget_tokens) and
 * every code below 2^bits; last_keep and last_scores are ignored.  Waits for the device, then
 * replaces the cache of (stream, layer); the next kv_step continues the stream exactly as the
 * exporting handle would have.  KV_E_STATE in KV_UNCOMPRESSED_BF16 mode, KV_E_INVAL / KV_E_RANGE
 * for inconsistent buffers (the cache is then left as it was). */
int kv_import(kv_handle* h, int32_t stream, int32_t layer, const kv_export_t* bufs);

/* Free everything.  NULL is allowed. */
void kv_destroy(kv_handle* h);

/* Text of the last error on this handle (or of the last failed kv_init when h is NULL).
 * The string is owned by the library and valid until the next call. */
const char* kv_last_error(kv_handle* h);

/* Launch classes of a step, for kv_set_timing / kv_read_timing. */
enum kv_kernel_id {
  KV_K_ATTENTION = 0, /* fused de-quantise + attention (Eq. 1, Eq. 10)          */
  KV_K_COMBINE = 1,   /* merge of the split-KV partial results                   */
  KV_K_POOL = 2,      /* pooled query (Eq. 2-3 and the row mean of Eq. 6)        */
  KV_K_SCORE = 3,     /* per-head q~ . K~ over the cached tokens (Eq. 4-5)       */
  KV_K_SELECT = 4,    /* head sum, top-k, keep list                              */
  KV_K_REBUILD_K = 5, /* compaction + per-channel key (re)quantisation (Eq. 7-9) */
  KV_K_REBUILD_V = 6, /* value carry / per-token quantisation, token ids         */
  KV_K_COUNT = 7
};

/* Measurement aid: while bit (1 << id) of kernel_mask is set, every launch of that class
 * is bracketed by HIP events recorded on the stream it runs on.  kv_read_timing waits
 * for the recorded events, writes per class the summed duration in milliseconds and the
 * number of launches (host arrays of KV_K_COUNT entries) and clears the record. */
int kv_set_timing(kv_handle* h, uint32_t kernel_mask);
int kv_read_timing(kv_handle* h, float* total_ms, int32_t* launches);

/* Tuning knobs (not needed for correct results):
 *   "attention_splits"            0 = choose automatically, 1..16 = key-range splits (never more than the
 *                                 partial-result buffers, sized in kv_init for the automatic choice, hold)
 *   "attention_target_workgroups" workgroups the automatic choice aims for
 *   "timing_every"                n >= 1 (default 1): kv_set_timing brackets the launches of every n-th
 *                                 step call only; the event pairs cost a few microseconds of stream
 *                                 time each, so a benchmark samples them rather than paying them per step
 *   "debug_checks"                1: every step first scans q, k and v for infinities and NaNs
 *                                 and reports them through kv_stats (nonfinite_flag); 0 (default)
 *   "overlap_update"              1 (default): when attention alone cannot fill the chip (one or
 *                                 a few caches per call), scoring, pruning and re-quantisation
 *                                 run on a second stream of the library next to attention,
 *                                 joined back into hip_stream before kv_step returns (slot
 *                                 layout: pooling, scoring and selection do; its writers always
 *                                 follow attention); 2: the same at any launch size; 0:
 *                                 everything in order on hip_stream */
int kv_set_option(kv_handle* h, const char* name, int64_t value);

/* Machine probes (measurement aids, no handle needed; they allocate and free their own
 * device buffers and wait for their launches before returning).
 *   kv_probe_mfma_bf16: `repeats` launches of a register-resident loop of `iters` x 4 bf16
 *     32x32x16 matrix instructions per wave, eight waves on every compute unit, after one warm-up
 *     launch; writes the mean rate in TFLOP/s to *tflops (host).  This is the matrix-core rate the machine sustains under
 *     its power limit, the ceiling beside the published peak that Eq. 1's kernel is quoted against.
 *   kv_probe_copy: `repeats` streaming device-to-device copies of `bytes` bytes (multiple of 16,
 *     4 KiB .. 16 GiB) after one warm-up copy; writes the mean rate in GB/s (bytes read + bytes written) to
 *     *gbytes_per_s (host).  Also the known-size launch that HBM byte counters are scaled by.
 * Both return KV_OK or a negative kv_status. */
int kv_probe_mfma_bf16(int32_t iters, int32_t repeats, void* hip_stream, double* tflops);
int kv_probe_copy(int64_t bytes, int32_t repeats, void* hip_stream, double* gbytes_per_s);

#ifdef __cplusplus
}
#endif
#endif /* KVX_H */
