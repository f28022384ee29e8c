/*
 * buzz.h -- C ABI of the MI355X (gfx950) BUZZ sparse-KV-cache decode library.
 *
 * BUZZ (arxiv 2410.23079) keeps, per attention head, a bounded KV cache made of
 *   [ k attention-sink tokens | segmented heavy hitters ("old") | buffered new tokens | w window tokens ]
 * (Sec. 3.3, Fig. 3).  Every decode step appends the new key/value, attends over
 * all retained rows, and adds the attention probabilities to each row's
 * accumulated score; once T tokens have left the window, the "beehive"
 * eviction cuts them into segments of s, keeps the top-scoring row(s) of each
 * segment, interval-samples the older survivors with stride s^ and packs
 * the cache (Alg. 1, Alg. 2).
 *
 * General conventions
 *   - One handle = one layer's cache for `batch` sequences of equal length.
 *     (batch, kv-head) pairs are independent caches (Sec. 3.1 treats one head).
 *   - All tensor arguments are DEVICE pointers unless a comment says "host".
 *     They are borrowed until the work enqueued by the call has completed on
 *     the given stream; nothing is copied to or from the host.
 *   - Every call only enqueues kernels on `hip_stream` (a hipStream_t cast to
 *     void*, NULL = the default stream) and returns without synchronising.
 *     All sizes (rows retained, survivors, offsets) are functions of the
 *     configuration and the call history alone, so the host never reads back.
 *     One exception: the first buzz_prefill of a process on a GPU waits once
 *     for a short probe launch on `hip_stream` (see buzz_prefill).
 *   - Returns BUZZ_OK (0) or a negative buzz_status.  Arguments are validated
 *     before anything is enqueued: a failed call leaves the cache unchanged.
 *     Every call also checks, before it enqueues anything, that the rows it is
 *     about to touch lie inside the regions of the workspace layout, and
 *     returns BUZZ_ECAPACITY otherwise: no kernel is handed a row the
 *     workspace does not have.
 *   - A handle must not be used from two threads at once.
 *   - q, k, v share `kv_dtype`; attention output and scores are fp32.
 */
#ifndef BUZZ_H
#define BUZZ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct buzz_cache buzz_cache_t; /* opaque, host memory owned by the library */

typedef enum buzz_status {
    BUZZ_OK = 0,
    BUZZ_EINVAL = -1,       /* bad argument or configuration */
    BUZZ_ECAPACITY = -2,    /* the call would overflow the cache or the workspace */
    BUZZ_ESTATE = -3,       /* call not valid in the handle's current state */
    BUZZ_EHIP = -4,         /* a HIP runtime call or kernel launch failed */
    BUZZ_EUNSUPPORTED = -5  /* valid request the kernels do not cover (shape, dtype) */
} buzz_status;

enum { BUZZ_FP32 = 0, BUZZ_FP16 = 1, BUZZ_BF16 = 2 };

enum {
    BUZZ_FLAG_AUTO_EVICT = 1u, /* buzz_decode_step evicts by itself when T new tokens are buffered */
    BUZZ_FLAG_DRY_RUN = 2u,    /* do all host bookkeeping and validation but launch nothing (no GPU needed) */
    /* How the decode kernel reads K and V.  Default (neither flag): streaming loads when one step of this
       cache reads more than the GPU's 256 MB last-level cache, cached loads otherwise.  A caller that runs many
       layers (so that nothing survives in cache between two steps of one layer) should set STREAMING. */
    BUZZ_FLAG_STREAMING = 4u,
    BUZZ_FLAG_CACHED = 8u,
    /* Log-n scaled attention (Sec. 3.5): the softmax scale of a query is multiplied by log(n)/log(512),
       n = number of tokens it sees, itself included (prompt queries: their position + 1; decode step: tokens
       seen so far + 1).  The library tracks n. */
    BUZZ_FLAG_LOG_N = 16u,
    /* T bounds old + new tokens together instead of the new tokens alone: eviction fires when
       n_old + new_count reaches T.  This is how the proof of the Parameter Estimation theorem reads T; meant
       for old_stride > 1.  The old region then holds at most T rows, and a prefill keeps sampling until its
       survivors fit T rows (Remark 2 gives the size of that container) unless `capacity` says otherwise. */
    BUZZ_FLAG_THRESHOLD_TOTAL = 32u,
    /* Bitwise reproducible decode steps.  By default the waves of a decode block claim their next tile of
       cache rows from a shared counter, so which wave sums which rows depends on timing and the outputs and
       scores of two identical runs may differ in the last bits (always within the stated tolerances).  With
       this flag the assignment is fixed; measured cost: up to 5% of the step. */
    BUZZ_FLAG_DETERMINISTIC = 64u,
    /* Ablation "no local max" (Sec. 4.3): new tokens are interval-sampled like old ones -- the first `keep`
       rows of every segment survive whatever their scores.  (The other ablation of that section, swapped
       strides, needs no flag: segment = s^ and old_stride = s.) */
    BUZZ_FLAG_INTERVAL_NEW = 128u,
    /* Where the key range of a (batch, kv-head) pair is split over several blocks and the pairs divide evenly
       over the GPU's 8 dies, the blocks of a pair are placed on one die and exchange their partial results
       through that die's L2.  With this flag they always exchange them through device memory instead (the
       path taken anyway for other shapes).  Results are the same; meant for comparison. */
    BUZZ_FLAG_DEVICE_MERGE = 256u,
    /* H2O-style baseline (Sec. 4.1: greedy selection by accumulated attention score, no segmentation): at every
       eviction ALL rows between sink and window, old and new alike, form one segment of which the `keep`
       highest-scoring rows survive (ties to the lowest index), so the cache holds sink + keep + window rows plus
       up to T buffered ones.  `segment` and `old_stride` are ignored.  Not combinable with THRESHOLD_TOTAL or
       INTERVAL_NEW. */
    BUZZ_FLAG_GLOBAL_TOPK = 512u
};

/* Symbols follow the paper's notation table (Sec. 3.3). */
typedef struct buzz_config {
    int32_t batch;        /* sequences per call */
    int32_t n_q_heads;    /* query heads; 1 to 8 times n_kv_heads */
    int32_t n_kv_heads;   /* key/value heads; the score of a row is summed over its query group */
    int32_t head_dim;     /* d of eq. 3; 64, 128 or 256 */
    int32_t kv_dtype;     /* BUZZ_FP32 / BUZZ_FP16 / BUZZ_BF16 */
    int32_t sink;         /* k : first tokens always kept ("attention sink") */
    int32_t window;       /* w : most recent tokens always kept ("sliding window") */
    int32_t segment;      /* s : stride of the segments ("hives") for new tokens; >= 1 */
    int32_t keep;         /* rows kept per segment; the paper keeps 1; 0 keeps none (sink + window only) */
    int32_t evict_every;  /* T : number of tokens buffered outside the window before one eviction */
    int32_t old_stride;   /* s^: interval-sampling stride for old tokens; 0 => floor((s+1)/2) as in the paper,
                                 1 => survivors persist */
    uint32_t flags;       /* BUZZ_FLAG_* */
    int64_t max_context;  /* upper bound on prompt + decoded tokens; sizes the workspace */
    int64_t capacity;     /* retained rows per head the cache may hold, = sink + old capacity + window + T;
                             0 => derived from max_context so that it can never overflow.  With s^ > 1 a
                             prefill keeps sampling until the rows fit this capacity (Remark 2). */
    float softmax_scale;  /* 0 => 1/sqrt(head_dim) (eq. 3); the log-n variant of Sec. 3.5 passes
                             log(n)/log(512)/sqrt(head_dim) */
    int32_t reserved;     /* must be 0 */
} buzz_config_t;

/*
 * Bytes of device workspace a cache with this configuration needs (K and V
 * arenas, fp32 scores, int32 positions, split-softmax partials, logits,
 * prefill scratch).  `bytes` is a host pointer.
 * Errors: BUZZ_EINVAL (null pointer, inconsistent configuration),
 *         BUZZ_EUNSUPPORTED (head_dim / dtype / group size without a kernel).
 */
int buzz_workspace_bytes(const buzz_config_t* cfg, size_t* bytes);

/*
 * Create a cache over a caller-owned device workspace of at least
 * buzz_workspace_bytes() bytes, 256-byte aligned.  The workspace must outlive
 * the handle; the library never frees it.  Touches no device memory.
 * Errors: as buzz_workspace_bytes, plus BUZZ_ECAPACITY if `bytes` is too small.
 */
int buzz_cache_create(const buzz_config_t* cfg, void* dev_workspace, size_t bytes, buzz_cache_t** out);

/*
 * Load a prompt (eq. 1 gives K, V; the caller did the projections) and bring
 * the cache to its bounded form (Remark 2).
 *   k, v        [batch][n_kv_heads][n_prompt][head_dim], kv_dtype
 *   q_obs       [batch][n_q_heads][n_obs][head_dim]: queries of the last n_obs
 *               prompt positions (query t sits at position n_prompt-n_obs+t and
 *               attends causally); their attention probabilities initialise the
 *               accumulated scores.  NULL with n_obs = 0 for none.
 *   init_score  [batch][n_kv_heads][n_prompt] fp32 starting scores, or NULL for zeros.
 * If at least T prompt tokens lie between sink and window they are sampled at
 * once (all of them count as "new", Alg. 1 with n_old = 0); with s^ > 1 and an
 * explicit capacity the survivors are interval-sampled again until they fit.
 * Resets the handle: may be called again to start a new sequence.
 * The first call of a process on a GPU also runs a probe launch on `hip_stream`
 * and waits for it (tens of microseconds, once): it records which die every
 * block of a small grid ran on, which decides whether decode steps may merge
 * the splits of a (batch, kv-head) pair through one die's L2 (see
 * BUZZ_FLAG_DEVICE_MERGE).  The probe uses the library's static device scratch
 * array, like buzz_decode_step_static: do not run it concurrently with such a
 * call on another stream.
 * Errors: BUZZ_EINVAL, BUZZ_ECAPACITY (n_prompt > max_context, survivors do
 *         not fit), BUZZ_EHIP.
 */
int buzz_prefill(buzz_cache_t* cache, const void* k, const void* v, int64_t n_prompt,
                 const void* q_obs, int64_t n_obs, const float* init_score, void* hip_stream);

/*
 * One decode step (eq. 2, eq. 3 / eq. 5, score accumulation):
 *   append k_new, v_new as a new row (score 0, position = tokens seen so far);
 *   out[g] = softmax(scale * q[g] . K^T) V over every retained row, the new one included;
 *   score[row] += sum over the query heads g of the row's kv head of the probabilities;
 *   with BUZZ_FLAG_AUTO_EVICT, run buzz_evict when T new tokens are buffered (Alg. 1).
 *   q      [batch][n_q_heads][head_dim], kv_dtype
 *   k_new  [batch][n_kv_heads][head_dim], kv_dtype       v_new likewise
 *   out    [batch][n_q_heads][head_dim], fp32
 * Errors: BUZZ_EINVAL, BUZZ_ESTATE (no prefill yet), BUZZ_ECAPACITY (max_context
 *         reached; window + buffer full because eviction was not called; or, with
 *         BUZZ_FLAG_AUTO_EVICT, the eviction this step would end with leaves more
 *         survivors than an explicit `capacity` has room for -- checked before the
 *         step is enqueued, so the token is not appended), BUZZ_EHIP.
 */
int buzz_decode_step(buzz_cache_t* cache, const void* q, const void* k_new, const void* v_new,
                     float* out, void* hip_stream);

/*
 * buzz_decode_step for callers that cannot allocate device memory or let a library do so on their
 * behalf: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same results and same errors as buzz_decode_step; the difference is where the scratch
 * of the split softmax lives (one arrival counter per (batch, kv-head) and one (max, sum, partial
 * output) record per key-range split and query head): not in the caller's workspace but in an
 * array inside the library's device image, 8.25 MiB per GPU, held until the process ends.  The call
 * reaches no hipMalloc / hipFree and no allocating library routine, and clears the counters it uses
 * with a small kernel (no memset node), whatever the previous call left there.
 * Additional errors: BUZZ_ECAPACITY when batch * n_kv_heads * splits * group * (head_dim + 2) * 4
 * bytes exceed 8 MiB (the split count follows from the shape as in buzz_decode_step;
 * buzz_cache_set_splits lowers it); BUZZ_ESTATE while buzz_cache_profile is on (its events are
 * created per launch).
 * Every call on one GPU shares that GPU's array: calls whose kernels may overlap on one GPU (two
 * streams, two threads) race, whichever caches they are for; calls on one stream are safe.
 */
int buzz_decode_step_static(buzz_cache_t* cache, const void* q, const void* k_new, const void* v_new,
                            float* out, void* hip_stream);

/*
 * One eviction (the eviction branch of Alg. 1, with Alg. 2): old rows are interval-sampled
 * with stride s^, the rows between old region and window are cut into
 * segments of s from their start (the last may be ragged) and the top
 * min(keep, len) of each segment under (score descending, index ascending;
 * NaN lowest) survive in index order; K, V, score and position of the survivors
 * are packed behind the sink.  Does nothing while the cache holds no more than
 * sink + window rows (Remark 1).  May be called at any time.
 * Errors: BUZZ_EINVAL, BUZZ_ESTATE, BUZZ_ECAPACITY (survivors exceed the old
 *         capacity; only possible with many manual partial evictions), BUZZ_EHIP.
 */
int buzz_evict(buzz_cache_t* cache, void* hip_stream);

/* Free the host handle (never the workspace).  NULL is allowed. Errors: BUZZ_EINVAL on a stale handle. */
int buzz_cache_destroy(buzz_cache_t* cache);

/*
 * Current sizes (host pointers, any may be NULL): n rows retained, n_old rows
 * in the old region, new_count rows buffered between old region and window.
 */
int buzz_cache_len(const buzz_cache_t* cache, int64_t* n, int64_t* n_old, int64_t* new_count);

/*
 * Copy the retained rows out in cache order [sink | old | new | window]:
 *   k, v   [batch][n_kv_heads][n][head_dim] kv_dtype;  score [batch][n_kv_heads][n] fp32;
 *   pos    [batch][n_kv_heads][n] int32 original token index.   Any may be NULL.
 * Errors: BUZZ_EINVAL, BUZZ_ESTATE, BUZZ_EHIP.
 */
int buzz_cache_export(buzz_cache_t* cache, void* k, void* v, float* score, int32_t* pos, void* hip_stream);

/*
 * The inverse of buzz_cache_export (checkpoint / resume): load `n` retained rows per (batch, kv-head), given in
 * cache order [sink | old | new | window] with the layouts buzz_cache_export writes, of which `n_old` are old
 * rows, into a cache of the same configuration; `tokens_seen` = prompt + decoded tokens so far (it numbers the
 * next token and feeds the log-n scale).  Replaces whatever the handle held, like buzz_prefill; decode steps
 * continue from there exactly as they would have on the exporting cache (same rows, scores, sizes; sums may
 * differ in the last bits because the rows sit at other places of the ring).
 * Errors: BUZZ_EINVAL (null pointers, n_old > n, tokens_seen < n, old rows without a full sink),
 *         BUZZ_ECAPACITY (more old rows, buffered rows or tokens than the cache was sized for), BUZZ_EHIP.
 */
int buzz_cache_import(buzz_cache_t* cache, const void* k, const void* v, const float* score, const int32_t* pos,
                      int64_t n, int64_t n_old, int64_t tokens_seen, void* hip_stream);

/*
 * Tuning knob: number of key-range splits per (batch, kv-head) used by the
 * split softmax of the decode kernel; 0 restores the automatic choice.
 * Errors: BUZZ_EINVAL (negative, or above what the workspace was sized for).
 */
int buzz_cache_set_splits(buzz_cache_t* cache, int32_t n_splits);

/*
 * Failure-handling aid.  The die-local merge (see BUZZ_FLAG_DEVICE_MERGE) checks in every decode step that
 * each block runs on the die the placement probe recorded for its launch-order number mod 8 (`die_map`:
 * 4 bits per number), and turns the attention output of a (batch, kv-head) pair whose blocks do not into NaN.
 * This call replaces the record the check compares with for one cache, so that a test can make the check
 * fail from the host (every kernel still runs to its end); a negative value restores the probe's record.
 * No effect where the die-local merge is not used.  Errors: BUZZ_EINVAL.
 */
int buzz_cache_override_die_map(buzz_cache_t* cache, int64_t die_map);

/*
 * Benchmark aid: per-kernel device time measured with HIP events recorded on
 * the stream each kernel is launched on.  buzz_cache_profile(cache, 1) clears
 * the counters and starts recording (every launch then carries a start and a
 * stop event that take the kernel's own begin / end timestamps; use a separate
 * pass for end-to-end timing);
 * buzz_cache_profile(cache, 0) stops.  buzz_cache_profile_read waits for the
 * recorded events, then fills `out` (host pointer).
 * Errors: BUZZ_EINVAL, BUZZ_EHIP.
 */
typedef struct buzz_profile {
    int64_t attn_launches;     /* split decode-attention kernel */
    int64_t epilogue_launches; /* score flush kernel (pending score update applied before an eviction or export) */
    int64_t evictions;         /* whole evictions (all their kernels) */
    double attn_ms, epilogue_ms, evict_ms; /* summed device time */
    double attn_row_bytes;     /* sum over attn launches of units * rows * 2 * head_dim * sizeof(element) */
} buzz_profile_t;
int buzz_cache_profile(buzz_cache_t* cache, int enable);
int buzz_cache_profile_read(buzz_cache_t* cache, buzz_profile_t* out);

/*
 * Benchmark aid: a plain 16-byte-per-thread device-to-device copy of `bytes` bytes (multiple of 16,
 * both pointers 16-byte aligned, ranges must not overlap).  A copy of known size gives the factor by
 * which a hardware byte counter (FETCH_SIZE, WRITE_SIZE) has to be scaled on this machine.
 * Errors: BUZZ_EINVAL, BUZZ_EHIP.
 */
int buzz_bench_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/*
 * The eviction threshold the Parameter Estimation theorem (Sec. 3.4) recommends for stride s and window w
 * under BUZZ_FLAG_THRESHOLD_TOTAL: T = w (s^2 + 1)/(s + 1) for odd s, w (s - 1) for even s, rounded to the
 * nearest integer and at least 1.  Returns 0 for s < 1 or w < 0.  Pure host arithmetic.
 */
int64_t buzz_suggest_threshold(int32_t segment, int32_t window);

/* Static description of a status code (host string, never NULL). */
const char* buzz_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* BUZZ_H */
