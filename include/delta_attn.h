/*
 * delta_attn.h - C ABI of the MI355X (gfx950) hybrid delta attention library.
 *
 * One attention layer of DeltaLLM (arXiv 2507.19608): keys are turned into a
 * thresholded delta matrix (Sec. II-C Eq. 2-3, applied to K from its first row,
 * Sec. III-A strategy 3); attention scores are exact inside a local window and
 * rebuilt incrementally from the delta matrix outside it (Sec. III-B, Eq. 4);
 * softmax and PV follow Eq. 1.  Prefill and decode (Sec. III-C) are covered.
 *
 * Conventions
 *   - Every tensor pointer is DEVICE memory owned by the caller, contiguous,
 *     last dimension fastest.  The library owns only da_cache objects.
 *   - hip_stream is a hipStream_t passed as void* (NULL = default stream).  All
 *     work is enqueued on it; only delta_attn_sparsity synchronises.
 *   - Every entry returns a da_status.  Arguments, workspace and cache state are checked before anything is
 *     enqueued: after DA_ERR_INVALID_ARG / UNSUPPORTED / WORKSPACE / STATE no buffer has been touched.  After
 *     DA_ERR_HIP (a launch or copy failed part-way) the outputs, and a cache that was passed, are undefined.
 *   - Grouped-query attention: n_q_heads % n_kv_heads == 0; query head h reads
 *     KV head h / (n_q_heads / n_kv_heads).  There is one delta matrix, mask and
 *     nnz per (batch, KV head).
 *   - Threshold decision: fabsf((float)k - (float)held) > theta in IEEE binary32,
 *     strict inequality (Eq. 2); the first row of a sequence is the basis and is
 *     kept whole.  NaN keys never fire (not checked).
 */
#ifndef DELTA_ATTN_H
#define DELTA_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DA_OK = 0,
    DA_ERR_INVALID_ARG = 1,   /* null pointer, non-positive size, Hq % Hkv != 0, window < 1, theta < 0 or NaN */
    DA_ERR_UNSUPPORTED = 2,   /* head_dim not a multiple of 32 or > 256, unknown dtype or mode */
    DA_ERR_WORKSPACE = 3,     /* workspace pointer null, not 256-byte aligned, or smaller than *_workspace_bytes() */
    DA_ERR_STATE = 4,         /* cache full, prefill into a non-empty cache, cache/params mismatch (shape, dtype,
                                 theta, or a score scale other than the cache's) */
    DA_ERR_HIP = 5            /* a HIP runtime call failed */
} da_status;

typedef enum { DA_F32 = 0, DA_BF16 = 1 } da_dtype;

/* How scores outside the window are produced.  Both give the same real-number result.
 *   DA_SCORE_GATHER  Eq. 4 as written: a running score per query row, updated per key
 *                    column with only the surviving (channel, delta) entries.
 *   DA_SCORE_REBASE  the telescoped form of Eq. 4: sum_{u<=j} dk(u) = k_hat(j), so the
 *                    score is the dense product q . k_hat(j) (no multiply is skipped). */
typedef enum { DA_SCORE_GATHER = 0, DA_SCORE_REBASE = 1 } da_score_mode;

/* Shape of the prefill's exact region (Sec. III-B).
 *   DA_WINDOW_BLOCK    squares of side W along the diagonal: (i, j) exact iff j <= i and
 *                      floor(i / W) == floor(j / W) - the prefill stage as the paper draws it and
 *                      the region whose area Eq. 6 uses.
 *   DA_WINDOW_SLIDING  a band: (i, j) exact iff 0 <= i - j < W - the decode stage's rule applied to
 *                      every prefill row, so prefill row t equals the decode step at position t with
 *                      decode_window W. */
typedef enum { DA_WINDOW_BLOCK = 0, DA_WINDOW_SLIDING = 1 } da_window_mode;

typedef struct {
    int32_t batch, n_q_heads, n_kv_heads, head_dim, seq_len;
    int32_t window;     /* W >= 1: side of the exact squares on the diagonal / width of the band;
                           W >= seq_len gives dense causal attention */
    float theta;        /* >= 0 (may be +inf) */
    float scale;        /* score scale; 0 selects 1/sqrt(head_dim) (Eq. 1) */
    int32_t dtype;      /* da_dtype of Q, K, V, O */
    int32_t score_mode; /* da_score_mode */
    int32_t window_mode; /* da_window_mode */
} da_prefill_params;

typedef struct da_cache da_cache;   /* decode-time cache (Sec. III-C), opaque */

const char *delta_attn_version(void);
const char *delta_attn_status_string(da_status s);
/* Text of the last DA_ERR_HIP on the calling thread: "<stage>: <hip error name> (<description>)" (also set by
 * delta_attn_prefill_noalloc when the params need more scratch than it has); empty if none occurred.  Points to
 * thread-local storage owned by the library. */
const char *delta_attn_last_error(void);

/*
 * Per-stage timing for benchmarks.  While enabled, prefill and decode calls bracket each of their
 * kernels with HIP events on the call's own stream (at most 8192 brackets between reads).
 * delta_attn_stage_timing_read, called after the caller has synchronised those streams, sums the
 * elapsed milliseconds and the number of launches per stage since the previous read and returns
 * the number of brackets read (-1 on a null pointer).  Both arrays have DA_NUM_STAGES entries.
 * A benchmarking aid, off by default: the switch and the event pool are process-wide (guarded by a mutex), so
 * with timing on, calls from several threads are bracketed into one common pool.
 */
enum { DA_STAGE_SCAN = 0, DA_STAGE_EMIT = 1, DA_STAGE_ATTN = 2, DA_STAGE_CACHE_FILL = 3,
       DA_STAGE_APPEND = 4, DA_STAGE_CHUNK = 5, DA_STAGE_COMBINE = 6, DA_NUM_STAGES = 7 };
void delta_attn_stage_timing_enable(int32_t on);
int32_t delta_attn_stage_timing_read(double *ms_per_stage, int32_t *calls_per_stage);

/* Eq. 5: min(floor(gamma * n), w_max), clamped to >= 1.  Host only. */
int32_t delta_attn_window_from_gamma(int32_t n, double gamma, int32_t w_max);

/* Bytes of device scratch delta_attn_prefill / delta_attn_delta_scan need for these params
 * (0 if the params are invalid). */
size_t delta_attn_prefill_workspace_bytes(const da_prefill_params *p);

/* Bytes of device scratch delta_attn_delta_scan needs (0 if the params are invalid). */
size_t delta_attn_delta_scan_workspace_bytes(const da_prefill_params *p);

/*
 * Delta matrix only (Eq. 2-3 on K; Sec. III-A).  Uses batch, n_kv_heads, head_dim, seq_len,
 * theta, dtype of p.
 *   K         [B, Hkv, n, d]   in
 *   mask_bits [B, Hkv, n, d/32] uint32 out: bit (c % 32) of word c/32 is 1 iff delta entry
 *             (t, c) is kept; row 0 is all ones
 *   nnz       [B, Hkv] uint64 out: number of set mask bits
 *   k_hat     [B, Hkv, n, d] out or NULL: reference keys after each row (Eq. 3), dtype of K
 *   workspace device scratch of at least delta_attn_delta_scan_workspace_bytes(p)
 */
da_status delta_attn_delta_scan(const da_prefill_params *p, const void *K, uint32_t *mask_bits,
                                uint64_t *nnz, void *k_hat, void *workspace, size_t workspace_bytes,
                                void *hip_stream);

/*
 * Prefill (Sec. III-B prefill stage + Sec. III-C): builds the delta matrix of K, then for every
 * query row i and key j <= i the score is q_i.k_j if floor(i/W) == floor(j/W), else the Eq. 4
 * running score; scaled, softmaxed over j <= i, multiplied with V (Eq. 1).
 *   Q, O      [B, Hq, n, d];  K, V [B, Hkv, n, d]
 *   mask_bits, nnz as in delta_attn_delta_scan
 *   cache     NULL, or an EMPTY cache with matching batch/heads/head_dim/theta/dtype and
 *             max_seq >= n: left holding the n rows, ready for delta_attn_decode at position n
 *   workspace device scratch of at least delta_attn_prefill_workspace_bytes(p), 256-byte aligned
 */
da_status delta_attn_prefill(const da_prefill_params *p, const void *Q, const void *K, const void *V,
                             void *O, uint32_t *mask_bits, uint64_t *nnz, da_cache *cache,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * delta_attn_prefill for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation and same kernels as
 * delta_attn_prefill without a cache, masks and nnz bit-identical; outputs bit-identical too unless delta_attn_prefill
 * cuts a small launch along the keys (several work groups per row tile, merged afterwards) and the built-in buffer has
 * no room for the parts: this call then runs uncut and the outputs differ in rounding order only.  The scratch is a
 * buffer of DA_NOALLOC_SCRATCH_BYTES built into the library's device image (one copy per GPU, held until the process
 * ends), so the call itself allocates nothing.
 *   - Returns DA_ERR_WORKSPACE, with the two sizes in delta_attn_last_error(), when
 *     delta_attn_prefill_workspace_bytes(p) exceeds DA_NOALLOC_SCRATCH_BYTES (nothing has been enqueued then).
 *   - Every call on a GPU uses that GPU's one buffer: two calls whose kernels overlap in time on the same GPU (two
 *     streams, two threads) race.  Calls on one stream, or ordered by events, are safe; the buffer keeps the previous
 *     call's contents and no call depends on them.
 *   - The first call on a device looks the buffer's address up (hipGetSymbolAddress) and raises the kernels' LDS
 *     limits; make that call outside graph capture.
 */
#define DA_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
da_status delta_attn_prefill_noalloc(const da_prefill_params *p, const void *Q, const void *K, const void *V,
                                     void *O, uint32_t *mask_bits, uint64_t *nnz, void *hip_stream);

/*
 * Chunked prefill (Sec. III-C: the cache built so far is carried on): the m = p->seq_len rows of Q, K, V
 * are positions t0 .. t0 + m - 1 of a sequence whose first t0 rows the cache holds (t0 = cache length; 0
 * is allowed).  The delta rows of the new keys continue from the cache's reference key (Eq. 2-3), the new
 * query rows attend over all t0 + m keys with the window squares anchored at position 0 (or the band, by
 * p->window_mode), exactly as rows t0 .. t0 + m - 1 of one prefill over the whole sequence would, and the
 * new rows are appended to the cache.
 *   Q, O [B, Hq, m, d];  K, V [B, Hkv, m, d];  mask_bits [B, Hkv, m, d/32], nnz [B, Hkv]: the new rows only
 *   cache     bf16, head_dim 64 or 128, decode_window >= min(64, max_seq) (and >= min(p->window, t0 + m) unless the cache
 *             is empty: the exact scores against cached keys are taken from the cache's ring of raw keys;
 *             a decode_window above max_seq counts as max_seq),
 *             at most 32 query heads per KV head; otherwise DA_ERR_UNSUPPORTED
 *   workspace device scratch of at least delta_attn_prefill_append_workspace_bytes(p, cache) (0 if the arguments
 *             are invalid), 256-byte aligned; it depends on p->seq_len and (through the key split
 *             of launches that do not fill the chip) on the cache length at the time of the call
 * The cache keeps the sequence so far as the plain arrays the prefill kernels read (keys, reference keys, values in
 * two orders, mask rows, and in DA_SCORE_GATHER mode the entry lists and gather plans of all key columns), with
 * max_seq rows of room: about 8 * head_dim + 4 * head_dim / 32 bytes per (KV head, row), 16 * head_dim + 8 in
 * gather mode.  The first call on a cache allocates them (hipMalloc + hipMemset, released by
 * delta_attn_cache_destroy; DA_ERR_HIP if that fails; make that call outside graph capture); a call that follows
 * another such call, or delta_attn_cache_reset, then only adds its own rows.  After decode steps or a one-shot
 * delta_attn_prefill into the cache the arrays are rebuilt from the cache by the next call, at a cost proportional to
 * the cache length.
 */
size_t delta_attn_prefill_append_workspace_bytes(const da_prefill_params *p, const da_cache *cache);
da_status delta_attn_prefill_append(const da_prefill_params *p, const void *Q, const void *K, const void *V,
                                    void *O, uint32_t *mask_bits, uint64_t *nnz, da_cache *cache,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/* Decode cache: per (batch, KV head) the delta matrix in compact form (mask bits + surviving key
 * values), the reference key at the start of every 64 rows, the current reference key, a ring of
 * the last decode_window raw keys, and V (Sec. III-A last paragraph, Sec. III-C).  All sequences of
 * the batch advance together.  A cache may start empty (the first decoded row is then the basis
 * row) or be filled by delta_attn_prefill.  Allocates device memory on the current device; owned
 * by the library until delta_attn_cache_destroy. */
da_status delta_attn_cache_create(da_cache **out, int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                  int32_t head_dim, int32_t max_seq, int32_t decode_window, float theta,
                                  float scale, int32_t dtype);
da_status delta_attn_cache_destroy(da_cache *c);
da_status delta_attn_cache_reset(da_cache *c, void *hip_stream);   /* back to length 0 */
int64_t delta_attn_cache_length(const da_cache *c);                /* rows held, -1 if c is NULL */
const uint64_t *delta_attn_cache_nnz(const da_cache *c);           /* device [B, Hkv] uint64 */
/* mask bits of the cached rows: device [B, Hkv, max_seq, d/32] (rows >= length undefined) */
const uint32_t *delta_attn_cache_mask(const da_cache *c);
/* How a decode step on this cache is laid out over the GPU (Sec. III-B decode stage; results do not
 * depend on it).  bf16 caches with head_dim 64 / 128 and decode_window >= min(64, max_seq) split the cached rows of a
 * (batch, KV head) unit into chunks of 64 rows; a wave (head_dim 128: a pair of waves, 64 channels each) walks
 * `chunks per wave` consecutive chunks.
 *   merge_in_kernel  1: one work group per unit, its waves merge their partial results on chip (head_dim 64
 *                       only; at head_dim 128 the value is accepted and ignored);
 *                    0: one chunk walker per work group, partial results merged by a second launch;
 *                   -1: chosen per step from the unit count and the wave slots (default).
 *   wave_slots       resident waves the launch is sized for; 0 = derived from the device (default).
 * Other caches ignore the plan.  Returns DA_ERR_INVALID_ARG for NULL or values outside these ranges. */
da_status delta_attn_cache_set_launch_plan(da_cache *c, int32_t merge_in_kernel, int32_t wave_slots);

/*
 * One decode step at position t = cache length (Sec. III-B decode stage, Sec. III-C): appends
 * the delta row of k_new and v_new to the cache, then attends q_new over keys 0..t with exact
 * scores for the decode_window most recent keys (the new one included) and Eq. 4 scores for
 * older keys.  The cache length advances when the step has been enqueued without error (the call does not wait for
 * the GPU).
 *   q_new [B, Hq, d], k_new, v_new [B, Hkv, d] in;  o [B, Hq, d] out
 *   mask_row [B, Hkv, d/32] out or NULL: mask of the appended row
 */
da_status delta_attn_decode(da_cache *c, const void *q_new, const void *k_new, const void *v_new,
                            void *o, uint32_t *mask_row, void *hip_stream);

/* Eq. 6.  Reads nnz (device, [batch * n_kv_heads]) after synchronising the stream.
 *   s_m = 1 - sum(nnz) / (batch * n_kv_heads * rows * head_dim)
 *   s_c = s_m * (1 - min(window, rows) / rows) */
da_status delta_attn_sparsity(const uint64_t *nnz_dev, int32_t batch, int32_t n_kv_heads, int64_t rows,
                              int32_t head_dim, int32_t window, void *hip_stream, double *s_m,
                              double *s_c);

#ifdef __cplusplus
}
#endif
#endif /* DELTA_ATTN_H */
