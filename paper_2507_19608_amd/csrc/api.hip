// C ABI of the hybrid delta attention library: argument checks, workspace carving, launches.
#include <math.h>
#include <mutex>
#include <new>
#include <stdlib.h>
#include <string.h>

#include "../../include/delta_attn.h"
#include "cache.hpp"
#include "common.hpp"
#include "kernels.hpp"

using namespace da;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline size_t elt_size(int dtype) { return dtype == DA_F32 ? 4 : 2; }

struct WsLayout {
    size_t khat, chunk_out, ents, counts, nch8, plan, dense, vt, part, total;
    int ksplit;   // work groups per tile of the attention launch (prefill_mfma_ksplit); `part` holds their results
};

// what prefill_mfma_ksplit reads, for a prefill of p's rows behind `cached` rows
PrefillArgs split_args(const da_prefill_params *p, int64_t cached) {
    PrefillArgs a = {};
    a.dtype = p->dtype;
    a.B = p->batch;
    a.Hq = p->n_q_heads;
    a.Hkv = p->n_kv_heads;
    a.d = p->head_dim;
    a.n = (int)cached + p->seq_len;
    a.q_off = (int)cached;
    a.nq = p->seq_len;
    a.ksplit = 1;
    a.rebase = p->score_mode == DA_SCORE_REBASE;
    a.fused = cached == 0 && prefill_mfma_supported(a) && (int64_t)p->seq_len * p->head_dim <= kFusedMaxElems;
    return a;
}

da_status check_params(const da_prefill_params *p) {
    if (!p) return DA_ERR_INVALID_ARG;
    if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->head_dim < 1 || p->seq_len < 1)
        return DA_ERR_INVALID_ARG;
    if (p->n_q_heads % p->n_kv_heads != 0) return DA_ERR_INVALID_ARG;
    if (p->window < 1) return DA_ERR_INVALID_ARG;
    if (!(p->theta >= 0.f)) return DA_ERR_INVALID_ARG;          // also rejects NaN
    if (!(p->scale >= 0.f) || isinf(p->scale)) return DA_ERR_INVALID_ARG;
    if (p->head_dim % 32 != 0 || p->head_dim > 256) return DA_ERR_UNSUPPORTED;
    if (p->dtype != DA_F32 && p->dtype != DA_BF16) return DA_ERR_UNSUPPORTED;
    if (p->score_mode != DA_SCORE_GATHER && p->score_mode != DA_SCORE_REBASE) return DA_ERR_UNSUPPORTED;
    if (p->window_mode != DA_WINDOW_BLOCK && p->window_mode != DA_WINDOW_SLIDING) return DA_ERR_UNSUPPORTED;
    if ((int64_t)p->batch * p->n_q_heads > 65535 * 64) return DA_ERR_UNSUPPORTED;
    return DA_OK;
}

// split: cut the attention launch along the keys where that pays (more scratch); false: never
WsLayout layout(const da_prefill_params *p, bool split = true) {
    const size_t units = (size_t)p->batch * p->n_kv_heads;
    const size_t rows = units * (size_t)p->seq_len;
    WsLayout w;
    size_t off = 0;
    w.khat = off;
    off += align_up(rows * p->head_dim * elt_size(p->dtype));
    w.chunk_out = off;
    off += align_up(2 * units * (size_t)delta_scan_num_chunks(p->seq_len) * p->head_dim * elt_size(p->dtype));
    w.ents = off;
    off += align_up(rows * p->head_dim * 8);   // EntryChunk storage: 8 bytes per possible entry
    w.counts = off;
    off += align_up(rows * sizeof(uint32_t));
    w.nch8 = off;
    off += align_up(units * (size_t)prefill_mfma_n_pad(p->seq_len));
    w.plan = off;
    off += align_up(units * (size_t)prefill_mfma_n_pad(p->seq_len) * 2);   // 8 waves x 8 bytes per block of 32 columns
    w.dense = off;
    off += align_up(units * (size_t)(prefill_mfma_n_pad(p->seq_len) / 32) * 4);
    w.vt = off;
    off += align_up(units * (size_t)p->head_dim * prefill_mfma_n_pad(p->seq_len) * 2);
    const PrefillArgs a = split_args(p, 0);
    w.ksplit = split ? prefill_mfma_ksplit(a) : 1;
    w.part = off;
    off += align_up(prefill_mfma_part_bytes(a, w.ksplit));
    w.total = off;
    return w;
}

inline float score_scale(float scale, int d) { return resolved_scale(scale, d); }

da_status prefill_checked(const da_prefill_params *p, const WsLayout &w, const void *Q, const void *K, const void *V,
                          void *O, uint32_t *mask_bits, uint64_t *nnz, da_cache *cache, void *workspace, hipStream_t s);

// ---- built-in scratch of delta_attn_prefill_noalloc.  One copy per GPU, held from the time the library is loaded
// on that GPU until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress, not a
// device address: its address on a device is looked up once per device, with that device current, and only that
// pointer is ever handed to kernels.
constexpr size_t kScratchBytes = DA_NOALLOC_SCRATCH_BYTES;
__device__ __align__(256) unsigned char scratch[kScratchBytes];

void *scratch_of_current_device() {
    static std::mutex mu;
    static void *ptr_of[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        set_last_error("delta_attn_prefill_noalloc: no current device, or a device ordinal above 63");
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of[dev]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            set_last_error("delta_attn_prefill_noalloc: hipGetSymbolAddress: %s", hipGetErrorName(e));
            (void)hipGetLastError();
            return nullptr;
        }
        ptr_of[dev] = ptr;
    }
    return ptr_of[dev];
}

// the kernels read the workspace with 16-byte loads and 64-byte entry chunks; regions are carved at multiples of 256
inline bool ws_aligned(const void *ws) { return ((uintptr_t)ws & (kAlign - 1)) == 0; }

}  // namespace

extern "C" {

const char *delta_attn_last_error(void) { return last_error_text(); }

void delta_attn_stage_timing_enable(int32_t on) { timing_enable(on != 0); }

int32_t delta_attn_stage_timing_read(double *ms_per_stage, int32_t *calls_per_stage) {
    if (!ms_per_stage || !calls_per_stage) return -1;
    return timing_collect(ms_per_stage, calls_per_stage);
}

const char *delta_attn_version(void) { return "delta_attn 0.1 (gfx950)"; }

const char *delta_attn_status_string(da_status s) {
    switch (s) {
        case DA_OK: return "ok";
        case DA_ERR_INVALID_ARG: return "invalid argument";
        case DA_ERR_UNSUPPORTED: return "unsupported configuration";
        case DA_ERR_WORKSPACE: return "workspace missing or too small";
        case DA_ERR_STATE: return "cache state does not allow this call";
        case DA_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

int32_t delta_attn_window_from_gamma(int32_t n, double gamma, int32_t w_max) {
    if (n < 1 || w_max < 1 || !(gamma > 0.0)) return 1;
    double w = floor(gamma * (double)n);
    if (w > (double)w_max) w = (double)w_max;
    if (w < 1.0) w = 1.0;
    return (int32_t)w;
}

size_t delta_attn_prefill_workspace_bytes(const da_prefill_params *p) {
    if (check_params(p) != DA_OK) return 0;
    return layout(p).total;
}

size_t delta_attn_delta_scan_workspace_bytes(const da_prefill_params *p) {
    if (check_params(p) != DA_OK) return 0;
    const WsLayout w = layout(p);
    return w.ents;   // reference keys + per-chunk states: the first two regions of the prefill layout
}

da_status delta_attn_delta_scan(const da_prefill_params *p, const void *K, uint32_t *mask_bits, uint64_t *nnz,
                                void *k_hat, void *workspace, size_t workspace_bytes, void *hip_stream) {
    da_status st = check_params(p);
    if (st != DA_OK) return st;
    if (!K || !mask_bits || !nnz) return DA_ERR_INVALID_ARG;
    const WsLayout w = layout(p);
    if (!workspace || workspace_bytes < w.ents || !ws_aligned(workspace)) return DA_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    (void)hipGetLastError();
    launch_delta_scan(p->dtype, K, k_hat ? k_hat : ws + w.khat, mask_bits, ws + w.chunk_out, nnz,
                      p->batch * p->n_kv_heads, p->seq_len, p->head_dim, p->theta, s);
    return launch_ok("delta_scan") ? DA_OK : DA_ERR_HIP;
}

da_status delta_attn_prefill(const da_prefill_params *p, const void *Q, const void *K, const void *V, void *O,
                             uint32_t *mask_bits, uint64_t *nnz, da_cache *cache, void *workspace,
                             size_t workspace_bytes, void *hip_stream) {
    da_status st = check_params(p);
    if (st != DA_OK) return st;
    if (!Q || !K || !V || !O || !mask_bits || !nnz) return DA_ERR_INVALID_ARG;
    const WsLayout w = layout(p);
    if (!workspace || workspace_bytes < w.total || !ws_aligned(workspace)) return DA_ERR_WORKSPACE;
    if (cache) {
        st = cache_check_for_prefill(cache, p);
        if (st != DA_OK) return st;
    }
    return prefill_checked(p, w, Q, K, V, O, mask_bits, nnz, cache, workspace, (hipStream_t)hip_stream);
}

da_status delta_attn_prefill_noalloc(const da_prefill_params *p, const void *Q, const void *K, const void *V, void *O,
                                     uint32_t *mask_bits, uint64_t *nnz, void *hip_stream) {
    da_status st = check_params(p);
    if (st != DA_OK) return st;
    if (!Q || !K || !V || !O || !mask_bits || !nnz) return DA_ERR_INVALID_ARG;
    WsLayout w = layout(p);
    if (w.total > kScratchBytes) w = layout(p, false);   // without the key split of small launches: less scratch
    if (w.total > kScratchBytes) {
        set_last_error("delta_attn_prefill_noalloc: these params need %zu bytes of scratch, the built-in buffer holds %zu",
                       w.total, kScratchBytes);
        return DA_ERR_WORKSPACE;
    }
    void *ws = scratch_of_current_device();
    if (!ws) return DA_ERR_HIP;
    // Nothing in the buffer has to start at zero: every region is written by the scan, compaction and re-order
    // kernels before the attention kernel reads it (the nnz counters, which do, are the caller's and are cleared by
    // a fill kernel on the stream).
    return prefill_checked(p, w, Q, K, V, O, mask_bits, nnz, nullptr, ws, (hipStream_t)hip_stream);
}

}  // extern "C"

namespace {
// the body shared by the two prefill entry points; arguments, workspace and cache have been checked
da_status prefill_checked(const da_prefill_params *p, const WsLayout &w, const void *Q, const void *K, const void *V,
                          void *O, uint32_t *mask_bits, uint64_t *nnz, da_cache *cache, void *workspace,
                          hipStream_t s) {
    char *ws = (char *)workspace;
    void *khat = ws + w.khat;
    void *ents = ws + w.ents;
    uint32_t *counts = (uint32_t *)(ws + w.counts);
    uint8_t *nch8 = (uint8_t *)(ws + w.nch8);
    const int units = p->batch * p->n_kv_heads;

    (void)hipGetLastError();   // do not inherit an earlier, unrelated error
    PrefillArgs a;
    a.dtype = p->dtype;
    a.d = p->head_dim;
    a.B = p->batch;
    a.Hkv = p->n_kv_heads;
    a.Hq = p->n_q_heads;
    a.n = p->seq_len;
    // Short prompts on the matrix-core kernel: one launch does everything (the scan, the compaction and the V
    // re-order run inside the attention launch, once per work group); longer ones take a launch per stage.
    const bool fused = prefill_mfma_supported(a) && (int64_t)p->seq_len * p->head_dim <= kFusedMaxElems;
    // (the scan's first launch takes the V re-order of the matrix-core kernels along where it can)
    const bool vt_in_scan = !fused && prefill_mfma_supported(a) && delta_scan_takes_v(p->dtype, p->seq_len, p->head_dim);
    if (!fused) {
        stage_begin(kStageScan, s);
        launch_delta_scan(p->dtype, K, khat, mask_bits, ws + w.chunk_out, nnz, units, p->seq_len, p->head_dim,
                          p->theta, s, nullptr, vt_in_scan ? V : nullptr, vt_in_scan ? ws + w.vt : nullptr,
                          prefill_mfma_n_pad(p->seq_len));
        stage_end(kStageScan, s);
        if (!launch_ok("delta_scan")) return DA_ERR_HIP;
        if (p->score_mode == DA_SCORE_GATHER || cache) {
            stage_begin(kStageEmit, s);
            launch_emit_entries(p->dtype, K, khat, mask_bits, ents, counts, nch8, ws + w.plan,
                                (uint32_t *)(ws + w.dense), units, p->seq_len, prefill_mfma_n_pad(p->seq_len),
                                p->head_dim, s);
            stage_end(kStageEmit, s);
            if (!launch_ok("emit_entries")) return DA_ERR_HIP;
        }
    }
    a.fused = fused ? 1 : 0;
    a.mask_bits = mask_bits;
    a.nnz = nnz;
    a.theta = p->theta;
    a.dtype = p->dtype;
    a.B = p->batch;
    a.Hq = p->n_q_heads;
    a.Hkv = p->n_kv_heads;
    a.d = p->head_dim;
    a.n = p->seq_len;
    a.q_off = 0;
    a.nq = p->seq_len;
    a.W = p->window;
    a.scale_log2 = score_scale(p->scale, p->head_dim) * 1.4426950408889634f;
    a.rebase = p->score_mode == DA_SCORE_REBASE;
    a.sliding = p->window_mode == DA_WINDOW_SLIDING;
    a.Q = Q;
    a.K = K;
    a.V = V;
    a.Khat = khat;
    a.O = O;
    a.ents = ents;
    a.counts = counts;
    a.nch8 = nch8;
    a.ksplit = w.ksplit;
    a.part = ws + w.part;
    a.vt_from = vt_in_scan ? prefill_mfma_n_pad(p->seq_len) / 32 : 0;   // (every block of V is in place already)
    a.plan = ws + w.plan;
    a.dense = (const uint32_t *)(ws + w.dense);
    stage_begin(kStageAttn, s);
    bool launched = true;
    if (prefill_mfma_supported(a))
        launch_prefill_mfma(a, ws + w.vt, s);
    else
        launched = launch_prefill_generic(a, s);
    stage_end(kStageAttn, s);
    if (!launched) return DA_ERR_UNSUPPORTED;
    if (!launch_ok("prefill attention")) return DA_ERR_HIP;
    if (cache) {
        stage_begin(kStageCacheFill, s);
        cache_fill_from_prefill(cache, p, K, V, khat, mask_bits, counts, nnz, s);
        stage_end(kStageCacheFill, s);
        if (!launch_ok("cache_fill")) return DA_ERR_HIP;
    }
    return DA_OK;
}

// workspace of delta_attn_prefill_append: what the scan of the new rows needs (the whole-sequence arrays live in the
// cache, see da_prefix)
struct AppendLayout {
    size_t hnew, chunk_out, part, total;
    int ksplit;
};

AppendLayout append_layout(const da_prefill_params *p, int64_t cached) {
    const size_t units = (size_t)p->batch * p->n_kv_heads, d = p->head_dim, es = elt_size(p->dtype);
    const size_t m = p->seq_len;
    AppendLayout w;
    size_t off = 0;
    w.hnew = off;
    off += align_up(units * m * d * es);
    w.chunk_out = off;
    off += align_up(2 * units * (size_t)delta_scan_num_chunks((int)m) * d * es);
    const PrefillArgs a = split_args(p, cached);
    w.ksplit = prefill_mfma_ksplit(a);
    w.part = off;
    off += align_up(prefill_mfma_part_bytes(a, w.ksplit));
    w.total = off;
    return w;
}

// The cache's whole-sequence arrays (da_prefix), allocated on first use and zero-filled (rows nothing has written yet
// must hold finite numbers: the kernels load whole tiles and discard what lies past the sequence).
da_status ensure_prefix(da_cache *c, bool gather) {
    if (!c->pf) {
        c->pf = new (std::nothrow) da_prefix();
        if (!c->pf) return DA_ERR_HIP;
        memset(c->pf, 0, sizeof(*c->pf));
    }
    da_prefix *f = c->pf;
    const size_t units = (size_t)c->B * c->Hkv, d = c->d, ld = c->max_seq, ld_pad = prefill_mfma_n_pad(c->max_seq);
    bool ok = true;
    auto room = [&](void **ptr, size_t bytes) {
        if (!ok || *ptr) return;
        ok = hipMalloc(ptr, bytes) == hipSuccess && hipMemset(*ptr, 0, bytes) == hipSuccess;
    };
    room(&f->k, units * ld * d * 2);
    room(&f->h, units * ld * d * 2);
    room(&f->v, units * ld * d * 2);
    room((void **)&f->m, units * ld * (d / 32) * 4);
    room(&f->vt, units * d * ld_pad * 2);
    if (gather) {
        room(&f->ents, units * ld * d * 8);
        room((void **)&f->counts, units * ld * 4);
        room((void **)&f->nch8, units * ld_pad);
        room(&f->plan, units * ld_pad * 2);
        room((void **)&f->dense, units * (ld_pad / 32) * 4);
    }
    if (!ok) {
        (void)launch_ok("prefill_append: room for the cached sequence as plain arrays");   // records the error text
        return DA_ERR_HIP;
    }
    return DA_OK;
}

da_status check_append(const da_prefill_params *p, const da_cache *c) {
    da_status st = check_params(p);
    if (st != DA_OK) return st;
    if (!c) return DA_ERR_INVALID_ARG;
    if (!c->fast) return DA_ERR_UNSUPPORTED;                 // only the column-run cache layout can be continued
    if (c->B != p->batch || c->Hq != p->n_q_heads || c->Hkv != p->n_kv_heads || c->d != p->head_dim ||
        c->dtype != p->dtype || c->theta != p->theta)
        return DA_ERR_STATE;
    if (!cache_scale_matches(c, p->scale)) return DA_ERR_STATE;   // one score scale for prefill and decode (Eq. 1)
    if (c->len + p->seq_len > c->max_seq) return DA_ERR_STATE;
    // raw keys of a window come from the ring of the decode_window newest rows; no window reaches back further
    // than the sequence is long
    const int64_t reach = p->window < c->len + p->seq_len ? p->window : c->len + p->seq_len;
    if (c->len > 0 && reach > c->Wd) return DA_ERR_UNSUPPORTED;
    if (!prefill_mfma_supported(split_args(p, c->len))) return DA_ERR_UNSUPPORTED;   // (more tiles than a grid holds)
    return DA_OK;
}
}  // namespace

extern "C" {

size_t delta_attn_prefill_append_workspace_bytes(const da_prefill_params *p, const da_cache *cache) {
    if (check_append(p, cache) != DA_OK) return 0;
    return append_layout(p, cache->len).total;
}

da_status delta_attn_prefill_append(const da_prefill_params *p, const void *Q, const void *K, const void *V, void *O,
                                    uint32_t *mask_bits, uint64_t *nnz, da_cache *cache, void *workspace,
                                    size_t workspace_bytes, void *hip_stream) {
    da_status st = check_append(p, cache);
    if (st != DA_OK) return st;
    if (!Q || !K || !V || !O || !mask_bits || !nnz) return DA_ERR_INVALID_ARG;
    const int t0 = (int)cache->len, m = p->seq_len, nk = t0 + m, d = p->head_dim;
    const AppendLayout w = append_layout(p, t0);
    if (!workspace || workspace_bytes < w.total || !ws_aligned(workspace)) return DA_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    const int units = p->batch * p->n_kv_heads;
    const bool gather = p->score_mode == DA_SCORE_GATHER;
    (void)hipGetLastError();
    st = ensure_prefix(cache, gather);
    if (st != DA_OK) return st;
    da_prefix *f = cache->pf;
    const int ld = cache->max_seq;
    const int n_pad = prefill_mfma_n_pad(nk);

    // 1. the cached rows as plain arrays: kept from the previous piece, or (after decode steps or a one-shot prefill
    //    into this cache) unpacked from the cache; the new rows behind them
    const bool kept = f->rows == t0;
    f->rows = -1;                                   // in flux until this call has gone through
    if (!kept) {
        expand_cache_runs(cache, t0, ld, f->k, f->h, f->v, f->m, s);
        f->ent_rows = 0;
    }
    // 2. Eq. 2-3 over the new rows, continuing from the cache's reference key (row 0 of an empty cache is the basis);
    //    the new rows (keys, values, reference keys, mask rows) go behind the cached ones
    stage_begin(kStageScan, s);
    launch_delta_scan(p->dtype, K, ws + w.hnew, mask_bits, ws + w.chunk_out, nnz, units, m, d, p->theta, s,
                      t0 > 0 ? cache->khat : nullptr);
    launch_append_rows(K, V, ws + w.hnew, mask_bits, f->k, f->v, f->h, f->m, units, t0, m, ld, d, s);
    stage_end(kStageScan, s);
    if (!launch_ok("delta_scan")) return DA_ERR_HIP;
    // 3. entry lists and plans of the key columns that do not have them yet, from the first block of 32 columns that
    //    is new or was incomplete (cached columns from reference keys: where a bit is set they equal the key)
    if (gather) {
        const int64_t have = f->ent_rows < t0 ? f->ent_rows : t0;
        stage_begin(kStageEmit, s);
        launch_emit_entries(p->dtype, f->k, f->h, f->m, f->ents, f->counts, f->nch8, f->plan, f->dense, units, nk, n_pad,
                            d, s, ld, (int)(have / 32));
        stage_end(kStageEmit, s);
        if (!launch_ok("emit_entries")) return DA_ERR_HIP;
    }
    // 4. attention of the new rows over all nk keys
    PrefillArgs a;
    a.dtype = p->dtype;
    a.B = p->batch;
    a.Hq = p->n_q_heads;
    a.Hkv = p->n_kv_heads;
    a.d = d;
    a.n = nk;
    a.q_off = t0;
    a.nq = m;
    a.ld = ld;
    a.vt_from = kept ? t0 / 32 : 0;
    a.ksplit = w.ksplit;
    a.part = ws + w.part;
    a.W = p->window;
    a.scale_log2 = score_scale(p->scale, d) * 1.4426950408889634f;
    a.rebase = p->score_mode == DA_SCORE_REBASE;
    a.sliding = p->window_mode == DA_WINDOW_SLIDING;
    a.Q = Q;
    a.K = f->k;
    a.V = f->v;
    a.Khat = f->h;
    a.O = O;
    a.ents = f->ents;
    a.counts = f->counts;
    a.nch8 = f->nch8;
    a.plan = f->plan;
    a.dense = f->dense;
    a.fused = 0;
    a.mask_bits = nullptr;
    a.nnz = nullptr;
    a.theta = p->theta;
    stage_begin(kStageAttn, s);
    launch_prefill_mfma(a, f->vt, s);                  // (supported: check_append has asked)
    stage_end(kStageAttn, s);
    if (!launch_ok("prefill_append attention")) return DA_ERR_HIP;
    // 5. the new rows join the cache
    stage_begin(kStageCacheFill, s);
    cache_fill_runs(cache, t0, nk, ld, f->k, V, f->h, f->m, nnz, s);
    stage_end(kStageCacheFill, s);
    if (!launch_ok("cache_fill")) return DA_ERR_HIP;
    cache->len = nk;
    f->rows = nk;
    if (gather) f->ent_rows = nk;
    return DA_OK;
}

da_status delta_attn_sparsity(const uint64_t *nnz_dev, int32_t batch, int32_t n_kv_heads, int64_t rows,
                              int32_t head_dim, int32_t window, void *hip_stream, double *s_m, double *s_c) {
    if (!nnz_dev || !s_m || !s_c || batch < 1 || n_kv_heads < 1 || rows < 1 || head_dim < 1 || window < 1)
        return DA_ERR_INVALID_ARG;
    const size_t units = (size_t)batch * n_kv_heads;
    uint64_t *host = new (std::nothrow) uint64_t[units];
    if (!host) return DA_ERR_HIP;
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e = hipMemcpyAsync(host, nnz_dev, units * sizeof(uint64_t), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        delete[] host;
        return DA_ERR_HIP;
    }
    uint64_t total = 0;
    for (size_t u = 0; u < units; ++u) total += host[u];
    delete[] host;
    const double all = (double)units * (double)rows * (double)head_dim;
    *s_m = 1.0 - (double)total / all;
    const double w = (double)(window < rows ? window : rows);
    *s_c = *s_m * (1.0 - w / (double)rows);
    return DA_OK;
}

}  // extern "C"
