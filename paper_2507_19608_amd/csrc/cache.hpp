// Decode-time cache object (Sec. III-A last paragraph, Sec. III-C).
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/delta_attn.h"

constexpr int kChunk = 64;   // rows per decode chunk; one reference-key checkpoint per chunk

// What delta_attn_prefill_append keeps between its calls on one cache (Sec. III-C, a prompt processed in pieces):
// the sequence so far as the plain arrays the prefill kernels read, so that a piece only adds its own rows instead
// of unpacking and compacting the whole prefix again.  Device memory with max_seq rows of room per unit (row stride
// max_seq, padded strides from prefill_mfma_n_pad(max_seq)), allocated by the first such call (the entry-list
// arrays by the first one in gather mode), freed with the cache.  Host-side bookkeeping: kernels never see it.
struct da_prefix {
    void *k, *h, *v;      // [units][max_seq][d]     keys (raw where a window may need them, see expand_cache_kernel),
                          //                         reference keys, values
    uint32_t *m;          // [units][max_seq][d/32]  mask rows
    void *vt;             // V in matrix-core operand order (transpose_v_kernel)
    void *ents;           // entry lists, counts, chunk counts, gather plan, re-based columns (emit_entries_kernel)
    uint32_t *counts;
    uint8_t *nch8;
    void *plan;
    uint32_t *dense;
    int64_t rows;         // k, h, v, m, vt describe rows 0 .. rows - 1 of the cached sequence; only trusted while
                          // rows == the cache's length (decode steps and one-shot prefills do not maintain them)
    int64_t ent_rows;     // key columns 0 .. ent_rows - 1 have their entry lists and plans
};

struct da_cache {
    int B, Hq, Hkv, d, max_seq, Wd, dtype;
    float theta, scale;
    int64_t len;          // rows held (all sequences of the batch advance together)
    int device;
    int cus;              // compute units of `device` (0 until the first decode step has asked)
    int nck;              // checkpoints per unit: max_seq / kChunk + 1
    int max_chunks;       // (max_seq + kChunk - 1) / kChunk
    int vrows;            // max_seq rounded up to a whole chunk (row capacity of V)
    int plan_merge;       // launch plan of the column-run layout: -1 auto, 0 second launch, 1 merge in the kernel
    int plan_slots;       // wave slots a launch is sized for, 0 = from the device
    int fast;             // 1: bf16, head_dim 64 or 128, decode window >= kChunk or >= max_seq, <= 32 query heads per KV
                          //    head: the column-run layout below
    // per (batch, KV head) unit, all device memory:
    uint32_t *mask;       // [units][max_seq][d/32]   delta mask bits
    // Surviving key values (the new reference values at the positions the mask marks), run_room_stride(d)
    // elements of room per chunk.
    //   row layout (fast == 0): row after row, channels ascending inside a row, appended one row per step.
    //   column-run layout (fast == 1): written once per chunk, when its last row has arrived ("sealed"):
    //     for every channel in ascending order one run = the reference value held when the chunk starts,
    //     then the channel's surviving values in row order.  Rows of an unsealed chunk are always inside
    //     the decode window (window >= kChunk, or the whole cache), where raw keys are used, so they need no run.  At head_dim
    //     128 the runs of channels 64.. start at the next multiple of 8 elements.
    void *surv;           // [units][max_chunks][run_room_stride(d)]
    uint32_t *ccnt;       // [units][max_chunks]      row layout: elements stored in the chunk's room; column-run
                          //                          layout: that in the low half, the start of the runs of
                          //                          channels 64.. (head_dim 64: the same number) in the high half
    void *ck;             // [units][nck][d]          ck[m] = reference key after row m*kChunk - 1 (m >= 1)
    void *khat;           // [units][d]               current reference key
    void *ring;           // [units][Wd][d]           raw key of position p at slot p % Wd
    void *V;              // fast == 0: [units][vrows / 8][d][8], 8 rows interleaved per channel;
                          // fast == 1: [units][vrows / 16][d][16], 16 rows per channel in matrix-core
                          //            accumulator order (slot 8 k + i holds row 8 (i / 4) + 4 k + i % 4)
    uint64_t *nnz;        // [units]
    float *part;          // [B*Hq][max_chunks][d + 4] partial (o[d], m, l, 2 unused) rows of one decode step
    da_prefix *pf;        // host pointer, NULL until delta_attn_prefill_append has run on this cache
};

// elements of room per chunk for the surviving values: one per key element, one carried-in value per channel, and
// the alignment gap of the column-run layout
__host__ __device__ inline size_t run_room_stride(int d) { return (size_t)(kChunk + 1) * d + 8; }

// floats per partial row: o[d], running maximum, running sum, padded to a 16-byte multiple
__host__ __device__ inline int part_stride(int d) { return d + 4; }

namespace da {
// the scale a params value stands for: 0 selects 1 / sqrt(head_dim) (Eq. 1)
inline float resolved_scale(float scale, int d) { return scale > 0.f ? scale : 1.0f / sqrtf((float)d); }
inline bool cache_scale_matches(const da_cache *c, float scale) {
    return resolved_scale(scale, c->d) == resolved_scale(c->scale, c->d);
}
da_status cache_check_for_prefill(const da_cache *c, const da_prefill_params *p);
void cache_fill_from_prefill(da_cache *c, const da_prefill_params *p, const void *K, const void *V,
                             const void *Khat, const uint32_t *mask_bits, const uint32_t *counts,
                             const uint64_t *nnz, hipStream_t s);
// column-run layout (fast == 1)
// appends rows t0 .. n_k - 1 (t0 = rows already held) from whole-sequence arrays [units][ld][...] (ld >= n_k rows of
// room per unit)
void cache_fill_runs(da_cache *c, int t0, int n_k, int ld, const void *Kfull, const void *Vnew, const void *Hfull,
                     const uint32_t *Mfull, const uint64_t *nnz_new, hipStream_t s);
// writes the cached rows 0 .. t0 - 1 out as whole-sequence arrays with ld >= t0 rows of room per unit
void expand_cache_runs(da_cache *c, int t0, int ld, void *Kfull, void *Hfull, void *Vfull, uint32_t *Mfull,
                       hipStream_t s);
// returns the number of partial rows written per head, 0 if the launch wrote the output itself
int decode_step_runs(da_cache *c, const void *q, const void *k, const void *v, void *o, uint32_t *mask_row, int t,
                     float scale_log2, hipStream_t s);
void seal_chunk_runs(da_cache *c, int chunk, hipStream_t s);
}  // namespace da
