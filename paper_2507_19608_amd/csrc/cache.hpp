// Decode-time cache object (Sec. III-A last paragraph, Sec. III-C).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/delta_attn.h"

constexpr int kChunk = 64;   // rows per decode chunk; one reference-key checkpoint per chunk

struct da_cache {
    int B, Hq, Hkv, d, max_seq, Wd, dtype;
    float theta, scale;
    int64_t len;          // rows held (all sequences of the batch advance together)
    int device;
    int nck;              // checkpoints per unit: max_seq / kChunk + 1
    int max_chunks;       // (max_seq + kChunk - 1) / kChunk
    int vrows;            // max_seq rounded up to a whole chunk (row capacity of V)
    // per (batch, KV head) unit, all device memory:
    uint32_t *mask;       // [units][max_seq][d/32]   delta mask bits
    void *surv;           // [units][max_chunks][kChunk * d] surviving key values of a chunk: row after row, channel order
    uint32_t *ccnt;       // [units][max_chunks]      survivors stored in each chunk
    void *ck;             // [units][nck][d]          ck[m] = reference key after row m*kChunk - 1 (m >= 1)
    void *khat;           // [units][d]               current reference key
    void *ring;           // [units][Wd][d]           raw key of position p at slot p % Wd
    void *V;              // [units][vrows / 8][d][8]: 8 rows interleaved per channel
    uint64_t *nnz;        // [units]
    float *part;          // [B*Hq][max_chunks][d + 2] per-chunk (o, m, l) partials of one decode step
};

namespace da {
da_status cache_check_for_prefill(const da_cache *c, const da_prefill_params *p);
void cache_fill_from_prefill(da_cache *c, const da_prefill_params *p, const void *K, const void *V,
                             const void *Khat, const uint32_t *mask_bits, const uint32_t *counts,
                             const uint64_t *nnz, hipStream_t s);
}  // namespace da
