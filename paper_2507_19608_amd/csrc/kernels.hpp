// Host-side launch functions of the kernels (one .hip file each).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace da {

// Raises the dynamic-LDS limit of kernel `fn` to `bytes` on the current device, once per device (`done` holds one bit
// per device ordinal; safe to call from several threads).  On failure the error is left for launch_ok() to report
// and the next call tries again.
void ensure_dynamic_lds(const void *fn, int bytes, std::atomic<uint64_t> &done);

// Checks hipGetLastError(); on failure records "<stage>: <hip error>" for delta_attn_last_error()
// and returns false.
bool launch_ok(const char *stage);
const char *last_error_text();
// records a printf-style message as the calling thread's last error text
void set_last_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));

// Optional per-stage timing with HIP events recorded on the caller's stream (off by default).
enum Stage { kStageScan = 0, kStageEmit, kStageAttn, kStageCacheFill, kStageAppend, kStageChunk, kStageCombine,
             kNumStages };
void stage_begin(int stage, hipStream_t s);   // no-ops unless timing is enabled
void stage_end(int stage, hipStream_t s);
void timing_enable(bool on);
int timing_collect(double *ms_per_stage, int *calls_per_stage);

struct PrefillArgs {
    int dtype;            // 0 f32, 1 bf16
    int B, Hq, Hkv, d, n, W;   // n = number of key rows
    int q_off, nq;             // the query rows are positions q_off .. q_off + nq - 1 (q_off + nq == n)
    int ld = 0;                // > 0 (matrix-core path only): K, V, Khat, ents, counts have ld >= n rows of room per
                               // unit and nch8, plan, dense, vt the strides of prefill_mfma_n_pad(ld); 0: exactly n
    int vt_from = 0;           // blocks of 32 rows below this one are already in vt (V re-order of earlier rows kept)
    int ksplit = 1;            // matrix-core path: work groups per tile (prefill_mfma_ksplit), each on a part of the keys
    void *part = nullptr;      // ksplit > 1: prefill_mfma_part_bytes of scratch for the parts' results
    float scale_log2;     // score scale * log2(e)
    int rebase;           // 1: outside scores from q . k_hat instead of the entry lists
    int sliding;          // 1: exact region is the band i - j < W instead of squares of side W
    const void *Q, *K, *V, *Khat;
    void *O;
    const void *ents;     // EntryChunk lists, column (unit, j) at chunk (unit * n + j) * d / 8
    const uint32_t *counts;
    const uint8_t *nch8;  // chunks per column, stride prefill_mfma_n_pad(n) per unit
    const void *plan;     // gather mode: the column plan written by launch_emit_entries
    const uint32_t *dense;   // gather mode: per unit and block of 32 columns, the columns re-based instead of gathered
    // fused short-prompt launch (matrix-core kernel only): the attention launch itself runs the delta scan, the
    // compaction and the V re-order; then K_hat, ents, counts, nch8, plan, dense are scratch it fills first
    int fused;
    uint32_t *mask_bits;  // out (fused)
    uint64_t *nnz;        // out (fused)
    float theta;          // (fused)
};

// the fused launch is used for prompts of at most this many key elements per unit (seq_len * head_dim): their keys,
// reference keys and mask words fit in LDS side by side
constexpr int kFusedMaxElems = 32768;

void launch_fill_u64(uint64_t *p, uint64_t v, int n, hipStream_t s);

// Chunked prefill: rows of the new piece - K, V, H [units][m][d] (bf16) and M [units][m][d/32] - are copied behind
// row t0 of the whole-sequence arrays [units][ld][...].
void launch_append_rows(const void *K, const void *V, const void *H, const uint32_t *M, void *Kfull, void *Vfull,
                        void *Hfull, uint32_t *Mfull, int units, int t0, int m, int ld, int d, hipStream_t s);
int delta_scan_num_chunks(int n);
// V, Vt (both or neither; used only where delta_scan_takes_v() says so): the value rows [units][n][d] are re-ordered
// into Vt [units][d][n_pad], the operand order of the matrix-core prefill kernels, by extra work groups of the scan's
// first launch (they have nothing to do with the scan; it saves the prefill a launch).
bool delta_scan_takes_v(int dtype, int n, int d);
void launch_delta_scan(int dtype, const void *K, void *Khat, uint32_t *mask_bits, void *chunk_out, uint64_t *nnz,
                       int units, int n, int d, float theta, hipStream_t s, const void *init = nullptr,
                       const void *V = nullptr, void *Vt = nullptr, int n_pad = 0);
// plan: NULL, or room for units * n_pad * 2 bytes: the gather loop's column plan; dense (used with plan): room for
// units * n_pad / 32 words (see emit_entries_kernel)
void launch_emit_entries(int dtype, const void *K, const void *Khat, const uint32_t *mask_bits, void *ents,
                         uint32_t *counts, uint8_t *nch8, void *plan, uint32_t *dense, int units, int n, int n_pad,
                         int d, hipStream_t s, int ld = 0, int blk0 = 0);
// Generic path: any head_dim in {32, 64, ..., 256}, both dtypes, VALU only.  Returns false if
// the head_dim has no instantiation.
bool launch_prefill_generic(const PrefillArgs &a, hipStream_t s);
// Matrix-core path: bf16, head_dim 64 or 128.  vt is scratch for V^T: units * d * prefill_mfma_n_pad(n) bf16.
bool prefill_mfma_supported(const PrefillArgs &a);
int prefill_mfma_n_pad(int n);
void launch_prefill_mfma(const PrefillArgs &a, void *vt, hipStream_t s);
// Key-range split of the matrix-core launch (flash-decoding style, for launches that do not fill the chip): the
// number of work groups per tile that pays for these arguments on the current device (1: none; reads B, Hq, Hkv, d,
// nq, q_off, fused, dtype) and the scratch that many need.
int prefill_mfma_ksplit(const PrefillArgs &a);
size_t prefill_mfma_part_bytes(const PrefillArgs &a, int ksplit);
// compute units of the current device (256 if it cannot be asked)
int device_cu_count();

}  // namespace da
