// Delta matrix construction on the key matrix (Sec. II-C Eq. 2-3; Sec. III-A strategy 3) and
// compaction of the surviving entries per key column.
#include "common.hpp"
#include "kernels.hpp"
#include "scan_device.hpp"
#include "vt_device.hpp"

#include <stdarg.h>
#include <stdio.h>

#include <mutex>

namespace da {

static thread_local char g_last_error[256] = "";

bool launch_ok(const char *stage) {
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return true;
    snprintf(g_last_error, sizeof(g_last_error), "%s: %s (%s)", stage, hipGetErrorName(e), hipGetErrorString(e));
    return false;
}

const char *last_error_text() { return g_last_error; }

void set_last_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
    va_end(ap);
}

void ensure_dynamic_lds(const void *fn, int bytes, std::atomic<uint64_t> &done) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) dev = 63;   // ordinals past 62 share a bit: set every time
    const uint64_t bit = (uint64_t)1 << dev;
    if (dev < 63 && (done.load(std::memory_order_acquire) & bit)) return;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess)
        done.fetch_or(bit, std::memory_order_release);
}

// ---- stage timing: a pool of event pairs, filled in call order, summed and recycled by the reader
namespace {
constexpr int kMaxPairs = 8192;
struct Pair {
    hipEvent_t a, b;
    int stage;
};
std::mutex g_timing_mutex;   // the pool is process-wide: a benchmarking aid, serialised rather than per call
std::atomic<bool> g_timing{false};
Pair g_pairs[kMaxPairs];
int g_created = 0, g_used = 0, g_open[kNumStages];
}  // namespace

void stage_begin(int stage, hipStream_t s) {
    if (!g_timing.load(std::memory_order_relaxed)) return;
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    if (g_used >= kMaxPairs) return;
    if (g_used >= g_created) {
        if (hipEventCreate(&g_pairs[g_created].a) != hipSuccess) return;
        if (hipEventCreate(&g_pairs[g_created].b) != hipSuccess) return;
        ++g_created;
    }
    g_pairs[g_used].stage = stage;
    g_open[stage] = g_used;
    (void)hipEventRecord(g_pairs[g_used].a, s);
    ++g_used;
}

void stage_end(int stage, hipStream_t s) {
    if (!g_timing.load(std::memory_order_relaxed)) return;
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    if (g_open[stage] < 0) return;
    (void)hipEventRecord(g_pairs[g_open[stage]].b, s);
    g_open[stage] = -1;
}

void timing_enable(bool on) {
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    g_timing.store(on);
    g_used = 0;
    for (int i = 0; i < kNumStages; ++i) g_open[i] = -1;
}

// Sums elapsed ms per stage over everything recorded since the last read; the caller has
// synchronised the streams involved.  Returns the number of event pairs read.
int timing_collect(double *ms_per_stage, int *calls_per_stage) {
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    for (int i = 0; i < kNumStages; ++i) {
        ms_per_stage[i] = 0.0;
        calls_per_stage[i] = 0;
    }
    int n = 0;
    for (int i = 0; i < g_used; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_pairs[i].a, g_pairs[i].b) == hipSuccess) {
            ms_per_stage[g_pairs[i].stage] += ms;
            calls_per_stage[g_pairs[i].stage] += 1;
            ++n;
        }
    }
    g_used = 0;
    return n;
}

// The recurrence of Eq. 2-3 is sequential in t and is not an associative scan, but it forgets its
// past every time a channel fires: from then on the held value is k(t) whatever it was before.
// So time is cut into chunks that are scanned in parallel from a guessed incoming state:
//
//   pass 1  (one wave per (unit, 64 channels, time chunk)): chunk 0 starts from the basis row (or, when the
//           rows continue a sequence, from the reference key `init` carried over from it) and is exact.
//           Chunk c > 0 starts from the guess "held = k(t0 - 1)" and records only its final held value.  That final value is already the true one for every channel that fired at
//           least once inside the chunk at a row where the true chain fired too - nearly all.
//   pass 2  same scan, but chunk c starts from pass 1's final value of chunk c - 1, and writes mask
//           words, held keys, nnz and its own final values.
//   pass 3  (one wave per (unit, 64 channels), chunks in order): carries the true held value along.
//           Where it equals the value pass 2 started a chunk from, pass 2's results for the chunk
//           are the true ones and nothing is touched; otherwise the chunk's rows are re-run from the
//           true state until it meets pass 2's chain (both hold the same value), correcting mask
//           words, held keys and nnz on the way.  Exact for any input.
//
// One lane per channel; the wave ballot of the threshold decision is the mask word itself.
template <typename T, bool kFinal>
__global__ __launch_bounds__(64) void delta_scan_chunks_kernel(const T *__restrict__ K, T *__restrict__ Khat,
                                                               uint32_t *__restrict__ mask_bits,
                                                               const T *__restrict__ guess_out,
                                                               T *__restrict__ chunk_out,
                                                               unsigned long long *__restrict__ nnz, int n, int d,
                                                               int L, int nchunks, float theta,
                                                               const T *__restrict__ init,
                                                               const bf16_t *__restrict__ V = nullptr,
                                                               bf16_t *__restrict__ Vt = nullptr, int n_pad = 0) {
    const int unit = blockIdx.z, chunk = blockIdx.y;
    const int lane = threadIdx.x;
    // Work groups past the channel waves (the first pass has some when the launcher was given V) have nothing to do
    // with the scan: each re-orders one block of 32 value rows - blocks (L / 32) chunk .. of the unit - for the
    // matrix-core prefill kernels, which need that done before they start and would otherwise pay a launch of its own
    // for it (in the first pass, so that what the later passes write is still in the caches when it is read again).
    if ((int)blockIdx.x >= (d + kWave - 1) / kWave) {
        const int blk = chunk * (L / kTB) + (int)blockIdx.x - (d + kWave - 1) / kWave;
        if (kFinal || blk >= n_pad / kTB) return;
        __shared__ bf16_t tile[kTB * (128 + 2)];
        auto wave_sync = [] {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        };
        if (d == 64)
            transpose_v_block<64, kWave>(V + (size_t)unit * n * 64,
                                         (u32x4 *)(Vt + (size_t)unit * 64 * n_pad) + (size_t)blk * (2 * 2 * 64), blk * kTB,
                                         n, (bf16_t(*)[64 + 2]) tile, lane, wave_sync);
        else
            transpose_v_block<128, kWave>(V + (size_t)unit * n * 128,
                                          (u32x4 *)(Vt + (size_t)unit * 128 * n_pad) + (size_t)blk * (2 * 4 * 64), blk * kTB,
                                          n, (bf16_t(*)[128 + 2]) tile, lane, wave_sync);
        return;
    }
    const int c = blockIdx.x * kWave + lane;
    const bool active = c < d;
    const T *Kp = K + (size_t)unit * n * d;
    T *Hp = Khat + (size_t)unit * n * d;
    uint32_t *Mp = mask_bits + (size_t)unit * n * (d >> 5);
    const int t0 = chunk * L, t1 = min(n, t0 + L);
    float start = 0.f;
    if (chunk > 0 && active)
        start = kFinal ? load_f32(guess_out, ((size_t)unit * nchunks + chunk - 1) * d + c)
                       : load_f32(Kp, (size_t)(t0 - 1) * d + c);
    unsigned long long cnt = 0;
    const float held = scan_rows<T, kFinal>(Kp, Hp, Mp, d, c, lane, t0, t1, chunk == 0,
                                            init ? init + (size_t)unit * d : nullptr, start, theta, &cnt);
    if (active) store_from_f32(chunk_out, ((size_t)unit * nchunks + chunk) * d + c, held);
    if (kFinal && lane == 0) atomicAdd(nnz + unit, cnt);
    // (the first pass, when there is one, also clears the unit's counter for the final pass that follows it in the
    // stream; a single-chunk scan has no first pass and its launcher clears the counters itself)
    if (!kFinal && lane == 0 && blockIdx.x == 0 && chunk == 0) nnz[unit] = 0ull;
}

template <typename T>
__global__ __launch_bounds__(64) void delta_scan_fixup_kernel(const T *__restrict__ K, T *__restrict__ Khat,
                                                              uint32_t *__restrict__ mask_bits,
                                                              const T *__restrict__ out1,   // pass 1 final values
                                                              const T *__restrict__ out2,   // pass 2 final values
                                                              unsigned long long *__restrict__ nnz, int n, int d,
                                                              int L, int nchunks, float theta) {
    const int unit = blockIdx.y;
    const int lane = threadIdx.x;
    const int c = blockIdx.x * kWave + lane;
    const bool active = c < d;
    const int cs = active ? c : 0;
    const int wpr = d >> 5;
    const T *Kp = K + (size_t)unit * n * d;
    T *Hp = Khat + (size_t)unit * n * d;
    uint32_t *Mp = mask_bits + (size_t)unit * n * wpr;
    const bool writer = active && ((lane & 31) == 0);
    const int word = c >> 5;
    const T *o1 = out1 + (size_t)unit * nchunks * d + cs;
    const T *o2 = out2 + (size_t)unit * nchunks * d + cs;

    float held = load_f32(o2, 0);   // chunk 0 is exact
    long long adjust = 0;
    constexpr int G = 4;            // chunks whose boundary values are fetched together
    for (int cb = 1; cb < nchunks; cb += G) {
        float g1[G], g2[G];
#pragma unroll
        for (int u = 0; u < G; ++u) {
            const int ch = min(cb + u, nchunks - 1);
            g1[u] = load_f32(o1, (size_t)(ch - 1) * d);   // the value pass 2 started chunk ch from
            g2[u] = load_f32(o2, (size_t)ch * d);         // the value pass 2 ended chunk ch with
        }
#pragma unroll
        for (int u = 0; u < G; ++u) {
            const int chunk = cb + u;
            if (chunk < nchunks) {
                float spec = g1[u];
                bool synced = !active || (__float_as_uint(held) == __float_as_uint(spec));
                if (__any(!synced)) {
                    // Re-run the chunk's rows until every channel has met pass 2's chain.  The rows are fetched 16 at
                    // a time, the next batch requested before this one is worked on (indices clamped to the chunk):
                    // one row at a time the loop paid a full memory round trip per row.
                    const int t1 = min(n, chunk * L + L);
                    constexpr int U = 16;
                    auto load_batch = [&](float (&k)[U], int tb) {
#pragma unroll
                        for (int r = 0; r < U; ++r) k[r] = load_f32(Kp, (size_t)min(tb + r, t1 - 1) * d + cs);
                    };
                    auto work_batch = [&](const float (&kk)[U], int tb) -> bool {   // true: nothing left to do
#pragma unroll
                        for (int r = 0; r < U; ++r) {
                            const int t = tb + r;
                            if (t >= t1 || !__any(!synced)) return true;
                            const float k = kk[r];
                            const bool fs = fabsf(k - spec) > theta;
                            const bool ft = fabsf(k - held) > theta;
                            spec = fs ? k : spec;
                            if (!synced) {
                                held = ft ? k : held;
                                store_from_f32(Hp, (size_t)t * d + c, held);
                            }
                            const uint64_t bt = __ballot(synced ? fs : ft);
                            const uint64_t bs = __ballot(fs);
                            if (writer) Mp[(size_t)t * wpr + word] = (uint32_t)(bt >> (lane & 32));
                            adjust += (long long)__popcll(bt) - (long long)__popcll(bs);
                            synced = synced || (__float_as_uint(held) == __float_as_uint(spec));
                        }
                        return false;
                    };
                    float ka[U], kb[U];
                    load_batch(ka, chunk * L);
                    for (int tb = chunk * L; tb < t1; tb += 2 * U) {
                        load_batch(kb, tb + U);
                        if (work_batch(ka, tb)) break;
                        load_batch(ka, tb + 2 * U);
                        if (work_batch(kb, tb + U)) break;
                    }
                }
                // a synced channel ends the chunk where pass 2's chain ended; an unsynced one walked all of it
                held = synced ? g2[u] : held;
            }
        }
    }
    if (lane == 0 && adjust != 0) atomicAdd(nnz + unit, (unsigned long long)adjust);
}

// One work group per block of 32 key columns, a wave per column at a time: ballot + prefix count turn the mask row into
// a dense list of (channel, delta) pairs in EntryChunk form, padded with (0, 0.0f) to whole chunks and to at
// least one chunk.  The chunks of column j of a unit start at chunk (unit * n + j) * d / 8;
// counts holds the unpadded length, nch8 (stride n_pad per unit) the number of chunks.
// plan (may be NULL): which of the block's columns each of the 8 waves of the matrix-core prefill kernel takes in its
// gather loop, and in which pairs.  Full columns - lists that fill all d / 8 chunks, i.e. more than d - 8 surviving
// entries: the whole-vector jumps of the key stream, and the basis row - can be left out of the gather: the running
// score of Eq. 4 is then re-based at such a column from the dense product q . k_hat(j), which the telescoped sum makes
// exact, on the matrix cores.  That costs a block a fixed amount (one K_hat Q^T tile) and saves the gather of each
// full column, so it is done in blocks with at least kRouteMin full columns (measured break-even: about three), and
// only if every reference key of the block fits fp16, the tile's operand format.  Re-based columns get chunk count 0
// in the plan and their bit set in the block's word of `dense` ([units][n_pad / 32]).  The other
// columns are ranked by chunk count (ties: lower index first), neighbours in that order form the 16 pairs (so the two
// columns of a pair have nearly the same length), and every wave is dealt two pairs so that the four SIMDs carry
// nearly equal numbers of gather steps (plan_block).  A wave's 8
// bytes: the four column indices (first pair, longer column first; second pair), then their chunk counts; blocks that
// reach past row n get zero counts and no dense bits (that kernel only gathers in blocks left of every row's window).
// Which wave sums a column does not change the sum.
template <typename T>
__global__ __launch_bounds__(256) void emit_entries_kernel(const T *__restrict__ K, const T *__restrict__ Khat,
                                                           const uint32_t *__restrict__ mask_bits,
                                                           EntryChunk *__restrict__ ents, uint32_t *__restrict__ counts,
                                                           uint8_t *__restrict__ nch8, uint8_t *__restrict__ plan,
                                                           uint32_t *__restrict__ dense, int n, int ld, int ld_pad,
                                                           int blk0, int d) {
    constexpr int kCols = kPlanCols, kPlanWaves = kPlanWaveCount;
    __shared__ uint32_t blk_cnt[kCols];
    const int unit = blockIdx.y, blk = blk0 + blockIdx.x;
    const int lane = threadIdx.x & 63;
    const size_t row0 = (size_t)unit * ld;
    // the 4 waves take every 4th column of the block
    emit_columns(K + row0 * d, Khat + row0 * d, mask_bits + row0 * (d >> 5), ents + row0 * (d / kGroup), counts + row0,
                 nch8 + (size_t)unit * ld_pad, blk_cnt, n, d, lane, blk * kCols + (int)(threadIdx.x >> 6), 4,
                 (blk + 1) * kCols, blk * kCols);
    if (!plan) return;
    __syncthreads();
    if (threadIdx.x < kWave)                                  // the first wave; its lanes 0 .. 31 own a column each
        plan_block(blk_cnt, plan + ((size_t)unit * (ld_pad / kCols) + blk) * kPlanWaves * 8,
                   dense + (size_t)unit * (ld_pad / kCols) + blk, (blk + 1) * kCols <= n, d, threadIdx.x);
}

__global__ void fill_u64_kernel(unsigned long long *p, unsigned long long v, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// Chunked prefill: the m new rows of every unit join the whole-sequence arrays behind the t0 rows these already
// hold - keys, values and reference keys (rows of row16 16-byte pieces, [units][m] -> [units][ld] at row t0) and mask
// rows (mwords words each) - in one launch.  blockIdx.y = unit; the threads of a unit walk the four copies in turn.
__global__ __launch_bounds__(256) void append_rows_kernel(const uint4 *__restrict__ K, const uint4 *__restrict__ V,
                                                          const uint4 *__restrict__ H, const uint32_t *__restrict__ M,
                                                          uint4 *__restrict__ Kfull, uint4 *__restrict__ Vfull,
                                                          uint4 *__restrict__ Hfull, uint32_t *__restrict__ Mfull, int t0,
                                                          int m, int ld, int row16, int mwords) {
    const size_t unit = blockIdx.y;
    const int pieces = m * row16, words = m * mwords;
    const size_t src = unit * (size_t)pieces, dst = (unit * (size_t)ld + (size_t)t0) * row16;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < 3 * pieces + words; i += gridDim.x * blockDim.x) {
        if (i < pieces) Kfull[dst + i] = K[src + i];
        else if (i < 2 * pieces) Vfull[dst + i - pieces] = V[src + i - pieces];
        else if (i < 3 * pieces) Hfull[dst + i - 2 * pieces] = H[src + i - 2 * pieces];
        else {
            const int k = i - 3 * pieces;
            Mfull[(unit * (size_t)ld + (size_t)t0) * mwords + k] = M[unit * (size_t)words + k];
        }
    }
}

void launch_append_rows(const void *K, const void *V, const void *H, const uint32_t *M, void *Kfull, void *Vfull,
                        void *Hfull, uint32_t *Mfull, int units, int t0, int m, int ld, int d, hipStream_t s) {
    if (units <= 0 || m <= 0) return;
    const int row16 = d * 2 / 16, mwords = d / 32;
    const long long per_unit = (long long)m * (3 * row16 + mwords);
    const int blocks = (int)((per_unit + 1023) / 1024 < 1024 ? (per_unit + 1023) / 1024 : 1024);   // ~4 pieces a thread
    hipLaunchKernelGGL(append_rows_kernel, dim3(blocks, units), dim3(256), 0, s, (const uint4 *)K, (const uint4 *)V,
                       (const uint4 *)H, M, (uint4 *)Kfull, (uint4 *)Vfull, (uint4 *)Hfull, Mfull, t0, m, ld, row16,
                       mwords);
}

int device_cu_count() {
    static std::atomic<int> cached[64];                          // per device ordinal; 0 = not asked yet
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return 256;
    }
    cus = cached[dev].load(std::memory_order_relaxed);
    if (cus > 0) return cus;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
        (void)hipGetLastError();
        return 256;
    }
    cached[dev].store(cus, std::memory_order_relaxed);
    return cus;
}

void launch_fill_u64(uint64_t *p, uint64_t v, int n, hipStream_t s) {
    if (n <= 0) return;
    hipLaunchKernelGGL(fill_u64_kernel, dim3((n + 255) / 256), dim3(256), 0, s, (unsigned long long *)p,
                       (unsigned long long)v, n);
}

int delta_scan_chunk_len(int n) { return n >= 1024 ? 128 : 64; }
int delta_scan_num_chunks(int n) { return (n + delta_scan_chunk_len(n) - 1) / delta_scan_chunk_len(n); }

template <typename T>
static void scan_typed(const void *K, void *Khat, uint32_t *mask_bits, void *chunk_out, uint64_t *nnz, int units,
                       int n, int d, float theta, const void *init, hipStream_t s, const void *V, void *Vt, int n_pad) {
    const int L = delta_scan_chunk_len(n), nchunks = delta_scan_num_chunks(n);
    const int cw = (d + kWave - 1) / kWave;
    T *out1 = (T *)chunk_out;
    T *out2 = out1 + (size_t)units * nchunks * d;
    if (nchunks > 1)
        hipLaunchKernelGGL((delta_scan_chunks_kernel<T, false>), dim3(cw + (V ? L / kTB : 0), nchunks, units),
                           dim3(kWave), 0, s, (const T *)K, (T *)Khat, mask_bits, (const T *)nullptr, out1,
                           (unsigned long long *)nnz, n, d, L, nchunks, theta, (const T *)init, (const bf16_t *)V,
                           (bf16_t *)Vt, n_pad);
    hipLaunchKernelGGL((delta_scan_chunks_kernel<T, true>), dim3(cw, nchunks, units), dim3(kWave), 0, s,
                       (const T *)K, (T *)Khat, mask_bits, (const T *)out1, out2, (unsigned long long *)nnz, n, d, L,
                       nchunks, theta, (const T *)init);
    if (nchunks > 1)
        hipLaunchKernelGGL(delta_scan_fixup_kernel<T>, dim3(cw, units), dim3(kWave), 0, s, (const T *)K, (T *)Khat,
                           mask_bits, (const T *)out1, (const T *)out2, (unsigned long long *)nnz, n, d, L, nchunks,
                           theta);
}

// Khat [units][n][d] and chunk_out [2][units][delta_scan_num_chunks(n)][d] are required scratch/outputs.
// init: NULL (row 0 is the basis row) or [units][d], the reference key the rows continue from.
bool delta_scan_takes_v(int dtype, int n, int d) {
    return dtype == 1 && (d == 64 || d == 128) && delta_scan_num_chunks(n) > 1;
}

void launch_delta_scan(int dtype, const void *K, void *Khat, uint32_t *mask_bits, void *chunk_out, uint64_t *nnz,
                       int units, int n, int d, float theta, hipStream_t s, const void *init, const void *V, void *Vt,
                       int n_pad) {
    if (delta_scan_num_chunks(n) <= 1) launch_fill_u64(nnz, 0, units, s);   // (else the first pass clears them)
    if (!V || !Vt || !delta_scan_takes_v(dtype, n, d)) V = nullptr;
    if (dtype == 0)
        scan_typed<float>(K, Khat, mask_bits, chunk_out, nnz, units, n, d, theta, init, s, nullptr, nullptr, 0);
    else
        scan_typed<bf16_t>(K, Khat, mask_bits, chunk_out, nnz, units, n, d, theta, init, s, V, Vt, n_pad);
}

// ld > 0: the arrays have ld rows of room per unit (padded strides from prefill_mfma_n_pad(ld)) of which n are valid,
// and only the blocks of 32 columns from blk0 on are (re)written; ld == 0: the arrays are exactly n rows per unit.
void launch_emit_entries(int dtype, const void *K, const void *Khat, const uint32_t *mask_bits, void *ents,
                         uint32_t *counts, uint8_t *nch8, void *plan, uint32_t *dense, int units, int n, int n_pad,
                         int d, hipStream_t s, int ld, int blk0) {
    const int ld_pad = ld > 0 ? prefill_mfma_n_pad(ld) : n_pad;
    if (ld <= 0) ld = n;
    if (blk0 >= n_pad / 32) return;
    dim3 grid(n_pad / 32 - blk0, units), block(256);
    if (dtype == 0)
        hipLaunchKernelGGL(emit_entries_kernel<float>, grid, block, 0, s, (const float *)K, (const float *)Khat,
                           mask_bits, (EntryChunk *)ents, counts, nch8, (uint8_t *)plan, dense, n, ld, ld_pad, blk0, d);
    else
        hipLaunchKernelGGL(emit_entries_kernel<bf16_t>, grid, block, 0, s, (const bf16_t *)K,
                           (const bf16_t *)Khat, mask_bits, (EntryChunk *)ents, counts, nch8, (uint8_t *)plan, dense, n,
                           ld, ld_pad, blk0, d);
}

}  // namespace da
