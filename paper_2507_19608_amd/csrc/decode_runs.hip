// Decode stage for bf16 caches in the column-run layout (Sec. III-B decode stage, Sec. III-C): head_dim 64
// or 128, decode window of at least one chunk (or of the whole cache).  The compact delta cache keeps, per chunk of kChunk rows
// and per channel, the run of surviving key values; a chunk is sealed into that form once, when its last
// row has arrived, while its rows are still inside the decode window.
#include <math.h>

#include "cache.hpp"
#include "common.hpp"
#include "kernels.hpp"

using namespace da;

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// V cache, column-run layout: 16 rows per channel, [unit][t / 16][channel][16].  Inside a group of 16 the
// slot of row p is 8 k + i with k = (p / 4) % 2 and i = 4 (p / 8) + p % 4: the order in which the 32x32
// matrix-core accumulator hands 8 consecutive registers of lane half k to the next contraction.
__device__ __forceinline__ size_t v16_index(int unit, int vrows, int d, int t, int ch) {
    const int p = t & 15;
    const int slot = 8 * ((p >> 2) & 1) + 4 * (p >> 3) + (p & 3);
    return (((size_t)unit * (vrows >> 4) + (t >> 4)) * d + ch) * 16 + slot;
}

__device__ __forceinline__ bf16_t *run_room(const da_cache &c, int unit, int chunk) {
    return (bf16_t *)c.surv + ((size_t)unit * c.max_chunks + chunk) * run_room_stride(c.d);
}

// The runs of channels 64.. (head_dim 128) start at a multiple of 8 elements, so that the decode step can copy
// either half of a chunk's runs with 16-byte pieces.
__device__ __forceinline__ uint32_t second_half_start(uint32_t first_half_elems) { return (first_half_elems + 7u) & ~7u; }

// Seals chunk `chunk` of one unit (one wave): for every channel the run {reference value held when the
// chunk starts, surviving values in row order}, runs stored one after another in channel order.
// Mp: the chunk's kChunk mask rows; rowp(r): raw key row r of the chunk; heldp(ch): reference value of
// channel ch before the chunk's first row.  lane = channel (mod 64).
template <typename RowFn, typename HeldFn>
__device__ void seal_chunk(const da_cache &c, int unit, int chunk, int lane, const uint32_t *__restrict__ Mp,
                           RowFn rowp, HeldFn heldp) {
    const int d = c.d, wpr = d >> 5;
    bf16_t *room = run_room(c, unit, chunk);
    uint32_t base = 0, half = 0;
    for (int c0 = 0; c0 < d; c0 += kWave) {
        const int ch = c0 + lane;
        // rows in batches of 16: all loads of a batch are issued before anything is stored, so that their latency
        // is paid once per batch, not once per row
        uint64_t cm = 0;
        for (int rb = 0; rb < kChunk; rb += 16) {
            uint32_t w[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) w[u] = Mp[(size_t)(rb + u) * wpr + (ch >> 5)];
#pragma unroll
            for (int u = 0; u < 16; ++u) cm |= (uint64_t)((w[u] >> (ch & 31)) & 1u) << (rb + u);
        }
        uint32_t total;
        uint32_t p = base + wave_exclusive_scan((uint32_t)__popcll(cm) + 1u, &total);
        room[p++] = heldp(ch);
        for (int rb = 0; rb < kChunk; rb += 16) {
            bf16_t kv[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) kv[u] = rowp(rb + u)[ch];
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if ((cm >> (rb + u)) & 1ull) room[p++] = kv[u];
        }
        base += total;
        if (c0 == 0) {
            half = base;                                     // elements of channels 0..63
            if (d > kWave) base = second_half_start(base);
        }
    }
    // low half: elements in the room (the gap included); high half: where the runs of channels 64.. start
    if (lane == 0) c.ccnt[(size_t)unit * c.max_chunks + chunk] = base | ((d > kWave ? second_half_start(half) : base) << 16);
}

// Seal from the raw-key ring: runs right after the step that appended the chunk's last row.
__global__ __launch_bounds__(64) void seal_from_ring_kernel(da_cache c, int chunk) {
    const int unit = blockIdx.x, lane = threadIdx.x;
    const int d = c.d, r0 = chunk * kChunk;
    const uint32_t *Mp = c.mask + ((size_t)unit * c.max_seq + r0) * (d >> 5);
    const bf16_t *ring = (const bf16_t *)c.ring + (size_t)unit * c.Wd * d;
    const bf16_t *ckp = (const bf16_t *)c.ck + ((size_t)unit * c.nck + chunk) * d;
    seal_chunk(
        c, unit, chunk, lane, Mp, [&](int r) { return ring + (size_t)((r0 + r) % c.Wd) * d; },
        [&](int ch) { return chunk > 0 ? ckp[ch] : (bf16_t)0; });
}

// Hand-off of prefilled rows to the cache (Sec. III-C): rows t0 .. n_k - 1 (t0 = rows the cache already
// holds) are appended; two waves per (chunk that contains such a row, unit).  Kfull, Hfull, Mfull describe the
// whole sequence [units][ld][...] (ld >= n_k rows of room per unit): keys (for rows the decode window no longer
// holds raw, the reference key stands in - the two agree wherever a mask bit is set, which is all that is read),
// reference keys, mask
// rows; Vnew [units][n_k - t0][d] the new value rows.  With t0 = 0 these are the prefill's own arrays.
__global__ __launch_bounds__(128) void cache_fill_runs_kernel(const bf16_t *__restrict__ Kfull,
                                                             const bf16_t *__restrict__ Vnew,
                                                             const bf16_t *__restrict__ Hfull,
                                                             const uint32_t *__restrict__ Mfull,
                                                             const uint64_t *__restrict__ nnz_new, da_cache c, int t0,
                                                             int n_k, int ld) {
    // two waves: wave 0 takes mask rows, raw-key ring, checkpoint, newest reference key and the chunk's runs; wave 1
    // the value rows (two chains of dependent memory round trips side by side instead of one after the other)
    const int chunk = blockIdx.x + t0 / kChunk, unit = blockIdx.y, lane = threadIdx.x & (kWave - 1);
    const bool values = threadIdx.x >= kWave;
    const int d = c.d, wpr = d >> 5, m = n_k - t0;
    const int r0 = chunk * kChunk;
    const int ra = max(r0, t0), rb = min(r0 + kChunk, n_k);          // new rows of this chunk
    const uint32_t *Mp = Mfull + ((size_t)unit * ld + r0) * wpr;     // the chunk's mask rows, old ones included
    const bf16_t *Kp = Kfull + ((size_t)unit * ld + r0) * d;
    const bf16_t *Hp = Hfull + ((size_t)unit * ld + r0) * d;
    const bf16_t *Vp = Vnew + (size_t)unit * m * d;
    if (values) {
        // V: 16 rows of one channel are contiguous.  A group that starts with a new row is written whole (32
        // bytes per lane, consecutive lanes adjacent; rows past the end as zeros), one that starts with old
        // rows only gets its new slots
        for (int ch = lane; ch < d; ch += kWave) {
            for (int g0 = r0; g0 < rb; g0 += 16) {
                if (g0 + 16 <= ra) continue;
                bf16_t *dst = (bf16_t *)c.V + (((size_t)unit * (c.vrows >> 4) + (g0 >> 4)) * d + ch) * 16;
                if (g0 >= ra) {
                    bf16_t v16[16];
#pragma unroll
                    for (int slot = 0; slot < 16; ++slot) {
                        const int k = slot >> 3, i = slot & 7;
                        const int row = g0 + 8 * (i >> 2) + 4 * k + (i & 3);
                        const bf16_t v = Vp[(size_t)(min(row, rb - 1) - t0) * d + ch];   // clamped: no conditional load
                        v16[slot] = row < rb ? v : (bf16_t)0;
                    }
#pragma unroll
                    for (int slot = 0; slot < 16; ++slot) dst[slot] = v16[slot];
                } else {
                    for (int row = ra; row < min(g0 + 16, rb); ++row)
                        ((bf16_t *)c.V)[v16_index(unit, c.vrows, d, row, ch)] = Vp[(size_t)(row - t0) * d + ch];
                }
            }
        }
        return;
    }
    uint32_t *Mc = c.mask + ((size_t)unit * c.max_seq + r0) * wpr;
    for (int i = (ra - r0) * wpr + lane; i < (rb - r0) * wpr; i += kWave) Mc[i] = Mp[i];
    if (lane == 0 && blockIdx.x == 0) c.nnz[unit] = (t0 == 0 ? 0ull : c.nnz[unit]) + nnz_new[unit];
    for (int ch = lane; ch < d; ch += kWave) {
        for (int rq = ra; rq < rb; rq += 16) {               // 16 rows at a time: loads first (clamped), then stores
            bf16_t kk[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) kk[u] = Kp[(size_t)(min(rq + u, rb - 1) - r0) * d + ch];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int row = rq + u;
                if (row < rb && row >= n_k - c.Wd)
                    ((bf16_t *)c.ring)[((size_t)unit * c.Wd + row % c.Wd) * d + ch] = kk[u];
            }
        }
        if (chunk > 0 && r0 >= t0) ((bf16_t *)c.ck)[((size_t)unit * c.nck + chunk) * d + ch] = Hp[ch - d];
        if (rb == n_k) ((bf16_t *)c.khat)[(size_t)unit * d + ch] = Hp[(size_t)(rb - 1 - r0) * d + ch];
    }
    // chunks completed by these rows are sealed here (the run's first element comes from the reference keys)
    if (rb - r0 == kChunk)
        seal_chunk(
            c, unit, chunk, lane, Mp, [&](int r) { return Kp + (size_t)r * d; },
            [&](int ch) { return chunk > 0 ? Hp[ch - d] : (bf16_t)0; });
}

// The inverse of the hand-off, for a prefill that continues a cached sequence: rows 0 .. t0 - 1 of the cache
// are written out as plain arrays [units][ld][...] (ld >= t0 rows of room per unit): reference keys (from
// the sealed runs, or for the unsealed last chunk from the ring), keys (raw for the rows the ring still
// holds, the reference key otherwise), values, mask rows.  One wave per (chunk, unit), lane = channel.
__global__ __launch_bounds__(64) void expand_cache_kernel(da_cache c, int t0, int ld, bf16_t *__restrict__ Kfull,
                                                          bf16_t *__restrict__ Hfull, bf16_t *__restrict__ Vfull,
                                                          uint32_t *__restrict__ Mfull) {
    const int chunk = blockIdx.x, unit = blockIdx.y, lane = threadIdx.x;
    const int d = c.d, wpr = d >> 5;
    const int r0 = chunk * kChunk, rows = min(kChunk, t0 - r0);
    const bool sealed = rows == kChunk;
    const uint32_t *Mp = c.mask + ((size_t)unit * c.max_seq + r0) * wpr;
    for (int i = lane; i < rows * wpr; i += kWave) Mfull[((size_t)unit * ld + r0) * wpr + i] = Mp[i];
    const bf16_t *room = run_room(c, unit, chunk);
    const bf16_t *ring = (const bf16_t *)c.ring + (size_t)unit * c.Wd * d;
    uint32_t base = 0;
    for (int c0 = 0; c0 < d; c0 += kWave) {
        const int ch = c0 + lane;
        // rows in batches of 16 (one group of the V layout): all loads of a batch are issued before anything is
        // stored, so that their latency is paid once per batch, not once per row
        uint64_t cm = 0;
        for (int rb = 0; rb < rows; rb += 16) {
            uint32_t w[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) w[u] = Mp[(size_t)min(rb + u, rows - 1) * wpr + (ch >> 5)];   // clamped: branch-free
#pragma unroll
            for (int u = 0; u < 16; ++u) cm |= (uint64_t)(rb + u < rows ? (w[u] >> (ch & 31)) & 1u : 0u) << (rb + u);
        }
        uint32_t total = 0, p = 0;
        bf16_t held = 0;
        if (sealed) {
            p = base + wave_exclusive_scan((uint32_t)__popcll(cm) + 1u, &total);
            held = room[p];
        } else if (chunk > 0) {
            held = ((const bf16_t *)c.ck)[((size_t)unit * c.nck + chunk) * d + ch];
        }
        for (int rb = 0; rb < rows; rb += 16) {
            bf16_t kraw[16], sv[16];
            // the 16 values of this channel and row group are contiguous in the V cache, in slot order
            const u32x4 *vp = (const u32x4 *)((const bf16_t *)c.V + (((size_t)unit * (c.vrows >> 4) + ((r0 + rb) >> 4)) * d + ch) * 16);
            const u32x4 v0 = vp[0], v1 = vp[1];
            const uint32_t bits = (uint32_t)(cm >> rb) & 0xffffu;      // the batch's mask bits of this channel
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int r = rb + u, row = r0 + r;
                // every load is in bounds whatever the row (ring slot of any position; p stays inside the room), so
                // none of them is conditional and all of a batch are in flight together
                kraw[u] = ring[(size_t)(row % c.Wd) * d + ch];
                p += (bits >> u) & 1u;                                      // p: position of the newest survivor
                sv[u] = room[p];
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int r = rb + u, row = r0 + r;
                const bool raw_here = row >= t0 - c.Wd;                     // always true for an unsealed chunk
                if ((bits >> u) & 1u) held = sealed ? sv[u] : kraw[u];
                const int slot = 8 * ((u >> 2) & 1) + 4 * (u >> 3) + (u & 3);
                const uint32_t vw = slot < 8 ? v0[slot >> 1] : v1[(slot - 8) >> 1];
                const size_t o = ((size_t)unit * ld + row) * d + ch;
                if (r < rows) {
                    Hfull[o] = held;
                    Kfull[o] = raw_here ? kraw[u] : held;
                    Vfull[o] = (bf16_t)((slot & 1) ? vw >> 16 : vw & 0xffffu);
                }
            }
        }
        base += total;
        if (c0 == 0 && d > kWave) base = second_half_start(base);
    }
}

// D1: delta of the new key against the carried reference key (Eq. 2-3).  One wave per unit.  The
// surviving values themselves are already in the raw-key ring; the run is built when the chunk is sealed.
__device__ void append_row_runs(const da_cache &c, int unit, int lane, const bf16_t *__restrict__ k_new,
                                const bf16_t *__restrict__ v_new, uint32_t *__restrict__ mask_row, int t) {
    const int d = c.d, wpr = d >> 5;
    const int chunk = t / kChunk;
    uint32_t fired = 0;
    for (int c0 = 0; c0 < d; c0 += kWave) {
        const int ch = c0 + lane;
        const bf16_t kraw = k_new[(size_t)unit * d + ch];
        bf16_t *hp = (bf16_t *)c.khat + (size_t)unit * d + ch;
        bool fire = true;   // basis row
        if (t > 0) {
            const bf16_t hraw = *hp;
            fire = fabsf(bf16_to_f32(kraw) - bf16_to_f32(hraw)) > c.theta;
            if (t % kChunk == 0) ((bf16_t *)c.ck)[((size_t)unit * c.nck + chunk) * d + ch] = hraw;
        }
        if (fire) *hp = kraw;
        ((bf16_t *)c.ring)[((size_t)unit * c.Wd + t % c.Wd) * d + ch] = kraw;
        ((bf16_t *)c.V)[v16_index(unit, c.vrows, d, t, ch)] = v_new[(size_t)unit * d + ch];
        const uint64_t b = __ballot(fire);
        if ((lane & 31) == 0) {
            const uint32_t w = (uint32_t)(b >> (lane & 32));
            c.mask[((size_t)unit * c.max_seq + t) * wpr + (ch >> 5)] = w;
            if (mask_row) mask_row[(size_t)unit * wpr + (ch >> 5)] = w;
        }
        fired += __popcll(b);
    }
    if (lane == 0) c.nnz[unit] = (t == 0 ? 0ull : c.nnz[unit]) + fired;
}

// One decode step: per (run of `nc` consecutive chunks, unit) one wave at head_dim 64, two waves at head_dim
// 128 that each take 64 of the channels (all query heads of the unit's group either way).
// A wave walks its chunks in order with flash-style running (max, sum, output) in registers, and asks for
// the next chunk's mask rows and runs while it works on the current one; a launch is sized so that all of
// its waves are resident at once (work-group dispatch, not memory, bounds a launch of one chunk per wave).
// Per chunk:
//   0. the wave that owns the newest row appends it (D1);
//   1. history chunks (rows left of the decode window): the runs of the wave's 64 channels are copied to LDS;
//      lane = row j takes, for every channel c, element B_c + #{marked rows <= j of channel c} of the staged
//      runs, which is the reference value k_hat(j)[c] (Eq. 3) - by telescoping Eq. 4 the history score of
//      row j is q . k_hat(j).  The column mask of a channel is the wave ballot of that channel's bit in
//      the lanes' mask rows; the count is one mbcnt pair, B_c a running scalar sum of the ballots'
//      popcounts.  Reads of one instruction touch at most 65 consecutive elements: no bank conflicts.
//      Window rows (lane = row again) are 128-bit loads from the raw-key ring, the newest from k_new.
//   2. a lane now holds 64 channels of a key row; one permlane32 swap per register pair turns that into the
//      32x32x16 operand order (lane l: row l % 32, channels 16 s + 8 (l / 32)..+7 of contraction step s);
//   3. scores S[row][head] on the matrix cores (heads padded to 32 columns); at head_dim 128 the two waves
//      exchange their halves of the contraction through LDS and both hold the full scores; softmax update in
//      the accumulator registers (lane = head, 32 rows per lane, the other 32 in lane + 32);
//   4. the accumulator registers, rounded to bf16, are the B operand of O^T += V^T P^T as they stand, because
//      the V cache stores each group of 16 rows in exactly that order; O^T (the wave's 64 channels) keeps
//      lane = head, so the running rescale needs no cross-lane traffic.
// The wave's (o, m, l) goes to scratch and a second launch merges the partials of a head - or, with NW > 1
// (head_dim 64), the waves of the work group hold every row of the unit and merge in LDS.
template <int D, int NW>
__global__ __launch_bounds__(64 * NW * (D / 64), 2) void decode_step_runs_kernel(da_cache c, const bf16_t *__restrict__ q_new,
                                                                              const bf16_t *__restrict__ k_new,
                                                                              const bf16_t *__restrict__ v_new,
                                                                              bf16_t *__restrict__ o_out,
                                                                              uint32_t *__restrict__ mask_row, int t,
                                                                              float scale_log2, int nc) {
    constexpr int H = D / 64;                                // waves that share a chunk, 64 channels each
    static_assert(H == 1 || NW == 1, "the on-chip merge is built for head_dim 64");
    constexpr int WPR = D / 32;                              // mask words per row
    constexpr int KS = 4, CT = 2, NK = 32;                   // per wave: contraction steps, output tiles, kreg pairs
    constexpr int kPieces = ((kChunk + 1) * 64 + 511) / 512; // 1 KiB copies (16 bytes per lane) that cover 64 channels' runs
    // two staging areas for the runs of a chunk, used in turn: separate arrays, so that reads of one are known
    // not to touch the other while its copy is still in flight
    __shared__ __attribute__((aligned(16))) bf16_t stage_a_all[NW * H][kPieces * 512];
    __shared__ __attribute__((aligned(16))) bf16_t stage_b_all[NW * H][kPieces * 512];
    __shared__ float ml_all[NW][32][2];
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wave = wv / H, half = wv % H, coff = 64 * half;   // part inside the work group; channel half
    bf16_t *stage_a = stage_a_all[wv], *stage_b = stage_b_all[wv];
    const int part_i = blockIdx.x * NW + wave, unit = blockIdx.y, lane = threadIdx.x & 63;
    const int nchunks = t / kChunk + 1;
    // the wave's chunks: c_begin, c_begin + c_step, ... below c_end.  Single walkers take nc consecutive chunks;
    // the NW walkers of one work group take every NW-th chunk, which spreads an uneven chunk count (and the
    // cheaper window chunks at the end) evenly over the waves and so over the SIMDs
    const int c_step = NW > 1 ? NW : 1;
    const int c_begin = NW > 1 ? wave : part_i * nc, c_end = NW > 1 ? nchunks : min(c_begin + nc, nchunks);
    const int g = c.Hq / c.Hkv;                              // <= 32 in this layout
    const int b = unit / c.Hkv, hk = unit % c.Hkv;
    const int n32 = lane & 31, kap = lane >> 5;
    const int win_begin = t + 1 - c.Wd;
    // rows of chunk ch left of the decode window (> 0 only for sealed chunks, because Wd >= kChunk)
    auto hist_of = [&](int ch) { return min(max(win_begin - ch * kChunk, 0), min(kChunk, t + 1 - ch * kChunk)); };

    // q operands (B operand of the score contraction): lane l = head l % 32, channels coff + 16 s + 8 (l / 32)..+7
    u32x4 qop[KS];
    {
        const bf16_t *qrow = q_new + ((size_t)b * c.Hq + hk * g + min(n32, g - 1)) * D + coff;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            qop[s] = *(const u32x4 *)(qrow + 16 * s + 8 * kap);
            if (n32 >= g) qop[s] = u32x4{0u, 0u, 0u, 0u};
        }
    }
    // History chunk ch: the runs of this wave's channels go straight from global memory to the LDS staging area
    // (128-bit LDS-direct loads: lane i of a copy lands at base + 16 i); its mask rows, lane = row.
    // cnt: the chunk's packed element counts (elements in the room | start of the runs of channels 64.. << 16).
    auto copy_runs = [&](int ch, uint32_t cnt, bf16_t *sv) {
        const uint32_t total = cnt & 0xffffu, second = cnt >> 16;
        const uint32_t first = half ? second : 0u;                       // where this wave's runs start (a multiple of 8)
        const uint32_t len = H == 1 ? total : (half ? total - second : second);
        const bf16_t *runs = run_room(c, unit, ch) + first;
#pragma unroll
        for (int p = 0; p < kPieces; ++p)
            if ((uint32_t)p * 512u < len && first + p * 512 + lane * 8 + 8 <= (uint32_t)run_room_stride(D))
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(runs + p * 512 + lane * 8),
                                                 (__attribute__((address_space(3))) void *)(sv + p * 512), 16, 0, 0);
    };
    auto total_of = [&](int ch) -> uint32_t {
        return hist_of(ch) > 0 ? __builtin_amdgcn_readfirstlane(c.ccnt[(size_t)unit * c.max_chunks + ch]) : 0u;
    };
    uint32_t mk_n[2];
    auto request_masks = [&](int ch) {
        if (hist_of(ch) > 0) {
            const uint32_t *Mp = c.mask + ((size_t)unit * c.max_seq + ch * kChunk + lane) * WPR + 2 * half;
#pragma unroll
            for (int w = 0; w < 2; ++w) mk_n[w] = Mp[w];
        }
    };
    if (c_begin < c_end) {
        copy_runs(c_begin, total_of(c_begin), stage_a);
        request_masks(c_begin);
    }
    uint32_t tot_v = 0;                                      // element counts of the chunk after the next one's copy
    if (c_begin + c_step < c_end && hist_of(c_begin + c_step) > 0)
        tot_v = c.ccnt[(size_t)unit * c.max_chunks + c_begin + c_step];

    f32x16 o[CT];                                            // O^T: lane = head, register r of tile ct =
#pragma unroll                                               // channel coff + 32 ct + 8 (r / 4) + 4 (l / 32) + r % 4
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[ct][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;                    // l_run: this lane half's share of the sum

    auto do_chunk = [&](int chunk, bf16_t *sv, bf16_t *sv_next, const bf16_t *sv_partner) {
        const bool newest = chunk == nchunks - 1;            // this wave owns row t
        const int r0 = chunk * kChunk;
        const int nrows = min(kChunk, t + 1 - r0);
        const int hist_rows = hist_of(chunk);
        __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): this chunk's runs have landed in LDS
        // the next chunk's runs and mask rows, and the element count of the one after it, fly in meanwhile
        uint32_t mk[2];
#pragma unroll
        for (int w = 0; w < 2; ++w) mk[w] = mk_n[w];
        if (chunk + c_step < c_end) {
            copy_runs(chunk + c_step, __builtin_amdgcn_readfirstlane(tot_v), sv_next);
            request_masks(chunk + c_step);
            tot_v = 0;
            if (chunk + 2 * c_step < c_end && hist_of(chunk + 2 * c_step) > 0)
                tot_v = c.ccnt[(size_t)unit * c.max_chunks + chunk + 2 * c_step];
        }
        // V operands of the chunk (needed last, requested first): lane l = channel coff + 32 ct + l % 32, rows of
        // lane half l / 32 of each 16-row group; the newest row is patched in from v_new
        u32x4 vop[CT][2][2];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const int row16 = r0 + 32 * T + 16 * s2, ch = coff + 32 * ct + n32;
                    vop[ct][T][s2] = *(const u32x4 *)((const bf16_t *)c.V +
                                                      (((size_t)unit * (c.vrows >> 4) + (row16 >> 4)) * D + ch) * 16 + 8 * kap);
                }
        if (newest) {
            // position, unit and lane are made opaque here so that the select conditions and the addresses of the
            // append are worked out inside this branch, once per step, instead of being kept in registers across
            // the whole chunk loop
            int tt = t, uo = unit, ln = lane;
            asm volatile("" : "+s"(tt), "+s"(uo), "+v"(ln));
            const int pt = tt & 15;
            const int kap_t = (pt >> 2) & 1, i_t = 4 * (pt >> 3) + (pt & 3);
            const int Tn = (tt >> 5) & 1, sn = (tt >> 4) & 1;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const uint32_t vn = v_new[(size_t)uo * D + coff + 32 * ct + (ln & 31)];
#pragma unroll
                for (int TT = 0; TT < 2; ++TT)
#pragma unroll
                    for (int ss = 0; ss < 2; ++ss)
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            const bool hit = TT == Tn && ss == sn && w == (i_t >> 1) && kap == kap_t;
                            const uint32_t old = vop[ct][TT][ss][w];
                            const uint32_t pat = (i_t & 1) ? ((old & 0xffffu) | (vn << 16)) : ((old & 0xffff0000u) | vn);
                            vop[ct][TT][ss][w] = hit ? pat : old;
                        }
            }
            // 0. the new row goes into the cache (other waves of this launch never read what is written here)
            if (half == 0) append_row_runs(c, uo, ln, k_new, v_new, mask_row, tt);
        }

        // 1. 64 channels of one key row per lane
        uint32_t kreg[NK];
        if (hist_rows > 0) {
            uint32_t run = 0;                                // uniform: survivors of the channels before this one
            const char *svb = (const char *)sv;
#pragma unroll
            for (int ch = 0; ch < 64; ch += 2) {
                uint32_t val[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const uint32_t bit = (mk[(ch + e) >> 5] >> ((ch + e) & 31)) & 1u;
                    const uint64_t cm = __ballot(bit != 0u);
                    const uint32_t idx =
                        __builtin_amdgcn_mbcnt_hi((uint32_t)(cm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)cm, bit));
                    val[e] = *(const bf16_t *)(svb + ((idx + run) << 1) + 2 * (ch + e));   // run start = run + ch + e
                    run += (uint32_t)__popcll(cm);
                }
                kreg[ch >> 1] = val[0] | (val[1] << 16);
            }
        }
        if (hist_rows < kChunk) {
            if (lane >= hist_rows) {
                if (lane < nrows) {
                    const int row = r0 + lane;
                    const bf16_t *src = (row == t ? k_new + (size_t)unit * D
                                                  : (const bf16_t *)c.ring + ((size_t)unit * c.Wd + row % c.Wd) * D) + coff;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const u32x4 v = *(const u32x4 *)(src + 8 * i);
                        kreg[4 * i] = v[0];
                        kreg[4 * i + 1] = v[1];
                        kreg[4 * i + 2] = v[2];
                        kreg[4 * i + 3] = v[3];
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < NK; ++i) kreg[i] = 0u;
                }
            }
            // the raw rows are awaited here, inside the branch only window chunks take: left to the compiler the
            // wait lands after the join and history chunks would drain their in-flight V and run copies there
            __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0)
        }
        // 2. operand order: kop[T][s] = rows 32 T + l % 32, channels coff + 16 s + 8 (l / 32)..+7
        u32x4 kop[2][KS];
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const auto sw = __builtin_amdgcn_permlane32_swap(kreg[8 * s + i], kreg[8 * s + 4 + i], false, false);
                kop[0][s][i] = sw[0];
                kop[1][s][i] = sw[1];
            }
        // 3. scores: lane l holds head l % 32 at rows 32 T + 8 (r / 4) + 4 (l / 32) + r % 4
        f32x16 acc[2];
#pragma unroll
        for (int T = 0; T < 2; ++T) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[T][r] = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s)
                acc[T] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kop[T][s]),
                                                                 __builtin_bit_cast(bf16x8, qop[s]), acc[T], 0, 0, 0);
        }
        if (H == 2) {
            // the other wave contracted the other 64 channels: the halves meet in the staging areas both waves have
            // just finished reading (register r of lane l at float 64 r + l: conflict free), and are added in the
            // same order by both, so both hold the same scores
            float *mine = (float *)sv;
            const float *theirs = (const float *)sv_partner;
            lds_barrier();                                   // both waves are done gathering from these areas
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r) mine[(16 * T + r) * 64 + lane] = acc[T][r];
            lds_barrier();
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float x = theirs[(16 * T + r) * 64 + lane];
                    acc[T][r] = half ? x + acc[T][r] : acc[T][r] + x;
                }
            lds_barrier();                                   // the areas may be copied into again
        }
        if (nrows < kChunk) {                                // only the newest chunk has rows that do not exist yet
            const int lim = nrows - 4 * kap;                     // compared with constants: nothing to keep in registers
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (32 * T + 8 * (r >> 2) + (r & 3) >= lim) acc[T][r] = -INFINITY;
        }
        float mx = acc[0][0];
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[T][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));                  // row r0 of a chunk is always valid, so mx is finite
        const float m = fmaxf(m_run, mx * scale_log2);       // running maximum in log2 units (the scale is positive)
        if (__any(m > m_run)) {
            const float alpha = __builtin_amdgcn_exp2f(m_run - m);   // first chunk: exp2(-inf) = 0 on zeros
            l_run *= alpha;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) o[ct] *= alpha;
            m_run = m;
        }
        u32x4 pa[2][2];
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(acc[T][r], scale_log2, -m));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(acc[T][r + 1], scale_log2, -m));
                // the sum runs over the probabilities as rounded to bf16, the weights P V uses: their rounding
                // then cannot bias the weighted mean
                const bf16x2 pk = __builtin_convertvector(f32x2{p0, p1}, bf16x2);
                l_run = __builtin_amdgcn_fdot2_f32_bf16(pk, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l_run, false);
                pa[T][r >> 3][(r & 7) >> 1] = __builtin_bit_cast(uint32_t, pk);
            }
        // 4. O^T += V^T P^T: channels x heads, contraction over the chunk's 64 rows in accumulator order
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
                    o[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vop[ct][T][s2]),
                                                                    __builtin_bit_cast(bf16x8, pa[T][s2]), o[ct], 0, 0, 0);
    };
    const bf16_t *partner_a = stage_a_all[wv ^ (H - 1)], *partner_b = stage_b_all[wv ^ (H - 1)];
    for (int chunk = c_begin; chunk < c_end; chunk += 2 * c_step) {
        do_chunk(chunk, stage_a, stage_b, partner_a);
        if (chunk + c_step < c_end) do_chunk(chunk + c_step, stage_b, stage_a, partner_b);
    }
    const float l_all = l_run + __shfl_xor(l_run, 32);
    if (NW == 1) {
        // partial (o, m, l) of this wave's rows and channels, merged by a second launch
        if (n32 < g) {
            float *out = c.part + (((size_t)b * c.Hq + hk * g + n32) * c.max_chunks + part_i) * part_stride(D);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq)
                    *(f32x4 *)(out + coff + 32 * ct + 8 * rq + 4 * kap) =
                        f32x4{o[ct][4 * rq], o[ct][4 * rq + 1], o[ct][4 * rq + 2], o[ct][4 * rq + 3]};
            if (kap == 0 && half == 0) {
                out[D] = m_run;
                out[D + 1] = l_all;
            }
        }
    } else {
        // the work group holds every row of the unit: its waves' (o, m, l) meet in LDS and the normalised
        // output row of each head is written here (a wave without chunks contributes m = -inf, l = 0)
        float *obuf = (float *)stage_a;                      // [g][D] of this wave; its staging areas are idle now
        if (n32 < g) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq)
                    *(f32x4 *)(obuf + n32 * D + 32 * ct + 8 * rq + 4 * kap) =
                        f32x4{o[ct][4 * rq], o[ct][4 * rq + 1], o[ct][4 * rq + 2], o[ct][4 * rq + 3]};
            if (kap == 0) {
                ml_all[wave][n32][0] = m_run;
                ml_all[wave][n32][1] = l_all;
            }
        }
        __syncthreads();
        for (int e = threadIdx.x; e < g * D; e += 64 * NW) {
            const int h = e / D;
            float M = -INFINITY;
#pragma unroll
            for (int w = 0; w < NW; ++w) M = fmaxf(M, ml_all[w][h][0]);
            float L = 0.f, O = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float f = __builtin_amdgcn_exp2f(ml_all[w][h][0] - M);   // wave 0 always has rows: M is finite
                L = fmaf(f, ml_all[w][h][1], L);
                O = fmaf(f, ((const float *)stage_a_all[w])[e], O);
            }
            o_out[((size_t)b * c.Hq + hk * g) * D + e] = f32_to_bf16(O / L);
        }
    }
}

}  // namespace

namespace da {

void cache_fill_runs(da_cache *c, int t0, int n_k, int ld, const void *Kfull, const void *Vnew, const void *Hfull,
                     const uint32_t *Mfull, const uint64_t *nnz_new, hipStream_t s) {
    const int units = c->B * c->Hkv;
    const int chunks = (n_k + kChunk - 1) / kChunk - t0 / kChunk;
    hipLaunchKernelGGL(cache_fill_runs_kernel, dim3(chunks, units), dim3(2 * kWave), 0, s, (const bf16_t *)Kfull,
                       (const bf16_t *)Vnew, (const bf16_t *)Hfull, Mfull, nnz_new, *c, t0, n_k, ld);
}

void expand_cache_runs(da_cache *c, int t0, int ld, void *Kfull, void *Hfull, void *Vfull, uint32_t *Mfull,
                       hipStream_t s) {
    if (t0 <= 0) return;
    hipLaunchKernelGGL(expand_cache_kernel, dim3((t0 + kChunk - 1) / kChunk, c->B * c->Hkv), dim3(64), 0, s, *c, t0,
                       ld, (bf16_t *)Kfull, (bf16_t *)Hfull, (bf16_t *)Vfull, Mfull);
}

int decode_step_runs(da_cache *c, const void *q, const void *k, const void *v, void *o, uint32_t *mask_row, int t,
                     float scale_log2, hipStream_t s) {
    const int units = c->B * c->Hkv, nchunks = t / kChunk + 1;
    // A launch is sized so that all of its waves are resident at once: 4 SIMDs per CU, 2 waves per SIMD by the
    // kernel's registers and LDS.  At head_dim 128 two waves share every chunk, so half as many chunk walkers fit.
    if (c->cus < 1 &&
        (hipDeviceGetAttribute(&c->cus, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess || c->cus < 1))
        c->cus = 256;
    const int cus = c->cus;
    const int slots = (c->plan_slots > 0 ? c->plan_slots : cus * 8) / (c->d == 64 ? 1 : 2);
    const bf16_t *qq = (const bf16_t *)q, *kk = (const bf16_t *)k, *vv = (const bf16_t *)v;
    // head_dim 64: one 8-wave work group per unit whose waves split the unit's chunks and merge in LDS (the
    // normalised output is written by this launch; returns 0: nothing left to merge) pays when its waves fill the
    // wave slots: measured over 64..512 units with the caches read from HBM, it wins from 3/4 of the slots on and
    // loses to single-wave work groups (which spread any unit count over every SIMD) below that.
    if (c->d == 64) {
        const int nw = 8;
        const int64_t waves = (int64_t)units * nw;
        const bool fills = waves * 4 >= (int64_t)slots * 3;
        if (c->plan_merge == 1 || (c->plan_merge < 0 && fills)) {
            const int nc = (nchunks + nw - 1) / nw;
            hipLaunchKernelGGL((decode_step_runs_kernel<64, 8>), dim3(1, units), dim3(64 * nw), 0, s, *c, qq, kk, vv,
                               (bf16_t *)o, mask_row, t, scale_log2, nc);
            return 0;
        }
    }
    // otherwise one chunk walker (1 or 2 waves) per work group, as few chunks each as keep the launch resident;
    // partial rows
    int nc = (int)(((int64_t)units * nchunks + slots - 1) / max(slots, 1));
    if (nc < 1) nc = 1;
    const int nparts = (nchunks + nc - 1) / nc;
    const dim3 grid(nparts, units);
    if (c->d == 64)
        hipLaunchKernelGGL((decode_step_runs_kernel<64, 1>), grid, dim3(64), 0, s, *c, qq, kk, vv, (bf16_t *)o, mask_row,
                           t, scale_log2, nc);
    else
        hipLaunchKernelGGL((decode_step_runs_kernel<128, 1>), grid, dim3(128), 0, s, *c, qq, kk, vv, (bf16_t *)o,
                           mask_row, t, scale_log2, nc);
    return nparts;
}

void seal_chunk_runs(da_cache *c, int chunk, hipStream_t s) {
    hipLaunchKernelGGL(seal_from_ring_kernel, dim3(c->B * c->Hkv), dim3(64), 0, s, *c, chunk);
}

}  // namespace da
