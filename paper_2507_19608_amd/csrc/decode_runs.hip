// Decode stage for bf16 caches in the column-run layout (Sec. III-B decode stage, Sec. III-C): head_dim 64
// or 128, decode window of at least one chunk.  The compact delta cache keeps, per chunk of kChunk rows
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

// V cache, column-run layout: 16 rows per channel, [unit][t / 16][channel][16].  Inside a group of 16 the
// slot of row p is 8 k + i with k = (p / 4) % 2 and i = 4 (p / 8) + p % 4: the order in which the 32x32
// matrix-core accumulator hands 8 consecutive registers of lane half k to the next contraction.
__device__ __forceinline__ size_t v16_index(int unit, int vrows, int d, int t, int ch) {
    const int p = t & 15;
    const int slot = 8 * ((p >> 2) & 1) + 4 * (p >> 3) + (p & 3);
    return (((size_t)unit * (vrows >> 4) + (t >> 4)) * d + ch) * 16 + slot;
}

__device__ __forceinline__ bf16_t *run_room(const da_cache &c, int unit, int chunk) {
    return (bf16_t *)c.surv + ((size_t)unit * c.max_chunks + chunk) * ((size_t)(kChunk + 1) * c.d);
}

// Seals chunk `chunk` of one unit (one wave): for every channel the run {reference value held when the
// chunk starts, surviving values in row order}, runs stored one after another in channel order.
// Mp: the chunk's kChunk mask rows; rowp(r): raw key row r of the chunk; heldp(ch): reference value of
// channel ch before the chunk's first row.  lane = channel (mod 64).
template <typename RowFn, typename HeldFn>
__device__ void seal_chunk(const da_cache &c, int unit, int chunk, int lane, const uint32_t *__restrict__ Mp,
                           RowFn rowp, HeldFn heldp) {
    const int d = c.d, wpr = d >> 5;
    bf16_t *room = run_room(c, unit, chunk);
    uint32_t base = 0;
    for (int c0 = 0; c0 < d; c0 += kWave) {
        const int ch = c0 + lane;
        uint64_t cm = 0;
        for (int r = 0; r < kChunk; ++r)
            cm |= (uint64_t)((Mp[(size_t)r * wpr + (ch >> 5)] >> (ch & 31)) & 1u) << r;
        uint32_t total;
        uint32_t p = base + wave_exclusive_scan((uint32_t)__popcll(cm) + 1u, &total);
        room[p++] = heldp(ch);
        for (int r = 0; r < kChunk; ++r)
            if ((cm >> r) & 1ull) room[p++] = rowp(r)[ch];
        base += total;
    }
    if (lane == 0) c.ccnt[(size_t)unit * c.max_chunks + chunk] = base;
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

// Prefill hand-off (Sec. III-C): one wave per (chunk, unit).
__global__ __launch_bounds__(64) void cache_fill_runs_kernel(const bf16_t *__restrict__ K,
                                                             const bf16_t *__restrict__ V,
                                                             const bf16_t *__restrict__ Khat,
                                                             const uint32_t *__restrict__ mask_bits,
                                                             const uint64_t *__restrict__ nnz_in, da_cache c, int n) {
    const int chunk = blockIdx.x, unit = blockIdx.y, lane = threadIdx.x;
    const int d = c.d, wpr = d >> 5;
    const int r0 = chunk * kChunk, rows = min(kChunk, n - r0);
    const uint32_t *Mp = mask_bits + ((size_t)unit * n + r0) * wpr;
    uint32_t *Mc = c.mask + ((size_t)unit * c.max_seq + r0) * wpr;
    for (int i = lane; i < rows * wpr; i += kWave) Mc[i] = Mp[i];
    if (lane == 0 && chunk == 0) c.nnz[unit] = nnz_in[unit];
    const bf16_t *Kp = K + ((size_t)unit * n + r0) * d;
    const bf16_t *Hp = Khat + ((size_t)unit * n + r0) * d;
    const bf16_t *Vp = V + ((size_t)unit * n + r0) * d;
    for (int ch = lane; ch < d; ch += kWave) {
        for (int r = 0; r < rows; ++r) {
            const int row = r0 + r;
            if (row >= n - c.Wd) ((bf16_t *)c.ring)[((size_t)unit * c.Wd + row % c.Wd) * d + ch] = Kp[(size_t)r * d + ch];
        }
        if (chunk > 0) ((bf16_t *)c.ck)[((size_t)unit * c.nck + chunk) * d + ch] = Hp[ch - d];
        if (r0 + rows == n) ((bf16_t *)c.khat)[(size_t)unit * d + ch] = Hp[(size_t)(rows - 1) * d + ch];
        // V: 16 rows of one channel are contiguous (32 bytes per lane, consecutive lanes adjacent)
        for (int g16 = 0; g16 * 16 < rows; ++g16) {
            bf16_t v16[16];
#pragma unroll
            for (int slot = 0; slot < 16; ++slot) {
                const int k = slot >> 3, i = slot & 7;
                const int p = 8 * (i >> 2) + 4 * k + (i & 3);
                v16[slot] = (g16 * 16 + p < rows) ? Vp[(size_t)(g16 * 16 + p) * d + ch] : (bf16_t)0;
            }
            bf16_t *dst = (bf16_t *)c.V + (((size_t)unit * (c.vrows >> 4) + ((r0 >> 4) + g16)) * d + ch) * 16;
#pragma unroll
            for (int slot = 0; slot < 16; ++slot) dst[slot] = v16[slot];
        }
    }
    // complete chunks are sealed here (the run's first element comes from the prefill's reference keys)
    if (rows == kChunk)
        seal_chunk(
            c, unit, chunk, lane, Mp, [&](int r) { return Kp + (size_t)r * d; },
            [&](int ch) { return chunk > 0 ? Hp[ch - d] : (bf16_t)0; });
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

// One decode step: one wave per (chunk of kChunk cached rows, unit), all query heads of the unit's group.
//   0. the wave that owns the newest row appends it (D1);
//   1. history chunks (rows left of the decode window): the chunk's runs are copied to LDS; lane = row j
//      takes, for every channel c, element B_c + #{marked rows <= j of channel c} of the staged runs,
//      which is the reference value k_hat(j)[c] (Eq. 3) - by telescoping Eq. 4 the history score of
//      row j is q . k_hat(j).  The column mask of a channel is the wave ballot of that channel's bit in
//      the lanes' mask rows; the count is one mbcnt pair, B_c a running scalar sum of the ballots'
//      popcounts.  Reads of one instruction touch at most 65 consecutive elements: no bank conflicts.
//      Window rows (lane = row again) are 128-bit loads from the raw-key ring, the newest from k_new.
//   2. a lane now holds a whole key row; one permlane32 swap per register pair turns that into the
//      32x32x16 operand order (lane l: row l % 32, channels 16 s + 8 (l / 32)..+7 of contraction step s);
//   3. scores S[row][head] on the matrix cores (heads padded to 32 columns), softmax of the chunk in the
//      accumulator registers (lane = head, 32 rows per lane, the other 32 in lane + 32);
//   4. the accumulator registers, rounded to bf16, are the A operand of P V as they stand, because the V
//      cache stores each group of 16 rows in exactly that order; partial (o, m, l) of the chunk to scratch.
template <int D>
__global__ __launch_bounds__(64, D == 64 ? 4 : 2) void decode_step_runs_kernel(da_cache c, const bf16_t *__restrict__ q_new,
                                                              const bf16_t *__restrict__ k_new,
                                                              const bf16_t *__restrict__ v_new,
                                                              uint32_t *__restrict__ mask_row, int t,
                                                              float scale_log2) {
    extern __shared__ float lds_f[];
    bf16_t *__restrict__ sv = (bf16_t *)lds_f;               // staged runs, <= (kChunk + 1) * D elements
    constexpr int WPR = D / 32, KS = D / 16, CT = D / 32, NK = D / 2;
    constexpr int kRoom = (kChunk + 1) * D;                  // elements
    constexpr int kPieces = (kRoom + 511) / 512;             // 1 KiB copies (16 bytes per lane) that cover the room
    constexpr int kEager = D / 16;                           // copies requested before the element count is known
    const int chunk = blockIdx.x, unit = blockIdx.y, lane = threadIdx.x;
    const int nchunks = t / kChunk + 1;
    const bool newest = chunk == nchunks - 1;
    const int r0 = chunk * kChunk;
    const int nrows = min(kChunk, t + 1 - r0);
    const int g = c.Hq / c.Hkv;
    const int b = unit / c.Hkv, hk = unit % c.Hkv;
    const int hist_rows = min(max(t + 1 - c.Wd - r0, 0), nrows);   // > 0 only for sealed chunks (Wd >= kChunk)
    const int n32 = lane & 31, kap = lane >> 5;

    // ---- requests whose addresses depend on nothing loaded
    uint32_t mk[WPR];
    u32x4 sp[kEager];
    uint32_t total = 0;
    const bf16_t *runs = run_room(c, unit, chunk);
    if (hist_rows > 0) {
        const uint32_t *Mp = c.mask + ((size_t)unit * c.max_seq + r0 + lane) * WPR;
#pragma unroll
        for (int w = 0; w < WPR; ++w) mk[w] = Mp[w];
        total = c.ccnt[(size_t)unit * c.max_chunks + chunk];
#pragma unroll
        for (int p = 0; p < kEager; ++p) sp[p] = *(const u32x4 *)(runs + p * 512 + lane * 8);
    }
    // q operands of the first 32 heads (B operand of the score contraction)
    u32x4 qop[KS];
    {
        const int gh0 = g;
        const bf16_t *qrow = q_new + ((size_t)b * c.Hq + hk * g + min(n32, gh0 - 1)) * D;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            qop[s] = *(const u32x4 *)(qrow + 16 * s + 8 * kap);
            if (n32 >= gh0) qop[s] = u32x4{0u, 0u, 0u, 0u};
        }
    }
    // V operands of the whole chunk (needed last): B operand of P V, lane l = channel 32 ct + l % 32, rows of
    // lane half l / 32 of the 16-row group; the newest row is patched in from v_new
    u32x4 vop[CT][2][2];
    auto load_v = [&]() {
        const int pt = t & 15;
        const int kap_t = (pt >> 2) & 1, i_t = 4 * (pt >> 3) + (pt & 3);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const int row16 = r0 + 32 * T + 16 * s2, ch = 32 * ct + n32;
                    vop[ct][T][s2] = *(const u32x4 *)((const bf16_t *)c.V +
                                                      (((size_t)unit * (c.vrows >> 4) + (row16 >> 4)) * D + ch) * 16 + 8 * kap);
                }
        if (newest) {
            const int T = (t >> 5) & 1, s2 = (t >> 4) & 1;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const uint32_t vn = v_new[(size_t)unit * D + 32 * ct + n32];
#pragma unroll
                for (int TT = 0; TT < 2; ++TT)
#pragma unroll
                    for (int ss = 0; ss < 2; ++ss)
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            const bool hit = TT == T && ss == s2 && w == (i_t >> 1) && kap == kap_t;
                            const uint32_t old = vop[ct][TT][ss][w];
                            const uint32_t pat = (i_t & 1) ? ((old & 0xffffu) | (vn << 16)) : ((old & 0xffff0000u) | vn);
                            vop[ct][TT][ss][w] = hit ? pat : old;
                        }
            }
        }
    };
    // 0. the new row goes into the cache (other waves of this launch never read what is written here)
    if (newest) append_row_runs(c, unit, lane, k_new, v_new, mask_row, t);

    // 1. one key row per lane
    uint32_t kreg[NK];
    if (hist_rows > 0) {
#pragma unroll
        for (int p = 0; p < kEager; ++p) *(u32x4 *)(sv + p * 512 + lane * 8) = sp[p];
        for (int p = kEager; p < kPieces && (uint32_t)p * 512u < total; ++p)
            if (p * 512 + lane * 8 + 8 <= kRoom)
                *(u32x4 *)(sv + p * 512 + lane * 8) = *(const u32x4 *)(runs + p * 512 + lane * 8);
        __syncthreads();
        uint32_t run = 0;                                    // uniform: survivors of the channels before this one
        const char *svb = (const char *)sv;
#pragma unroll
        for (int ch = 0; ch < D; ch += 2) {
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
                const bf16_t *src = row == t ? k_new + (size_t)unit * D
                                             : (const bf16_t *)c.ring + ((size_t)unit * c.Wd + row % c.Wd) * D;
#pragma unroll
                for (int i = 0; i < D / 8; ++i) {
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
    }
    // 2. operand order: kop[T][s] = rows 32 T + l % 32, channels 16 s + 8 (l / 32)..+7
    u32x4 kop[2][KS];
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const auto sw = __builtin_amdgcn_permlane32_swap(kreg[8 * s + i], kreg[8 * s + 4 + i], false, false);
            kop[0][s][i] = sw[0];
            kop[1][s][i] = sw[1];
        }

    load_v();

    {
        const int hbase = 0, gh = g;                         // at most 32 query heads per KV head in this layout
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
        float m = -INFINITY;
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const bool valid = 32 * T + 8 * (r >> 2) + 4 * kap + (r & 3) < nrows;
                acc[T][r] = valid ? acc[T][r] * scale_log2 : -INFINITY;
                m = fmaxf(m, acc[T][r]);
            }
        m = fmaxf(m, __shfl_xor(m, 32));                     // row r0 is always valid, so m is finite
        float l = 0.f;
        u32x4 pa[2][2];
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const float p0 = __builtin_amdgcn_exp2f(acc[T][r] - m);
                const float p1 = __builtin_amdgcn_exp2f(acc[T][r + 1] - m);
                l += p0 + p1;
                pa[T][r >> 3][(r & 7) >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{p0, p1}, bf16x2));
            }
        l += __shfl_xor(l, 32);
        if (lane < gh) {
            float *out = c.part + (((size_t)b * c.Hq + hk * g + hbase + lane) * c.max_chunks + chunk) * part_stride(D);
            out[D] = m;
            out[D + 1] = l;
        }
        // 4. P V: heads x channels, contraction over the chunk's 64 rows in accumulator order
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            f32x16 o;
#pragma unroll
            for (int r = 0; r < 16; ++r) o[r] = 0.f;
            const int ch = 32 * ct + n32;
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
                    o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pa[T][s2]),
                                                                __builtin_bit_cast(bf16x8, vop[ct][T][s2]), o, 0, 0, 0);
            // lane l holds channel 32 ct + l % 32 of heads 8 (r / 4) + 4 (l / 32) + r % 4
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                if (8 * rq >= gh) break;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int h = 8 * rq + 4 * kap + r4;
                    if (h < gh)
                        c.part[(((size_t)b * c.Hq + hk * g + hbase + h) * c.max_chunks + chunk) * part_stride(D) + ch] =
                            o[4 * rq + r4];
                }
            }
        }
    }
}

}  // namespace

namespace da {

void cache_fill_runs(da_cache *c, int n, const void *K, const void *V, const void *Khat, const uint32_t *mask_bits,
                     const uint64_t *nnz, hipStream_t s) {
    const int units = c->B * c->Hkv;
    hipLaunchKernelGGL(cache_fill_runs_kernel, dim3((n + kChunk - 1) / kChunk, units), dim3(64), 0, s,
                       (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)Khat, mask_bits, nnz, *c, n);
}

void decode_step_runs(da_cache *c, const void *q, const void *k, const void *v, uint32_t *mask_row, int t,
                      float scale_log2, hipStream_t s) {
    const int units = c->B * c->Hkv;
    const dim3 grid(t / kChunk + 1, units), block(64);
    const size_t lds = (size_t)(kChunk + 1) * c->d * sizeof(bf16_t);
    if (c->d == 64)
        hipLaunchKernelGGL(decode_step_runs_kernel<64>, grid, block, lds, s, *c, (const bf16_t *)q, (const bf16_t *)k,
                           (const bf16_t *)v, mask_row, t, scale_log2);
    else
        hipLaunchKernelGGL(decode_step_runs_kernel<128>, grid, block, lds, s, *c, (const bf16_t *)q,
                           (const bf16_t *)k, (const bf16_t *)v, mask_row, t, scale_log2);
}

void seal_chunk_runs(da_cache *c, int chunk, hipStream_t s) {
    hipLaunchKernelGGL(seal_from_ring_kernel, dim3(c->B * c->Hkv), dim3(64), 0, s, *c, chunk);
}

}  // namespace da
