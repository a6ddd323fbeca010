// Decode stage (Sec. III-B decode stage, Sec. III-C): cache object, append of the new key's delta
// row, history scores from the compact delta cache, window scores from the raw-key ring, softmax, PV.
#include <math.h>
#include <new>
#include <string.h>

#include "cache.hpp"
#include "common.hpp"
#include "kernels.hpp"

using namespace da;

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

inline size_t elt_size(int dtype) { return dtype == DA_F32 ? 4 : 2; }

// V cache layout: 8 rows interleaved per channel, [unit][t / 8][channel][t % 8], so that eight
// consecutive rows of one channel are contiguous (the k-contiguous operand order of the matrix
// cores).  vrows = row capacity (max_seq rounded up to a whole chunk).
__device__ __forceinline__ size_t v_index(int unit, int vrows, int d, int t, int ch) {
    return ((size_t)unit * (vrows >> 3) + (t >> 3)) * ((size_t)d * 8) + (size_t)ch * 8 + (t & 7);
}

// surviving key values of one chunk of kChunk rows: row after row, channel order, room of (kChunk + 1) * d
template <typename T>
__device__ __forceinline__ T *surv_chunk(const da_cache &c, int unit, int chunk) {
    return (T *)c.surv + ((size_t)unit * c.max_chunks + chunk) * run_room_stride(c.d);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v = fmaxf(v, __shfl_xor(v, s));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s);
    return v;
}
// ---------------------------------------------------------------------------------- cache fill
// Prefill hand-off (Sec. III-C): one wave per (chunk of kChunk rows, unit) turns the prefill's mask rows,
// keys, reference keys and values into the cache layout.
template <typename T>
__global__ __launch_bounds__(64) void cache_fill_kernel(const T *__restrict__ K, const T *__restrict__ V,
                                                        const T *__restrict__ Khat,
                                                        const uint32_t *__restrict__ mask_bits,
                                                        const uint64_t *__restrict__ nnz_in, da_cache c, int n) {
    const int chunk = blockIdx.x, unit = blockIdx.y, lane = threadIdx.x;
    const int d = c.d, wpr = d >> 5;
    const int r0 = chunk * kChunk, rows = min(kChunk, n - r0);
    const uint32_t *Mp = mask_bits + ((size_t)unit * n + r0) * wpr;
    uint32_t *Mc = c.mask + ((size_t)unit * c.max_seq + r0) * wpr;
    // lane = row: mask copy, number of survivors of the row, start of the row inside the chunk
    uint32_t cnt = 0;
    if (lane < rows)
        for (int w = 0; w < wpr; ++w) {
            const uint32_t m = Mp[(size_t)lane * wpr + w];
            Mc[(size_t)lane * wpr + w] = m;
            cnt += __popc(m);
        }
    uint32_t total;
    const uint32_t offv = wave_exclusive_scan(cnt, &total);
    if (lane == 0) {
        c.ccnt[(size_t)unit * c.max_chunks + chunk] = total;
        if (chunk == 0) c.nnz[unit] = nnz_in[unit];
    }
    // lane = channel
    T *surv = surv_chunk<T>(c, unit, chunk);
    const T *Kp = K + ((size_t)unit * n + r0) * d;
    const T *Hp = Khat + ((size_t)unit * n + r0) * d;
    const T *Vp = V + ((size_t)unit * n + r0) * d;
    for (int r = 0; r < rows; ++r) {
        uint32_t off = __builtin_amdgcn_readlane(offv, r);
        const int row = r0 + r;
        for (int c0 = 0; c0 < d; c0 += kWave) {
            const int ch = c0 + lane;
            const bool act = ch < d;
            bool bit = false;
            if (act) bit = (Mp[(size_t)r * wpr + (ch >> 5)] >> (ch & 31)) & 1u;
            const uint64_t b = __ballot(bit);
            if (act) {
                const T k = Kp[(size_t)r * d + ch];
                if (bit) surv[off + lanes_below(b)] = k;
                if (row >= n - c.Wd) ((T *)c.ring)[((size_t)unit * c.Wd + row % c.Wd) * d + ch] = k;
                if (r == 0 && chunk > 0) ((T *)c.ck)[((size_t)unit * c.nck + chunk) * d + ch] = Hp[ch - d];
                if (row == n - 1) ((T *)c.khat)[(size_t)unit * d + ch] = Hp[(size_t)r * d + ch];
            }
            off += __popcll(b);
        }
    }
    // V: 8 rows of one channel are contiguous in the cache
    for (int g8 = 0; g8 * 8 < rows; ++g8)
        for (int ch = lane; ch < d; ch += kWave) {
            T v8[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v8[e] = (g8 * 8 + e < rows) ? Vp[(size_t)(g8 * 8 + e) * d + ch] : (T)0;
            T *dst = (T *)c.V + v_index(unit, c.vrows, d, r0 + g8 * 8, ch);
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[e] = v8[e];
        }
}

// ---------------------------------------------------------------------------------- decode step
// D1: delta of the new key against the carried reference key (Eq. 2-3), appended to the compact cache.
// Executed by one wave per unit.
template <typename T>
__device__ void append_row(const da_cache &c, int unit, int lane, const T *__restrict__ k_new,
                           const T *__restrict__ v_new, uint32_t *__restrict__ mask_row, int t) {
    const int d = c.d, wpr = d >> 5;
    const int chunk = t / kChunk;
    T *surv = surv_chunk<T>(c, unit, chunk);
    uint32_t *cc = c.ccnt + (size_t)unit * c.max_chunks + chunk;
    const uint32_t start = (t % kChunk == 0) ? 0u : *cc;
    uint32_t off = start;
    for (int c0 = 0; c0 < d; c0 += kWave) {
        const int ch = c0 + lane;
        const bool act = ch < d;
        bool fire = false;
        T kraw = 0;
        if (act) {
            kraw = k_new[(size_t)unit * d + ch];
            T *hp = (T *)c.khat + (size_t)unit * d + ch;
            if (t == 0) {
                fire = true;   // basis row
            } else {
                const T hraw = *hp;
                const float diff = load_f32(&kraw, 0) - load_f32(&hraw, 0);
                fire = fabsf(diff) > c.theta;
                if (t % kChunk == 0) ((T *)c.ck)[((size_t)unit * c.nck + chunk) * d + ch] = hraw;
            }
            if (fire) *hp = kraw;
            ((T *)c.ring)[((size_t)unit * c.Wd + t % c.Wd) * d + ch] = kraw;
            ((T *)c.V)[v_index(unit, c.vrows, d, t, ch)] = v_new[(size_t)unit * d + ch];
        }
        const uint64_t b = __ballot(fire);
        if (fire) surv[off + lanes_below(b)] = kraw;
        if (act && (lane & 31) == 0) {
            const uint32_t w = (uint32_t)(b >> (lane & 32));
            c.mask[((size_t)unit * c.max_seq + t) * wpr + (ch >> 5)] = w;
            if (mask_row) mask_row[(size_t)unit * wpr + (ch >> 5)] = w;
        }
        off += __popcll(b);
    }
    if (lane == 0) {
        *cc = off;
        c.nnz[unit] = (t == 0 ? 0ull : c.nnz[unit]) + (off - start);
    }
}

template <typename T>
__global__ __launch_bounds__(64) void decode_append_kernel(da_cache c, const T *__restrict__ k_new,
                                                           const T *__restrict__ v_new,
                                                           uint32_t *__restrict__ mask_row, int t) {
    append_row<T>(c, blockIdx.x, threadIdx.x, k_new, v_new, mask_row, t);
}

// D2-D4, generic (fp32 caches): one wave per chunk of kChunk cached rows of one unit, vector ALU only.
// Phase A (lanes = channels): rebuild the reference keys k_hat(j) of the chunk from the chunk's
// checkpoint, the mask bits and the surviving values; by telescoping Eq. 4 the history score of
// row j is q . k_hat(j).  Phase B (lanes = rows): scores (raw-key ring inside the window), chunk
// softmax partials.  Phase C (lanes = channels): partial PV.
template <typename T>
__global__ __launch_bounds__(64) void decode_chunk_kernel(da_cache c, const T *__restrict__ q_new, int t,
                                                          float scale_log2) {
    // (16-byte accesses below, whatever static LDS precedes it)
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    float *lds = lds_f;
    const int d = c.d, wpr = d >> 5;
    const int ldk = d + 1;
    float *kh = lds;                    // [kChunk][d + 1]
    float *pb = lds + kChunk * ldk;     // [kChunk]
    const int chunk = blockIdx.x, unit = blockIdx.y, lane = threadIdx.x;
    const int r0 = chunk * kChunk;
    const int r1 = min(r0 + kChunk, t + 1);
    const int g = c.Hq / c.Hkv;
    const int b = unit / c.Hkv, hk = unit % c.Hkv;
    const int win_begin = t + 1 - c.Wd;   // rows >= win_begin use raw keys (may be negative)
    const T *surv = surv_chunk<T>(c, unit, chunk);
    const uint32_t *Mp = c.mask + (size_t)unit * c.max_seq * wpr;

    if (r0 < win_begin) {   // some row of the chunk is history
        float held[4] = {0.f, 0.f, 0.f, 0.f};
        if (r0 > 0) {
            const T *ckp = (const T *)c.ck + ((size_t)unit * c.nck + chunk) * d;
            for (int w = 0; w * kWave < d; ++w)
                if (w * kWave + lane < d) held[w] = load_f32(ckp, w * kWave + lane);
        }
        const int hist_end = min(r1, win_begin);
        uint32_t off = 0;
        for (int row = r0; row < hist_end; ++row) {
            for (int w = 0; w * kWave < d; ++w) {
                const int ch = w * kWave + lane;
                bool bit = false;
                if (ch < d) bit = (Mp[(size_t)row * wpr + (ch >> 5)] >> (ch & 31)) & 1u;
                const uint64_t bal = __ballot(bit);
                if (bit) held[w] = load_f32(surv, off + lanes_below(bal));
                off += __popcll(bal);
                if (ch < d) kh[(row - r0) * ldk + ch] = held[w];
            }
        }
    }
    __syncthreads();

    const int row = r0 + lane;
    const bool valid = row < r1;
    const bool in_win = row >= win_begin;
    const T *ringrow = (const T *)c.ring + ((size_t)unit * c.Wd + (valid ? row % c.Wd : 0)) * d;
    for (int hh = 0; hh < g; ++hh) {
        const int h = hk * g + hh;
        const T *q = q_new + ((size_t)b * c.Hq + h) * d;
        float s = 0.f;
        if (valid) {
            if (in_win) {
                for (int ch = 0; ch < d; ++ch) s = fmaf(load_f32(q, ch), load_f32(ringrow, ch), s);
            } else {
                for (int ch = 0; ch < d; ++ch) s = fmaf(load_f32(q, ch), kh[lane * ldk + ch], s);
            }
        }
        s = valid ? s * scale_log2 : -INFINITY;
        const float m = wave_max(s);              // at least row r0 is valid, so m is finite
        const float p = valid ? exp2f(s - m) : 0.f;
        const float l = wave_sum(p);
        __syncthreads();
        pb[lane] = p;
        __syncthreads();
        float *out = c.part + (((size_t)b * c.Hq + h) * c.max_chunks + chunk) * part_stride(d);
        const T *Vp = (const T *)c.V;
        for (int w = 0; w * kWave < d; ++w) {
            const int ch = w * kWave + lane;
            if (ch < d) {
                float acc = 0.f;
                for (int r = 0; r < r1 - r0; ++r)
                    acc = fmaf(pb[r], load_f32(Vp, v_index(unit, c.vrows, d, r0 + r, ch)), acc);
                out[ch] = acc;
            }
        }
        if (lane == 0) {
            out[d] = m;
            out[d + 1] = l;
        }
    }
}

// Merge of the partials (o, m, l) of one (batch, query head).  A partial row is read by G = d / 4 lanes
// (rounded up to a power of two) as 128-bit loads, so 64 / G partials are in flight side by side and kB
// per lane: all loads of a batch are independent.  Every lane keeps a running (max, sum, 4 channels);
// the lane groups are merged with two or three shuffle steps at the end.
template <typename T>
__global__ __launch_bounds__(64) void decode_combine_kernel(da_cache c, T *__restrict__ o, int nparts) {
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    constexpr int kB = 4;
    const int bh = blockIdx.x, lane = threadIdx.x, d = c.d, ps = part_stride(d);
    int G = 8;
    while (G * 4 < d) G <<= 1;
    const int li = lane & (G - 1), slot = lane / G, slots = kWave / G;
    const bool act = li * 4 < d;
    const float *part = c.part + (size_t)bh * c.max_chunks * ps;
    float M = -INFINITY, L = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < nparts; k0 += slots * kB) {
        f32x4 x[kB];
        f32x2 ml[kB];
#pragma unroll
        for (int u = 0; u < kB; ++u) {
            const float *row = part + (size_t)min(k0 + u * slots + slot, nparts - 1) * ps;
            x[u] = act ? *(const f32x4 *)(row + 4 * li) : f32x4{0.f, 0.f, 0.f, 0.f};
            ml[u] = *(const f32x2 *)(row + d);
        }
        float mb = M;
#pragma unroll
        for (int u = 0; u < kB; ++u)
            if (k0 + u * slots + slot < nparts) mb = fmaxf(mb, ml[u][0]);
        const float f = mb == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(M - mb);
        L *= f;
        acc *= f;
#pragma unroll
        for (int u = 0; u < kB; ++u) {
            const float w = (k0 + u * slots + slot < nparts) ? __builtin_amdgcn_exp2f(ml[u][0] - mb) : 0.f;
            L = fmaf(w, ml[u][1], L);
            acc += w * x[u];
        }
        M = mb;
    }
    for (int s = G; s < kWave; s <<= 1) {
        const float m2 = __shfl_xor(M, s), l2 = __shfl_xor(L, s);
        f32x4 a2;
#pragma unroll
        for (int i = 0; i < 4; ++i) a2[i] = __shfl_xor(acc[i], s);
        const float mn = fmaxf(M, m2);
        const float f1 = M == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(M - mn);
        const float f2 = m2 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m2 - mn);
        L = L * f1 + l2 * f2;
        acc = acc * f1 + a2 * f2;
        M = mn;
    }
    if (slot == 0 && act) {
        const float inv = 1.f / L;
#pragma unroll
        for (int i = 0; i < 4; ++i) store_from_f32(o + (size_t)bh * d, 4 * li + i, acc[i] * inv);
    }
}

template <typename T>
void launch_combine(da_cache *c, T *o, int nparts, hipStream_t s) {
    hipLaunchKernelGGL(decode_combine_kernel<T>, dim3(c->B * c->Hq), dim3(64), 0, s, *c, o, nparts);
}

// The decode step for bf16 caches in the row layout (head dims other than 64 / 128, decode windows below one
// chunk, more than 32 query heads per KV head; the column-run layout has its own kernel): one wave per chunk of
// kChunk cached rows of one unit, all query heads of the unit's group.
//   0. the wave that owns the newest row appends it (D1);
//   1. mask rows (lane = row) give the survivor count of every row, hence each row's start inside the
//      chunk's survivor run (a wave prefix sum) - no offset table is read; the run itself is copied to
//      LDS, its first 4 KiB requested before the masks have arrived;
//   2. lanes = channels walk the chunk's history rows in order: the mask word of a row, broadcast
//      from the lane that holds it, selects which lanes take their next surviving value, the rest
//      keep the held one (Eq. 3); each reference row k_hat(j) goes to an LDS tile (Eq. 4 telescoped:
//      the history score of row j is q . k_hat(j)); rows inside the decode window are copied from
//      the raw-key ring instead, the newest one from the call's k_new;
//   3. scores of 64 rows x up to 16 heads on the matrix cores (16x16x32: A lane l = tile row l % 16,
//      k = 8 (l / 16)..+7; B lane l = column l % 16, same k; D lane l = column l % 16, rows
//      4 (l / 16) + r); chunk softmax in that register layout;
//   4. P V on the matrix cores against the 8-row interleaved V cache; partial (o, m, l) to scratch.
// The partials are merged by a second launch: on this chip every XCD has its own L2, so handing them
// to a "last wave" inside the same launch needs device-scope fences that write the L2 back, which
// measured six times slower than the extra launch.
template <int DT>   // head_dim known at compile time (64, 128), or 0 for any multiple of 32
__global__ __launch_bounds__(64) void decode_step_bf16_kernel(da_cache c, const bf16_t *__restrict__ q_new,
                                                              const bf16_t *__restrict__ k_new,
                                                              const bf16_t *__restrict__ v_new,
                                                              uint32_t *__restrict__ mask_row, int t,
                                                              float scale_log2) {
    // (16-byte accesses below, whatever static LDS precedes it)
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    char *lds = (char *)lds_f;
    const int d = DT ? DT : c.d, wpr = d >> 5;
    const int nw = (d + kWave - 1) / kWave;
    const int ldk = d + 8;
    constexpr int kSlab = 16;                                // rows rebuilt and scored at a time
    bf16_t *__restrict__ ktile = (bf16_t *)lds;              // [kSlab][d + 8]
    bf16_t *__restrict__ sv = ktile + kSlab * ldk;           // staged surviving values, <= kChunk * d
    bf16_t *__restrict__ pt = sv + kChunk * d + 16;          // [16][kChunk + 8] probabilities, heads x rows
    const int chunk = blockIdx.x, unit = blockIdx.y, lane = threadIdx.x;
    const int nchunks = t / kChunk + 1;
    const bool newest = chunk == nchunks - 1;                // this wave owns row t
    const int r0 = chunk * kChunk;
    const int r1 = min(r0 + kChunk, t + 1);
    const int nrows = r1 - r0;
    const int g = c.Hq / c.Hkv;
    const int b = unit / c.Hkv, hk = unit % c.Hkv;
    const int win_begin = t + 1 - c.Wd;                      // rows >= win_begin use raw keys
    const int hist_rows = min(max(win_begin - r0, 0), nrows);
    const bf16_t *surv = surv_chunk<bf16_t>(c, unit, chunk);
    const uint32_t *Mp = c.mask + ((size_t)unit * c.max_seq + r0) * wpr;
    const int l16 = lane & 15, lg = lane >> 4;
    const int ks_n = d >> 5, ct_n = d >> 4;
    const int pieces = (kChunk * d) >> 9;                    // 16-byte-per-lane copies that cover the chunk's room

    // ---- everything whose address does not depend on loaded data is requested up front
    uint32_t mk[8];
    uint32_t held[4] = {0u, 0u, 0u, 0u};
    u32x4 sp[4];                                             // first 4 KiB of the survivor run
    if (hist_rows > 0) {
#pragma unroll
        for (int w2 = 0; w2 < 8; ++w2) mk[w2] = (w2 < wpr && lane < hist_rows) ? Mp[(size_t)lane * wpr + w2] : 0u;
        if (r0 > 0) {
            const bf16_t *ckp = (const bf16_t *)c.ck + ((size_t)unit * c.nck + chunk) * d;
#pragma unroll
            for (int w = 0; w < 4; ++w)
                if (w < nw && w * kWave + lane < d) held[w] = ckp[w * kWave + lane];
        }
#pragma unroll
        for (int p = 0; p < 4; ++p)
            if (p < pieces) sp[p] = *(const u32x4 *)(surv + p * 512 + lane * 8);
    }
    for (int i = lane; i < 16 * (kChunk + 8); i += kWave) pt[i] = 0;
    // V operands of the whole chunk (needed last, requested first); the newest row is patched in from v_new
    constexpr int kVregs = DT ? 2 * (DT / 16) : 1;
    u32x4 vop[kVregs];
    if (DT) {
#pragma unroll
        for (int i = 0; i < kVregs; ++i) {
            const int row8 = r0 + 32 * (i & 1) + 8 * lg, ch = 16 * (i >> 1) + l16;
            vop[i] = *(const u32x4 *)((const bf16_t *)c.V + v_index(unit, c.vrows, d, row8, ch));
            if (newest && (t & ~7) == row8) {
                const uint32_t vn = v_new[(size_t)unit * d + ch];
                const int e = t & 7;
                const uint32_t old = vop[i][e >> 1];
                vop[i][e >> 1] = (e & 1) ? ((old & 0xffffu) | (vn << 16)) : ((old & 0xffff0000u) | vn);
            }
        }
    }
    // q operand of the first 16 heads (B operand of the score MFMA), also requested early
    constexpr int kQregs = DT ? DT / 32 : 1;
    u32x4 qop[kQregs];
    if (DT) {
        const int gh0 = min(16, g);
        const bf16_t *qrow0 = q_new + ((size_t)b * c.Hq + hk * g + min(l16, gh0 - 1)) * d;
#pragma unroll
        for (int ks = 0; ks < kQregs; ++ks) {
            qop[ks] = *(const u32x4 *)(qrow0 + 32 * ks + 8 * lg);
            if (l16 >= gh0) qop[ks] = u32x4{0u, 0u, 0u, 0u};
        }
    }
    // 0. the new row goes into the cache (other waves of this launch never read what is written here)
    if (newest) append_row<bf16_t>(c, unit, lane, k_new, v_new, mask_row, t);

    uint32_t roffv = 0;
    if (hist_rows > 0) {
        // 1. row starts inside the chunk's survivor run, from the mask rows
        uint32_t cnt = 0;
#pragma unroll
        for (int w2 = 0; w2 < 8; ++w2) cnt += __popc(mk[w2]);
        uint32_t need;
        roffv = wave_exclusive_scan(cnt, &need);
#pragma unroll
        for (int p = 0; p < 4; ++p)
            if (p < pieces) *(u32x4 *)(sv + p * 512 + lane * 8) = sp[p];
        for (int p = 4; p < pieces && (uint32_t)p * 512u < need; ++p)
            *(u32x4 *)(sv + p * 512 + lane * 8) = *(const u32x4 *)(surv + p * 512 + lane * 8);
    }

    const int segs = d >> 3;
    const bf16_t *ringu = (const bf16_t *)c.ring + (size_t)unit * c.Wd * d;
    for (int hbase = 0; hbase < g; hbase += 16) {
        const int gh = min(16, g - hbase);
        const bf16_t *qrow = q_new + ((size_t)b * c.Hq + hk * g + hbase + min(l16, gh - 1)) * d;
        f32x4 acc[4];
        uint32_t hcur[4] = {held[0], held[1], held[2], held[3]};
#pragma unroll
        for (int slab = 0; slab < kChunk / kSlab; ++slab) {
            const int s0 = slab * kSlab;
            __syncthreads();                                 // survivors staged / previous slab's tile consumed
            // 2. reference keys of the slab's history rows, 8 rows per batch so that the LDS reads of a batch
            //    are in flight together (their addresses depend on the masks only, not on the held values)
            const int hist_here = min(max(hist_rows - s0, 0), kSlab);
            uint32_t off = hist_here > 0 ? __builtin_amdgcn_readlane(roffv, s0) : 0u;   // uniform, advanced per row
            for (int rb = 0; rb < hist_here; rb += 8) {
                uint32_t val[8][4];
                uint64_t msk[8][4];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int r = s0 + min(rb + u, hist_here - 1);
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        if (w < nw) {
                            const uint32_t lo = __builtin_amdgcn_readlane(mk[2 * w], r);
                            const uint32_t hi = __builtin_amdgcn_readlane(mk[2 * w + 1], r);
                            const uint64_t m64 = (rb + u < hist_here) ? ((uint64_t)lo | ((uint64_t)hi << 32)) : 0ull;
                            msk[u][w] = m64;
                            val[u][w] = sv[off + lanes_below(m64)];
                            off += __popcll(m64);
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (rb + u < hist_here) {
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            if (w < nw) {
                                hcur[w] = __builtin_amdgcn_inverse_ballot_w64(msk[u][w]) ? val[u][w] : hcur[w];
                                if (w * kWave + lane < d) ktile[(rb + u) * ldk + w * kWave + lane] = (bf16_t)hcur[w];
                            }
                        }
                    }
                }
            }
            // window rows of the slab: raw keys from the ring (the newest one from the call's argument),
            // zero past the newest key
            for (int i0 = hist_here * segs + lane; i0 < kSlab * segs; i0 += 2 * kWave) {
                u32x4 v[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int i = min(i0 + u * kWave, kSlab * segs - 1);
                    const int r = s0 + i / segs, seg = i % segs;
                    v[u] = u32x4{0u, 0u, 0u, 0u};
                    if (r < nrows) {
                        if (r0 + r == t)
                            v[u] = *(const u32x4 *)(k_new + (size_t)unit * d + seg * 8);
                        else
                            v[u] = *(const u32x4 *)(ringu + (size_t)((r0 + r) % c.Wd) * d + seg * 8);
                    }
                }
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int i = i0 + u * kWave;
                    if (i < kSlab * segs) *(u32x4 *)(ktile + (i / segs) * ldk + (i % segs) * 8) = v[u];
                }
            }
            __syncthreads();
            // 3. scores of the slab: lane l ends up with head l % 16 at rows s0 + 4 (l / 16) + r
            acc[slab] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < (DT ? DT / 32 : 8); ++ks) {
                if (!DT && ks >= ks_n) break;
                u32x4 bv;
                if (DT && hbase == 0) {
                    bv = qop[ks];
                } else {
                    bv = *(const u32x4 *)(qrow + 32 * ks + 8 * lg);
                    if (l16 >= gh) bv = u32x4{0u, 0u, 0u, 0u};
                }
                const u32x4 av = *(const u32x4 *)(ktile + l16 * ldk + 32 * ks + 8 * lg);
                acc[slab] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av),
                                                                    __builtin_bit_cast(bf16x8, bv), acc[slab], 0, 0, 0);
            }
        }
        // chunk softmax per head: 16 values in registers, then the 4 lane groups that share the head
        float m = -INFINITY;
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool valid = 16 * rt + 4 * lg + r < nrows;
                acc[rt][r] = valid ? acc[rt][r] * scale_log2 : -INFINITY;
                m = fmaxf(m, acc[rt][r]);
            }
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));                     // row r0 is always valid, so m is finite
        float l = 0.f;
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
            float p[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                p[r] = __builtin_amdgcn_exp2f(acc[rt][r] - m);
                l += p[r];
            }
            typedef __attribute__((ext_vector_type(2))) float f32x2;
            typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
            uint2 pk;
            pk.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{p[0], p[1]}, bf16x2));
            pk.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{p[2], p[3]}, bf16x2));
            *(uint2 *)(pt + l16 * (kChunk + 8) + 16 * rt + 4 * lg) = pk;
        }
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (lane < gh) {
            float *out = c.part + (((size_t)b * c.Hq + hk * g + hbase + lane) * c.max_chunks + chunk) * part_stride(d);
            out[d] = m;
            out[d + 1] = l;
        }
        __syncthreads();
        // 4. P V: heads x channels, contraction over the chunk's 64 rows
        u32x4 pa[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) pa[ks] = *(const u32x4 *)(pt + l16 * (kChunk + 8) + 32 * ks + 8 * lg);
#pragma unroll
        for (int ct = 0; ct < (DT ? DT / 16 : 16); ++ct) {
            if (!DT && ct >= ct_n) break;
            f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                u32x4 bv;
                if (DT) {
                    bv = vop[2 * ct + ks];
                } else {
                    const int row8 = r0 + 32 * ks + 8 * lg, ch = 16 * ct + l16;
                    bv = *(const u32x4 *)((const bf16_t *)c.V + v_index(unit, c.vrows, d, row8, ch));
                    if (newest && (t & ~7) == row8) {
                        const uint32_t vn = v_new[(size_t)unit * d + ch];
                        const int e = t & 7;
                        const uint32_t old = bv[e >> 1];
                        bv[e >> 1] = (e & 1) ? ((old & 0xffffu) | (vn << 16)) : ((old & 0xffff0000u) | vn);
                    }
                }
                o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pa[ks]),
                                                            __builtin_bit_cast(bf16x8, bv), o, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int h = 4 * lg + r;
                if (h < gh)
                    c.part[(((size_t)b * c.Hq + hk * g + hbase + h) * c.max_chunks + chunk) * part_stride(d) + 16 * ct + l16] =
                        o[r];
            }
        }
        __syncthreads();
    }

}

template <typename T>
void decode_launch(da_cache *c, const void *q, const void *k, const void *v, void *o, uint32_t *mask_row,
                   hipStream_t s) {
    const int t = (int)c->len;
    const int units = c->B * c->Hkv;
    const float sc = (c->scale > 0.f ? c->scale : 1.0f / sqrtf((float)c->d)) * 1.4426950408889634f;
    const int nchunks = t / kChunk + 1;
    if (c->fast) {
        stage_begin(kStageChunk, s);
        const int nparts = da::decode_step_runs(c, q, k, v, o, mask_row, t, sc, s);
        stage_end(kStageChunk, s);
        if (nparts > 0) {
            stage_begin(kStageCombine, s);
            launch_combine<T>(c, (T *)o, nparts, s);
            stage_end(kStageCombine, s);
        }
        if ((t + 1) % kChunk == 0) da::seal_chunk_runs(c, t / kChunk, s);
        return;
    }
    if (c->dtype == DA_BF16) {
        const size_t lds = ((size_t)16 * (c->d + 8) + (size_t)kChunk * c->d + 16) * 2 + 16 * (kChunk + 8) * 2;
        static std::atomic<uint64_t> lds_set;   // d = 256 needs more than 64 KiB; one bit per device
        ensure_dynamic_lds((const void *)decode_step_bf16_kernel<0>,
                           (int)(((size_t)16 * 264 + (size_t)kChunk * 256 + 16) * 2 + 16 * (kChunk + 8) * 2), lds_set);
        stage_begin(kStageChunk, s);
        const dim3 grid(nchunks, units), block(64);
        if (c->d == 64)
            hipLaunchKernelGGL(decode_step_bf16_kernel<64>, grid, block, lds, s, *c, (const bf16_t *)q,
                               (const bf16_t *)k, (const bf16_t *)v, mask_row, t, sc);
        else if (c->d == 128)
            hipLaunchKernelGGL(decode_step_bf16_kernel<128>, grid, block, lds, s, *c, (const bf16_t *)q,
                               (const bf16_t *)k, (const bf16_t *)v, mask_row, t, sc);
        else
            hipLaunchKernelGGL(decode_step_bf16_kernel<0>, grid, block, lds, s, *c, (const bf16_t *)q,
                               (const bf16_t *)k, (const bf16_t *)v, mask_row, t, sc);
        stage_end(kStageChunk, s);
        stage_begin(kStageCombine, s);
        launch_combine<T>(c, (T *)o, nchunks, s);
        stage_end(kStageCombine, s);
        return;
    }
    stage_begin(kStageAppend, s);
    hipLaunchKernelGGL(decode_append_kernel<T>, dim3(units), dim3(64), 0, s, *c, (const T *)k, (const T *)v,
                       mask_row, t);
    stage_end(kStageAppend, s);
    stage_begin(kStageChunk, s);
    {
        const size_t lds = ((size_t)kChunk * (c->d + 1) + kChunk) * sizeof(float);
        static std::atomic<uint64_t> lds_set;   // d = 256 needs slightly more than 64 KiB; one bit per device
        ensure_dynamic_lds((const void *)decode_chunk_kernel<T>, (int)(((size_t)kChunk * 257 + kChunk) * sizeof(float)),
                           lds_set);
        hipLaunchKernelGGL(decode_chunk_kernel<T>, dim3(nchunks, units), dim3(64), lds, s, *c, (const T *)q, t, sc);
    }
    stage_end(kStageChunk, s);
    stage_begin(kStageCombine, s);
    launch_combine<T>(c, (T *)o, nchunks, s);
    stage_end(kStageCombine, s);
}

void free_all(da_cache *c) {
    void *ptrs[] = {c->mask, c->surv, c->ccnt, c->ck, c->khat, c->ring, c->V, c->nnz, c->part};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    if (da_prefix *f = c->pf) {
        void *more[] = {f->k, f->h, f->v, f->m, f->vt, f->ents, f->counts, f->nch8, f->plan, f->dense};
        for (void *p : more)
            if (p) (void)hipFree(p);
        delete f;
    }
}

}  // namespace

namespace da {

da_status cache_check_for_prefill(const da_cache *c, const da_prefill_params *p) {
    if (c->len != 0) return DA_ERR_STATE;
    if (c->B != p->batch || c->Hq != p->n_q_heads || c->Hkv != p->n_kv_heads || c->d != p->head_dim ||
        c->dtype != p->dtype || c->theta != p->theta || c->max_seq < p->seq_len)
        return DA_ERR_STATE;
    if (!cache_scale_matches(c, p->scale)) return DA_ERR_STATE;   // one score scale for prefill and decode (Eq. 1)
    return DA_OK;
}

void cache_fill_from_prefill(da_cache *c, const da_prefill_params *p, const void *K, const void *V,
                             const void *Khat, const uint32_t *mask_bits, const uint32_t *counts,
                             const uint64_t *nnz, hipStream_t s) {
    (void)counts;
    const int units = c->B * c->Hkv, n = p->seq_len;
    if (c->fast) {
        da::cache_fill_runs(c, 0, n, n, K, V, Khat, mask_bits, nnz, s);
        c->len = n;
        return;
    }
    dim3 grid((n + kChunk - 1) / kChunk, units), block(64);
    if (c->dtype == DA_F32)
        hipLaunchKernelGGL(cache_fill_kernel<float>, grid, block, 0, s, (const float *)K, (const float *)V,
                           (const float *)Khat, mask_bits, nnz, *c, n);
    else
        hipLaunchKernelGGL(cache_fill_kernel<bf16_t>, grid, block, 0, s, (const bf16_t *)K, (const bf16_t *)V,
                           (const bf16_t *)Khat, mask_bits, nnz, *c, n);
    c->len = n;
}

}  // namespace da

extern "C" {

da_status delta_attn_cache_create(da_cache **out, int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                  int32_t head_dim, int32_t max_seq, int32_t decode_window, float theta,
                                  float scale, int32_t dtype) {
    if (!out) return DA_ERR_INVALID_ARG;
    *out = nullptr;
    if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 || max_seq < 1 || decode_window < 1)
        return DA_ERR_INVALID_ARG;
    if (n_q_heads % n_kv_heads != 0 || !(theta >= 0.f) || !(scale >= 0.f) || isinf(scale)) return DA_ERR_INVALID_ARG;
    if (head_dim % 32 != 0 || head_dim > 256) return DA_ERR_UNSUPPORTED;
    if (dtype != DA_F32 && dtype != DA_BF16) return DA_ERR_UNSUPPORTED;
    if ((int64_t)batch * n_kv_heads > 65535) return DA_ERR_UNSUPPORTED;
    if ((int64_t)max_seq * head_dim >= (int64_t)1 << 31) return DA_ERR_UNSUPPORTED;
    da_cache *c = new (std::nothrow) da_cache();
    if (!c) return DA_ERR_HIP;
    memset(c, 0, sizeof(*c));
    c->B = batch;
    c->Hq = n_q_heads;
    c->Hkv = n_kv_heads;
    c->d = head_dim;
    c->max_seq = max_seq;
    c->Wd = decode_window < max_seq ? decode_window : max_seq;
    c->dtype = dtype;
    c->theta = theta;
    c->scale = scale;
    c->len = 0;
    c->nck = max_seq / kChunk + 1;
    c->max_chunks = (max_seq + kChunk - 1) / kChunk;
    c->vrows = (max_seq + kChunk - 1) / kChunk * kChunk;
    c->plan_merge = -1;
    c->plan_slots = 0;
    // the column-run layout needs every row of an unsealed chunk inside the decode window: a window of at least
    // one chunk, or one that covers the whole cache
    c->fast = dtype == DA_BF16 && (head_dim == 64 || head_dim == 128) && (c->Wd >= kChunk || c->Wd == max_seq) &&
              n_q_heads / n_kv_heads <= 32;
    if (hipGetDevice(&c->device) != hipSuccess) {
        delete c;
        return DA_ERR_HIP;
    }
    const size_t units = (size_t)batch * n_kv_heads, es = elt_size(dtype), d = head_dim;
    bool ok = true;
    ok = ok && hipMalloc((void **)&c->mask, units * max_seq * (d / 32) * 4) == hipSuccess;
    ok = ok && hipMalloc(&c->surv, units * (size_t)c->max_chunks * run_room_stride(d) * es) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->ccnt, units * (size_t)c->max_chunks * 4) == hipSuccess;
    ok = ok && hipMalloc(&c->ck, units * c->nck * d * es) == hipSuccess;
    ok = ok && hipMalloc(&c->khat, units * d * es) == hipSuccess;
    ok = ok && hipMalloc(&c->ring, units * c->Wd * d * es) == hipSuccess;
    ok = ok && hipMalloc(&c->V, units * (size_t)c->vrows * d * es) == hipSuccess;
    if (ok) ok = hipMemset(c->V, 0, units * (size_t)c->vrows * d * es) == hipSuccess;   // rows never written must be finite
    ok = ok && hipMalloc((void **)&c->nnz, units * 8) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->part, (size_t)batch * n_q_heads * c->max_chunks * part_stride(d) * 4) == hipSuccess;
    if (ok) ok = hipMemset(c->nnz, 0, units * 8) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        free_all(c);
        delete c;
        return DA_ERR_HIP;
    }
    *out = c;
    return DA_OK;
}

da_status delta_attn_cache_destroy(da_cache *c) {
    if (!c) return DA_ERR_INVALID_ARG;
    free_all(c);
    delete c;
    return DA_OK;
}

da_status delta_attn_cache_reset(da_cache *c, void *hip_stream) {
    if (!c) return DA_ERR_INVALID_ARG;
    launch_fill_u64(c->nnz, 0, c->B * c->Hkv, (hipStream_t)hip_stream);
    c->len = 0;
    if (c->pf) c->pf->rows = c->pf->ent_rows = 0;   // an empty sequence, which the (empty) prefix arrays describe
    return launch_ok("cache_reset") ? DA_OK : DA_ERR_HIP;
}

da_status delta_attn_cache_set_launch_plan(da_cache *c, int32_t merge_in_kernel, int32_t wave_slots) {
    if (!c || merge_in_kernel < -1 || merge_in_kernel > 1 || wave_slots < 0) return DA_ERR_INVALID_ARG;
    c->plan_merge = merge_in_kernel;
    c->plan_slots = wave_slots;
    return DA_OK;
}

int64_t delta_attn_cache_length(const da_cache *c) { return c ? c->len : -1; }
const uint64_t *delta_attn_cache_nnz(const da_cache *c) { return c ? c->nnz : nullptr; }
const uint32_t *delta_attn_cache_mask(const da_cache *c) { return c ? c->mask : nullptr; }

da_status delta_attn_decode(da_cache *c, const void *q_new, const void *k_new, const void *v_new, void *o,
                            uint32_t *mask_row, void *hip_stream) {
    if (!c || !q_new || !k_new || !v_new || !o) return DA_ERR_INVALID_ARG;
    if (c->len >= c->max_seq) return DA_ERR_STATE;
    hipStream_t s = (hipStream_t)hip_stream;
    (void)hipGetLastError();
    if (c->dtype == DA_F32)
        decode_launch<float>(c, q_new, k_new, v_new, o, mask_row, s);
    else
        decode_launch<bf16_t>(c, q_new, k_new, v_new, o, mask_row, s);
    if (!launch_ok("decode")) return DA_ERR_HIP;
    c->len += 1;
    return DA_OK;
}

}  // extern "C"
