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

inline size_t elt_size(int dtype) { return dtype == DA_F32 ? 4 : 2; }

// V cache layout: 8 rows interleaved per channel, [unit][t / 8][channel][t % 8], so that eight
// consecutive rows of one channel are contiguous (the k-contiguous operand order of the matrix
// cores).  vmax8 = max_seq rounded up to 8.
__device__ __forceinline__ size_t v_index(int unit, int vmax8, int d, int t, int ch) {
    return ((size_t)unit * (vmax8 >> 3) + (t >> 3)) * ((size_t)d * 8) + (size_t)ch * 8 + (t & 7);
}

// ---------------------------------------------------------------------------------- cache fill
__global__ __launch_bounds__(256) void row_offsets_kernel(const uint32_t *__restrict__ counts,
                                                          uint32_t *__restrict__ roff, const uint64_t *nnz_in,
                                                          uint64_t *nnz_out, int n, int max_seq) {
    __shared__ uint32_t buf[256];
    const int unit = blockIdx.x, tid = threadIdx.x;
    const uint32_t *cp = counts + (size_t)unit * n;
    uint32_t *rp = roff + (size_t)unit * (max_seq + 1);
    uint32_t carry = 0;
    for (int base = 0; base < n; base += 256) {
        const uint32_t v = (base + tid < n) ? cp[base + tid] : 0u;
        buf[tid] = v;
        __syncthreads();
        for (int s = 1; s < 256; s <<= 1) {
            const uint32_t add = (tid >= s) ? buf[tid - s] : 0u;
            __syncthreads();
            buf[tid] += add;
            __syncthreads();
        }
        if (base + tid < n) rp[base + tid] = carry + buf[tid] - v;   // exclusive
        carry += buf[255];
        __syncthreads();
    }
    if (tid == 0) {
        rp[n] = carry;
        nnz_out[unit] = nnz_in[unit];
    }
}

// one wave per cached row
template <typename T>
__global__ __launch_bounds__(256) void cache_fill_kernel(const T *__restrict__ K, const T *__restrict__ V,
                                                         const T *__restrict__ Khat,
                                                         const uint32_t *__restrict__ mask_bits, da_cache c, int n) {
    const int unit = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    const int d = c.d, wpr = d >> 5;
    const size_t src = ((size_t)unit * n + row) * d;
    const uint32_t *Mp = mask_bits + ((size_t)unit * n + row) * wpr;
    uint32_t *Mc = c.mask + ((size_t)unit * c.max_seq + row) * wpr;
    T *surv = (T *)c.surv + (size_t)unit * c.max_seq * d;
    uint32_t off = c.roff[(size_t)unit * (c.max_seq + 1) + row];
    for (int c0 = 0; c0 < d; c0 += kWave) {
        const int ch = c0 + lane;
        const bool act = ch < d;
        bool bit = false;
        if (act) bit = (Mp[ch >> 5] >> (ch & 31)) & 1u;
        const uint64_t b = __ballot(bit);
        if (act) {
            const T k = K[src + ch];
            if (bit) surv[off + lanes_below(b)] = k;
            ((T *)c.V)[v_index(unit, c.vmax8, d, row, ch)] = V[src + ch];
            if (row >= n - c.Wd) ((T *)c.ring)[((size_t)unit * c.Wd + row % c.Wd) * d + ch] = k;
            if (row > 0 && row % kChunk == 0)
                ((T *)c.ck)[((size_t)unit * c.nck + row / kChunk) * d + ch] = Khat[src - d + ch];
            if (row == n - 1) ((T *)c.khat)[(size_t)unit * d + ch] = Khat[src + ch];
        }
        off += __popcll(b);
    }
    if (lane < wpr) Mc[lane] = Mp[lane];
}

// ---------------------------------------------------------------------------------- decode step
// D1: delta of the new key against the carried reference key, append to the compact cache.
template <typename T>
__global__ __launch_bounds__(64) void decode_append_kernel(da_cache c, const T *__restrict__ k_new,
                                                           const T *__restrict__ v_new,
                                                           uint32_t *__restrict__ mask_row, int t) {
    const int unit = blockIdx.x, lane = threadIdx.x;
    const int d = c.d, wpr = d >> 5;
    T *surv = (T *)c.surv + (size_t)unit * c.max_seq * d;
    uint32_t *rp = c.roff + (size_t)unit * (c.max_seq + 1);
    const uint32_t start = (t == 0) ? 0u : rp[t];
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
                if (t % kChunk == 0) ((T *)c.ck)[((size_t)unit * c.nck + t / kChunk) * d + ch] = hraw;
            }
            if (fire) *hp = kraw;
            ((T *)c.ring)[((size_t)unit * c.Wd + t % c.Wd) * d + ch] = kraw;
            ((T *)c.V)[v_index(unit, c.vmax8, d, t, ch)] = v_new[(size_t)unit * d + ch];
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
        if (t == 0) rp[0] = 0;
        rp[t + 1] = off;
        c.nnz[unit] = (t == 0 ? 0ull : c.nnz[unit]) + (off - start);
    }
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

// D2-D4 for one chunk of kChunk cached rows of one unit, all query heads of the unit's group.
// Phase A (lanes = channels): rebuild the reference keys k_hat(j) of the chunk from the chunk's
// checkpoint, the mask bits and the surviving values; by telescoping Eq. 4 the history score of
// row j is q . k_hat(j).  Phase B (lanes = rows): scores (raw-key ring inside the window), chunk
// softmax partials.  Phase C (lanes = channels): partial PV.
template <typename T>
__global__ __launch_bounds__(64) void decode_chunk_kernel(da_cache c, const T *__restrict__ q_new, int t,
                                                          float scale_log2) {
    extern __shared__ float lds_f[];
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
    const T *surv = (const T *)c.surv + (size_t)unit * c.max_seq * d;
    const uint32_t *rp = c.roff + (size_t)unit * (c.max_seq + 1);
    const uint32_t *Mp = c.mask + (size_t)unit * c.max_seq * wpr;

    if (r0 < win_begin) {   // some row of the chunk is history
        float held[4] = {0.f, 0.f, 0.f, 0.f};
        if (r0 > 0) {
            const T *ckp = (const T *)c.ck + ((size_t)unit * c.nck + chunk) * d;
            for (int w = 0; w * kWave < d; ++w)
                if (w * kWave + lane < d) held[w] = load_f32(ckp, w * kWave + lane);
        }
        const int hist_end = min(r1, win_begin);
        for (int row = r0; row < hist_end; ++row) {
            uint32_t off = rp[row];
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
        float *out = c.part + (((size_t)b * c.Hq + h) * c.max_chunks + chunk) * (d + 2);
        const T *Vp = (const T *)c.V;
        for (int w = 0; w * kWave < d; ++w) {
            const int ch = w * kWave + lane;
            if (ch < d) {
                float acc = 0.f;
                for (int r = 0; r < r1 - r0; ++r)
                    acc = fmaf(pb[r], load_f32(Vp, v_index(unit, c.vmax8, d, r0 + r, ch)), acc);
                out[ch] = acc;
            }
        }
        if (lane == 0) {
            out[d] = m;
            out[d + 1] = l;
        }
    }
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// D2-D4 for bf16 caches: one wave per chunk of kChunk cached rows of one unit, all query heads of the
// unit's group.
//   1. the chunk's surviving key values (one contiguous run of the compact cache) are copied to LDS;
//   2. lanes = channels walk the chunk's history rows in order: the mask word of a row, broadcast
//      from the lane that holds it, selects which lanes take their next surviving value, the rest
//      keep the held one (Eq. 3); each reference row k_hat(j) goes to an LDS tile (Eq. 4 telescoped:
//      the history score of row j is q . k_hat(j)); rows inside the decode window are copied from
//      the raw-key ring instead;
//   3. scores of 64 rows x up to 16 heads on the matrix cores (16x16x32: A lane l = tile row l % 16,
//      k = 8 (l / 16)..+7; B lane l = column l % 16, same k; D lane l = column l % 16, rows
//      4 (l / 16) + r);
//   4. per-head chunk softmax with lanes = rows; P V on the matrix cores against the 8-row
//      interleaved V cache, partial (o, m, l) to the per-chunk scratch.
template <int DT>   // head_dim known at compile time (64, 128), or 0 for any multiple of 32
__global__ __launch_bounds__(64) void decode_chunk_bf16_kernel(da_cache c, const bf16_t *__restrict__ q_new, int t,
                                                               float scale_log2) {
    extern __shared__ float lds_f[];
    char *lds = (char *)lds_f;
    const int d = DT ? DT : c.d, wpr = d >> 5;
    const int nw = (d + kWave - 1) / kWave;
    const int ldk = d + 8;
    bf16_t *ktile = (bf16_t *)lds;                           // [kChunk][d + 8]
    bf16_t *sv = ktile + kChunk * ldk;                       // staged surviving values, <= kChunk * d + 8
    bf16_t *pt = sv + kChunk * d + 16;                       // [16][kChunk + 8] probabilities, heads x rows
    const int chunk = blockIdx.x, unit = blockIdx.y, lane = threadIdx.x;
    const int r0 = chunk * kChunk;
    const int r1 = min(r0 + kChunk, t + 1);
    const int nrows = r1 - r0;
    const int g = c.Hq / c.Hkv;
    const int b = unit / c.Hkv, hk = unit % c.Hkv;
    const int win_begin = t + 1 - c.Wd;                      // rows >= win_begin use raw keys
    const int hist_rows = min(max(win_begin - r0, 0), nrows);
    const bf16_t *surv = (const bf16_t *)c.surv + (size_t)unit * c.max_seq * d;
    const uint32_t *rp = c.roff + (size_t)unit * (c.max_seq + 1);
    const uint32_t *Mp = c.mask + ((size_t)unit * c.max_seq + r0) * wpr;
    const int l16 = lane & 15, lg = lane >> 4;
    const int ks_n = d >> 5, ct_n = d >> 4;

    // everything whose address does not depend on loaded data is requested up front
    uint32_t roffv = 0, s_end = 0;
    uint32_t mk[8];
    uint32_t held[4] = {0u, 0u, 0u, 0u};
    if (hist_rows > 0) {
        roffv = rp[r0 + min(lane, hist_rows)];
        s_end = rp[r0 + hist_rows];
#pragma unroll
        for (int w2 = 0; w2 < 8; ++w2) mk[w2] = (w2 < wpr && lane < hist_rows) ? Mp[(size_t)lane * wpr + w2] : 0u;
        if (r0 > 0) {
            const bf16_t *ckp = (const bf16_t *)c.ck + ((size_t)unit * c.nck + chunk) * d;
#pragma unroll
            for (int w = 0; w < 4; ++w)
                if (w < nw && w * kWave + lane < d) held[w] = ckp[w * kWave + lane];
        }
    }
    // raw keys of the window rows (16 bytes per lane per copy) straight into the tile; zero past the newest key
    {
        const int segs = d >> 3;
        const int first = hist_rows * segs, last = kChunk * segs;
        const bf16_t *ringu = (const bf16_t *)c.ring + (size_t)unit * c.Wd * d;
        for (int i0 = first + lane; i0 < last; i0 += 4 * kWave) {
            u32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * kWave;
                const int r = min(i, last - 1) / segs, seg = min(i, last - 1) % segs;
                v[u] = u32x4{0u, 0u, 0u, 0u};
                if (i < last && r < nrows) v[u] = *(const u32x4 *)(ringu + (size_t)((r0 + r) % c.Wd) * d + seg * 8);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * kWave;
                if (i < last) *(u32x4 *)(ktile + (i / segs) * ldk + (i % segs) * 8) = v[u];
            }
        }
    }
    for (int i = lane; i < 16 * (kChunk + 8); i += kWave) pt[i] = 0;
    // V operands of the whole chunk (needed last, requested first)
    constexpr int kVregs = DT ? 2 * (DT / 16) : 1;
    u32x4 vop[kVregs];
    if (DT) {
#pragma unroll
        for (int i = 0; i < kVregs; ++i)
            vop[i] = *(const u32x4 *)((const bf16_t *)c.V +
                                      v_index(unit, c.vmax8, d, r0 + 32 * (i & 1) + 8 * lg, 16 * (i >> 1) + l16));
    }

    if (hist_rows > 0) {
        // 1. stage the chunk's survivors: rows r0 .. r0 + hist_rows - 1 occupy [rp[r0], rp[r0 + hist_rows])
        const uint32_t s_begin = __builtin_amdgcn_readfirstlane(roffv);
        const uint32_t base = s_begin & ~7u;
        for (uint32_t i = base + lane * 8; i < s_end; i += kWave * 8)
            *(u32x4 *)(sv + (i - base)) = *(const u32x4 *)(surv + i);
        __syncthreads();
        // 2. reference keys of the history rows, 8 rows per batch so that the LDS reads of a batch are
        //    in flight together (their addresses depend on the masks only, not on the held values)
        for (int rb = 0; rb < hist_rows; rb += 8) {
            uint32_t val[8][4];
            bool bit[8][4];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = min(rb + u, hist_rows - 1);
                uint32_t off = __builtin_amdgcn_readlane(roffv, r) - base;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    if (w < nw) {
                        const uint32_t lo = __builtin_amdgcn_readlane(mk[2 * w], r);
                        const uint32_t hi = __builtin_amdgcn_readlane(mk[2 * w + 1], r);
                        const uint64_t m64 = (uint64_t)lo | ((uint64_t)hi << 32);
                        bit[u][w] = (m64 >> lane) & 1ull;
                        val[u][w] = sv[off + lanes_below(m64)];
                        off += __popcll(m64);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (rb + u < hist_rows) {
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        if (w < nw) {
                            held[w] = bit[u][w] ? val[u][w] : held[w];
                            if (w * kWave + lane < d) ktile[(rb + u) * ldk + w * kWave + lane] = (bf16_t)held[w];
                        }
                    }
                }
            }
        }
    }
    __syncthreads();

    for (int hbase = 0; hbase < g; hbase += 16) {
        const int gh = min(16, g - hbase);
        // 3. scores: lane l ends up with head l % 16 at rows 16 rt + 4 (l / 16) + r
        const bf16_t *qrow = q_new + ((size_t)b * c.Hq + hk * g + hbase + min(l16, gh - 1)) * d;
        f32x4 acc[4];
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int ks = 0; ks < ks_n; ++ks) {
            u32x4 bv = *(const u32x4 *)(qrow + 32 * ks + 8 * lg);
            if (l16 >= gh) bv = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) {
                const u32x4 av = *(const u32x4 *)(ktile + (16 * rt + l16) * ldk + 32 * ks + 8 * lg);
                acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av),
                                                                  __builtin_bit_cast(bf16x8, bv), acc[rt], 0, 0, 0);
            }
        }
        // 4. chunk softmax per head: 16 values in registers, then the 4 lane groups that share the head
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
                p[r] = exp2f(acc[rt][r] - m);
                l += p[r];
            }
            uint2 pk;
            pk.x = (uint32_t)f32_to_bf16(p[0]) | ((uint32_t)f32_to_bf16(p[1]) << 16);
            pk.y = (uint32_t)f32_to_bf16(p[2]) | ((uint32_t)f32_to_bf16(p[3]) << 16);
            *(uint2 *)(pt + l16 * (kChunk + 8) + 16 * rt + 4 * lg) = pk;
        }
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (lane < gh) {
            float *out = c.part + (((size_t)b * c.Hq + hk * g + hbase + lane) * c.max_chunks + chunk) * (d + 2);
            out[d] = m;
            out[d + 1] = l;
        }
        __syncthreads();
        // P V: heads x channels, contraction over the chunk's 64 rows
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
                if (DT)
                    bv = vop[2 * ct + ks];
                else
                    bv = *(const u32x4 *)((const bf16_t *)c.V +
                                          v_index(unit, c.vmax8, d, r0 + 32 * ks + 8 * lg, 16 * ct + l16));
                o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pa[ks]),
                                                            __builtin_bit_cast(bf16x8, bv), o, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int h = 4 * lg + r;
                if (h < gh)
                    c.part[(((size_t)b * c.Hq + hk * g + hbase + h) * c.max_chunks + chunk) * (d + 2) + 16 * ct + l16] =
                        o[r];
            }
        }
        __syncthreads();
    }
}

// Merge of the per-chunk partials of one (batch, query head): lanes = chunks for the weights,
// lanes = channels for the output.
template <typename T>
__global__ __launch_bounds__(64) void decode_combine2_kernel(da_cache c, T *__restrict__ o, int nchunks) {
    const int bh = blockIdx.x, lane = threadIdx.x;
    const int d = c.d;
    const float *part = c.part + (size_t)bh * c.max_chunks * (d + 2);
    float M = -INFINITY;
    for (int k = lane; k < nchunks; k += kWave) M = fmaxf(M, part[(size_t)k * (d + 2) + d]);
    M = wave_max(M);
    float L = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < nchunks; k0 += kWave) {
        const int k = k0 + lane;
        const float wk = k < nchunks ? exp2f(part[(size_t)k * (d + 2) + d] - M) : 0.f;
        L += k < nchunks ? wk * part[(size_t)k * (d + 2) + d + 1] : 0.f;
        const int cnt = min(kWave, nchunks - k0);
        for (int kb = 0; kb < cnt; kb += 8) {
            float w[8], x[8][4];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int kk = min(kb + u, cnt - 1);
                w[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wk), kk));
                if (kb + u >= cnt) w[u] = 0.f;
                const float *row = part + (size_t)(k0 + kk) * (d + 2);
#pragma unroll
                for (int i = 0; i < 4; ++i) x[u][i] = (i * kWave + lane < d) ? row[i * kWave + lane] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i] = fmaf(w[u], x[u][i], acc[i]);
        }
    }
    L = wave_sum(L);
    const float inv = 1.f / L;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (i * kWave + lane < d) store_from_f32(o + (size_t)bh * d, i * kWave + lane, acc[i] * inv);
}

template <typename T>
__global__ __launch_bounds__(64) void decode_combine_kernel(da_cache c, T *__restrict__ o, int nchunks) {
    const int bh = blockIdx.x, lane = threadIdx.x;
    const int d = c.d;
    const float *part = c.part + (size_t)bh * c.max_chunks * (d + 2);
    float M = -INFINITY;
    for (int k = 0; k < nchunks; ++k) M = fmaxf(M, part[(size_t)k * (d + 2) + d]);
    float L = 0.f;
    for (int k = 0; k < nchunks; ++k)
        L += part[(size_t)k * (d + 2) + d + 1] * exp2f(part[(size_t)k * (d + 2) + d] - M);
    const float inv = 1.f / L;
    for (int ch = lane; ch < d; ch += kWave) {
        float acc = 0.f;
        for (int k = 0; k < nchunks; ++k)
            acc = fmaf(part[(size_t)k * (d + 2) + ch], exp2f(part[(size_t)k * (d + 2) + d] - M), acc);
        store_from_f32(o + (size_t)bh * d, ch, acc * inv);
    }
}

template <typename T>
void decode_launch(da_cache *c, const void *q, const void *k, const void *v, void *o, uint32_t *mask_row,
                   hipStream_t s) {
    const int t = (int)c->len;
    const int units = c->B * c->Hkv;
    const float sc = (c->scale > 0.f ? c->scale : 1.0f / sqrtf((float)c->d)) * 1.4426950408889634f;
    stage_begin(kStageAppend, s);
    hipLaunchKernelGGL(decode_append_kernel<T>, dim3(units), dim3(64), 0, s, *c, (const T *)k, (const T *)v,
                       mask_row, t);
    stage_end(kStageAppend, s);
    const int nchunks = t / kChunk + 1;
    stage_begin(kStageChunk, s);
    if (c->dtype == DA_BF16) {
        const size_t lds = ((size_t)kChunk * (c->d + 8) + (size_t)kChunk * c->d + 16) * 2 + 16 * (kChunk + 8) * 2;
        static bool attr16_done = false;   // d = 256 needs more than 64 KiB
        if (!attr16_done) {
            (void)hipFuncSetAttribute((const void *)decode_chunk_bf16_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)(((size_t)kChunk * 264 + (size_t)kChunk * 256 + 16) * 2 +
                                            16 * (kChunk + 8) * 2));
            attr16_done = true;
        }
        if (c->d == 64)
            hipLaunchKernelGGL(decode_chunk_bf16_kernel<64>, dim3(nchunks, units), dim3(64), lds, s, *c,
                               (const bf16_t *)q, t, sc);
        else if (c->d == 128)
            hipLaunchKernelGGL(decode_chunk_bf16_kernel<128>, dim3(nchunks, units), dim3(64), lds, s, *c,
                               (const bf16_t *)q, t, sc);
        else
            hipLaunchKernelGGL(decode_chunk_bf16_kernel<0>, dim3(nchunks, units), dim3(64), lds, s, *c,
                               (const bf16_t *)q, t, sc);
    } else {
        const size_t lds = ((size_t)kChunk * (c->d + 1) + kChunk) * sizeof(float);
        static bool attr_done = false;   // d = 256 needs slightly more than 64 KiB
        if (!attr_done) {
            (void)hipFuncSetAttribute((const void *)decode_chunk_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)(((size_t)kChunk * 257 + kChunk) * sizeof(float)));
            attr_done = true;
        }
        hipLaunchKernelGGL(decode_chunk_kernel<T>, dim3(nchunks, units), dim3(64), lds, s, *c, (const T *)q, t, sc);
    }
    stage_end(kStageChunk, s);
    stage_begin(kStageCombine, s);
    hipLaunchKernelGGL(decode_combine2_kernel<T>, dim3(c->B * c->Hq), dim3(64), 0, s, *c, (T *)o, nchunks);
    stage_end(kStageCombine, s);
}

void free_all(da_cache *c) {
    void *ptrs[] = {c->mask, c->surv, c->roff, c->ck, c->khat, c->ring, c->V, c->nnz, c->part};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
}

}  // namespace

namespace da {

da_status cache_check_for_prefill(const da_cache *c, const da_prefill_params *p) {
    if (c->len != 0) return DA_ERR_STATE;
    if (c->B != p->batch || c->Hq != p->n_q_heads || c->Hkv != p->n_kv_heads || c->d != p->head_dim ||
        c->dtype != p->dtype || c->theta != p->theta || c->max_seq < p->seq_len)
        return DA_ERR_STATE;
    return DA_OK;
}

void cache_fill_from_prefill(da_cache *c, const da_prefill_params *p, const void *K, const void *V,
                             const void *Khat, const uint32_t *mask_bits, const uint32_t *counts,
                             const uint64_t *nnz, hipStream_t s) {
    const int units = c->B * c->Hkv, n = p->seq_len;
    hipLaunchKernelGGL(row_offsets_kernel, dim3(units), dim3(256), 0, s, counts, c->roff, nnz, c->nnz, n,
                       c->max_seq);
    dim3 grid((n + 3) / 4, units), block(256);
    if (c->dtype == DA_F32)
        hipLaunchKernelGGL(cache_fill_kernel<float>, grid, block, 0, s, (const float *)K, (const float *)V,
                           (const float *)Khat, mask_bits, *c, n);
    else
        hipLaunchKernelGGL(cache_fill_kernel<bf16_t>, grid, block, 0, s, (const bf16_t *)K, (const bf16_t *)V,
                           (const bf16_t *)Khat, mask_bits, *c, n);
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
    c->vmax8 = (max_seq + kChunk - 1) / kChunk * kChunk;
    if (hipGetDevice(&c->device) != hipSuccess) {
        delete c;
        return DA_ERR_HIP;
    }
    const size_t units = (size_t)batch * n_kv_heads, es = elt_size(dtype), d = head_dim;
    bool ok = true;
    ok = ok && hipMalloc((void **)&c->mask, units * max_seq * (d / 32) * 4) == hipSuccess;
    ok = ok && hipMalloc(&c->surv, units * max_seq * d * es) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->roff, units * ((size_t)max_seq + 1) * 4) == hipSuccess;
    ok = ok && hipMalloc(&c->ck, units * c->nck * d * es) == hipSuccess;
    ok = ok && hipMalloc(&c->khat, units * d * es) == hipSuccess;
    ok = ok && hipMalloc(&c->ring, units * c->Wd * d * es) == hipSuccess;
    ok = ok && hipMalloc(&c->V, units * (size_t)c->vmax8 * d * es) == hipSuccess;
    if (ok) ok = hipMemset(c->V, 0, units * (size_t)c->vmax8 * d * es) == hipSuccess;   // rows never written must be finite
    ok = ok && hipMalloc((void **)&c->nnz, units * 8) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->part, (size_t)batch * n_q_heads * c->max_chunks * (d + 2) * 4) == hipSuccess;
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
    return launch_ok("cache_reset") ? DA_OK : DA_ERR_HIP;
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
