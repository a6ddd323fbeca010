// Hybrid-attention prefill for bf16 inputs, head_dim 64 or 128 (Sec. III-B prefill stage; Eq. 4; Eq. 1).
//
// Work group = 512 threads (8 waves) on 256 "score rows": RT consecutive query rows x GH query heads of
// one KV head (they share K, V and the delta matrix).  Key columns are walked left to right in blocks
// of 32.
//
//   far blocks   (every row of the tile has the column outside its window): Eq. 4 as written.  Wave w
//                takes columns w, w+8, w+16, w+24 of the block; a lane owns 4 score rows and adds
//                q[c] * delta for each surviving (channel, delta) entry of the column.  The entry list is
//                wave-uniform and arrives through scalar loads; q comes from a transposed fp16 copy of the
//                Q tile in LDS (one 8-byte read feeds 4 multiply-adds).  The per-column updates u are
//                exchanged through LDS; the owner of a score row adds them up in column order (its running
//                Eq. 4 score).
//   near blocks  (some row has the column inside its window): exact scores K Q^T on the matrix cores;
//                where a tile straddles window squares, the not-yet-exact entries come from K_hat Q^T
//                (Eq. 4 telescoped: sum of the deltas up to column j is the held key k_hat(j)).
//   every block  online softmax with lane-local row state, P V on the matrix cores with V pre-transposed.
//
// Matrix-core layouts (v_mfma_f32_32x32x16_bf16, wave64): A lane l holds row l%32, k = 8*(l/32)..+7;
// B lane l holds column l%32, same k; D lane l holds column l%32, rows 8*(r/4) + 4*(l/32) + r%4 for
// register r.  Scores are produced transposed (keys x score rows) so that a lane owns one score row,
// and D registers 8a..8a+7 are exactly the B operand of the a-th k-step of P V once V^T is fetched in
// the matching key order.
#include "common.hpp"
#include "kernels.hpp"

namespace da {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) _Float16 half4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kRows = 256;      // score rows per work group
constexpr int kTB = 32;         // key columns per block
constexpr int kWaves = 8;

struct MfmaArgs {
    const bf16_t *__restrict__ Q;
    const bf16_t *__restrict__ K;
    const bf16_t *__restrict__ Khat;
    const bf16_t *__restrict__ Vt;      // [unit][D][n_pad]
    bf16_t *__restrict__ O;
    const Entry *__restrict__ ents;
    const uint32_t *__restrict__ counts;
    int Hq, Hkv, n, n_pad, W, rebase;
    int GH, RT, tiles, hgroups;         // heads per group chunk, rows per tile, row tiles, head chunks per unit
    float scale_log2;
};

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

template <int D>
__global__ __launch_bounds__(512) void prefill_mfma_kernel(MfmaArgs a) {
    extern __shared__ char lds_raw[];
    _Float16 *qt = (_Float16 *)lds_raw;                                   // [D][256] fp16, scaled by 2^qexp
    float *ubuf = (float *)(lds_raw + (size_t)D * kRows * 2);             // [2][kTB][256]
    __shared__ float red[kWaves];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction; tell the compiler
    const int half = lane >> 5, li = lane & 31;

    // ---- which tile: heavy (late) row tiles first, units interleaved below them
    int bid = blockIdx.x;
    const int per_unit = a.tiles * a.hgroups;
    const int unit = bid / per_unit;
    bid -= unit * per_unit;
    const int hchunk = bid % a.hgroups;
    const int tile = a.tiles - 1 - bid / a.hgroups;
    const int b = unit / a.Hkv, hk = unit % a.Hkv;
    const int g = a.Hq / a.Hkv;
    const int head0 = hk * g + hchunk * a.GH;
    const int n = a.n, W = a.W, RT = a.RT;
    const int i0 = tile * RT;
    const int i_last = min(n - 1, i0 + RT - 1);

    const bf16_t *Kp = a.K + (size_t)unit * n * D;
    const bf16_t *Hp = a.Khat + (size_t)unit * n * D;
    const bf16_t *Vtp = a.Vt + (size_t)unit * D * a.n_pad;
    const Entry *Ep = a.ents + (size_t)unit * n * D;
    const uint32_t *Cp = a.counts + (size_t)unit * n;

    // score row sr = hh * RT + r  ->  query row i0 + r of head head0 + hh
    auto q_row_ptr = [&](int sr) -> const bf16_t * {
        const int hh = sr / RT, r = sr - hh * RT;
        const int i = min(i0 + r, n - 1);
        return a.Q + (((size_t)b * a.Hq + head0 + hh) * n + i) * D;
    };

    // ---- stage the Q tile: per-tile power-of-two scale so that the fp16 copy neither overflows nor
    //      loses bits that matter (|q| max lands in [2^14, 2^15)).
    float amax = 0.f;
    for (int idx = tid; idx < kRows * (D / 8); idx += 512) {
        const int sr = idx / (D / 8), c8 = idx % (D / 8);
        const u32x4 raw = *(const u32x4 *)(q_row_ptr(sr) + c8 * 8);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            amax = fmaxf(amax, fabsf(__uint_as_float(raw[k] << 16)));
            amax = fmaxf(amax, fabsf(__uint_as_float(raw[k] & 0xffff0000u)));
        }
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) amax = fmaxf(amax, __shfl_xor(amax, s));
    if (lane == 0) red[wave] = amax;
    __syncthreads();
    amax = red[0];
#pragma unroll
    for (int k = 1; k < kWaves; ++k) amax = fmaxf(amax, red[k]);
    int qexp = 0;
    if (amax > 0.f && amax < INFINITY) {
        const int e = (int)((__float_as_uint(amax) >> 23) & 0xff) - 127;   // floor(log2 amax) for normal values
        qexp = 14 - e;
    }
    const float qmul = __uint_as_float((uint32_t)(min(max(qexp, -126), 127) + 127) << 23);
    for (int idx = tid; idx < kRows * (D / 8); idx += 512) {
        const int sr = idx % kRows, c8 = idx / kRows;    // consecutive threads -> consecutive score rows
        const u32x4 raw = *(const u32x4 *)(q_row_ptr(sr) + c8 * 8);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float lo = __uint_as_float(raw[k] << 16) * qmul;
            const float hi = __uint_as_float(raw[k] & 0xffff0000u) * qmul;
            qt[(c8 * 8 + 2 * k) * kRows + sr] = (_Float16)lo;
            qt[(c8 * 8 + 2 * k + 1) * kRows + sr] = (_Float16)hi;
        }
    }
    const float far_scale = a.scale_log2 / qmul;   // undo the tile scale together with the softmax scale

    // ---- this wave's score rows for softmax / PV: sr = 32 * wave + li (both lane halves)
    const int my_sr = 32 * wave + li;
    const int my_hh = my_sr / RT, my_r = my_sr - my_hh * RT;
    const int my_i = i0 + my_r;
    const bool my_valid = my_i < n;
    const int my_win = (min(my_i, n - 1) / W) * W;
    const bf16_t *my_q = q_row_ptr(my_sr);

    constexpr int KS = D / 16;     // k-steps of Q K^T
    constexpr int MT = D / 32;     // channel tiles of the output
    u32x4 qreg[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[ks] = *(const u32x4 *)(my_q + ks * 16 + half * 8);

    f32x16 oacc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[mt][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f, r_run = 0.f;

    const int win_first = (i0 / W) * W;
    const bool aligned = (win_first % kTB == 0) && (i0 / W == i_last / W);
    const int far_blocks = a.rebase ? 0 : win_first / kTB;
    const int nblocks = i_last / kTB + 1;

    __syncthreads();   // Q tile staged

    // One block of PV: scores s[16] (already scaled, -inf where masked) for this lane's keys of block jb
    auto softmax_pv = [&](float (&s)[16], int jb) {
        float bm = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) bm = fmaxf(bm, s[r]);
        bm = fmaxf(bm, __shfl_xor(bm, 32));
        const float m_new = fmaxf(m_run, bm);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = exp2f(m_run - m_use);
        m_run = m_new;
        float psum = 0.f;
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            p[r] = exp2f(s[r] - m_use);
            psum += p[r];
        }
        l_run = l_run * alpha + psum;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[mt][r] *= alpha;
        }
#pragma unroll
        for (int ka = 0; ka < 2; ++ka) {
            u32x4 pb;
#pragma unroll
            for (int k = 0; k < 4; ++k) pb[k] = pack_bf16x2(p[8 * ka + 2 * k], p[8 * ka + 2 * k + 1]);
            const int key0 = jb + 16 * ka + 4 * half;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const bf16_t *vrow = Vtp + (size_t)(mt * 32 + li) * a.n_pad + key0;
                const u32x2 v0 = *(const u32x2 *)(vrow);
                const u32x2 v1 = *(const u32x2 *)(vrow + 8);
                u32x4 va;
                va[0] = v0[0];
                va[1] = v0[1];
                va[2] = v1[0];
                va[3] = v1[1];
                oacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va), as_bf16x8(pb), oacc[mt], 0, 0, 0);
            }
        }
    };

    // transposed score tile S^T[key][score row] = X[jb + key] . q for X = K or K_hat
    auto score_tile = [&](const bf16_t *X, int jb) -> f32x16 {
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        const bf16_t *xrow = X + (size_t)min(jb + li, n - 1) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const u32x4 xa = *(const u32x4 *)(xrow + ks * 16);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(xa), as_bf16x8(qreg[ks]), acc, 0, 0, 0);
        }
        return acc;
    };

    // ---------------------------------------------------------------- far blocks: gather (Eq. 4)
    auto gather_block = [&](int blk) {
        float *ub = ubuf + (size_t)(blk & 1) * kTB * kRows;
        const uint32_t lane_off = (uint32_t)lane * 8u;
#pragma unroll 1
        for (int cc = 0; cc < kTB / kWaves; ++cc) {
            const int jj = wave + cc * kWaves;
            const int j = blk * kTB + jj;                    // wave-uniform, < win_first <= n
            const uint32_t cnt = Cp[j];
            const u32x4 *e = (const u32x4 *)(Ep + (size_t)j * D);
            float u0 = 0.f, u1 = 0.f, u2 = 0.f, u3 = 0.f;
            for (uint32_t k = 0; k < cnt; k += 4) {
                const u32x4 ea = e[k >> 1], eb = e[(k >> 1) + 1];
                const half4 q0 = *(const half4 *)((const char *)qt + (ea[0] * (kRows * 2) + lane_off));
                const half4 q1 = *(const half4 *)((const char *)qt + (ea[2] * (kRows * 2) + lane_off));
                const half4 q2 = *(const half4 *)((const char *)qt + (eb[0] * (kRows * 2) + lane_off));
                const half4 q3 = *(const half4 *)((const char *)qt + (eb[2] * (kRows * 2) + lane_off));
                const float d0 = __uint_as_float(ea[1]), d1 = __uint_as_float(ea[3]);
                const float d2 = __uint_as_float(eb[1]), d3 = __uint_as_float(eb[3]);
                u0 = fmaf((float)q0[0], d0, u0); u1 = fmaf((float)q0[1], d0, u1);
                u2 = fmaf((float)q0[2], d0, u2); u3 = fmaf((float)q0[3], d0, u3);
                u0 = fmaf((float)q1[0], d1, u0); u1 = fmaf((float)q1[1], d1, u1);
                u2 = fmaf((float)q1[2], d1, u2); u3 = fmaf((float)q1[3], d1, u3);
                u0 = fmaf((float)q2[0], d2, u0); u1 = fmaf((float)q2[1], d2, u1);
                u2 = fmaf((float)q2[2], d2, u2); u3 = fmaf((float)q2[3], d2, u3);
                u0 = fmaf((float)q3[0], d3, u0); u1 = fmaf((float)q3[1], d3, u1);
                u2 = fmaf((float)q3[2], d3, u2); u3 = fmaf((float)q3[3], d3, u3);
            }
            f32x4 uv;
            uv[0] = u0; uv[1] = u1; uv[2] = u2; uv[3] = u3;
            *(f32x4 *)(ub + jj * kRows + lane * 4) = uv;
        }
    };

    if (far_blocks > 0) gather_block(0);
    for (int blk = 0; blk < far_blocks; ++blk) {
        __syncthreads();                                     // u of block blk complete
        // Keys of the block in groups of 4: group 2q belongs to lane half 0, group 2q+1 to half 1 (the
        // matrix-core D layout).  A lane sums inside its own groups and gets the other half's group
        // totals from its partner lane, so the running Eq. 4 score advances in column order.
        const float *ub = ubuf + (size_t)(blk & 1) * kTB * kRows + (4 * half) * kRows + my_sr;
        float w[16], t_own[4], t_oth[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float run = 0.f;
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) {
                run += ub[(8 * q + bb) * kRows];
                w[4 * q + bb] = run;
            }
            t_own[q] = run;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) t_oth[q] = __shfl_xor(t_own[q], 32);
        float s[16];
        float base = r_run;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float mine = half ? base + t_oth[q] : base;
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) s[4 * q + bb] = (mine + w[4 * q + bb]) * far_scale;
            base += t_own[q] + t_oth[q];
        }
        r_run = base;
        if (blk + 1 < far_blocks) gather_block(blk + 1);     // overlaps with slower waves still reading blk
        softmax_pv(s, blk * kTB);
    }

    // ---------------------------------------------------------------- near blocks (and all blocks in rebase mode)
    for (int blk = far_blocks; blk < nblocks; ++blk) {
        const int jb = blk * kTB;
        float s[16];
        const bool all_far = jb + kTB <= win_first;          // rebase mode only
        if (all_far) {
            const f32x16 sh = score_tile(Hp, jb);
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = sh[r] * a.scale_log2;
        } else {
            const f32x16 sk = score_tile(Kp, jb);
            if (aligned) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = jb + 8 * (r >> 2) + 4 * half + (r & 3);
                    s[r] = (j <= my_i) ? sk[r] * a.scale_log2 : -INFINITY;
                }
            } else {
                const f32x16 sh = score_tile(Hp, jb);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = jb + 8 * (r >> 2) + 4 * half + (r & 3);
                    const float pick = (j >= my_win) ? sk[r] : sh[r];
                    s[r] = (j <= my_i) ? pick * a.scale_log2 : -INFINITY;
                }
            }
        }
        softmax_pv(s, jb);
    }

    // ---------------------------------------------------------------- epilogue
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (my_valid) {
        const float inv = 1.f / l_tot;
        bf16_t *orow = a.O + (((size_t)b * a.Hq + head0 + my_hh) * n + my_i) * D;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                u32x2 w;
                w[0] = pack_bf16x2(oacc[mt][4 * q4 + 0] * inv, oacc[mt][4 * q4 + 1] * inv);
                w[1] = pack_bf16x2(oacc[mt][4 * q4 + 2] * inv, oacc[mt][4 * q4 + 3] * inv);
                *(u32x2 *)(orow + mt * 32 + 8 * q4 + 4 * half) = w;
            }
    }
}

// V [unit][n][D] -> Vt [unit][D][n_pad], zero beyond n
template <int D>
__global__ __launch_bounds__(256) void transpose_v_kernel(const bf16_t *__restrict__ V, bf16_t *__restrict__ Vt,
                                                          int n, int n_pad) {
    __shared__ bf16_t tile[64][D + 2];
    const int unit = blockIdx.y, t0 = blockIdx.x * 64, tid = threadIdx.x;
    const bf16_t *Vp = V + (size_t)unit * n * D;
    for (int idx = tid; idx < 64 * D; idx += 256) {
        const int r = idx / D, c = idx % D;
        tile[r][c] = (t0 + r < n) ? Vp[(size_t)(t0 + r) * D + c] : (bf16_t)0;
    }
    __syncthreads();
    bf16_t *Op = Vt + (size_t)unit * D * n_pad;
    for (int idx = tid; idx < 64 * D; idx += 256) {
        const int c = idx / 64, r = idx % 64;
        if (t0 + r < n_pad) Op[(size_t)c * n_pad + t0 + r] = tile[r][c];
    }
}

template <int D>
static void launch_d(const PrefillArgs &p, void *vt, int n_pad, hipStream_t s) {
    const int units = p.B * p.Hkv;
    hipLaunchKernelGGL((transpose_v_kernel<D>), dim3((n_pad + 63) / 64, units), dim3(256), 0, s,
                       (const bf16_t *)p.V, (bf16_t *)vt, p.n, n_pad);
    MfmaArgs a;
    a.Q = (const bf16_t *)p.Q;
    a.K = (const bf16_t *)p.K;
    a.Khat = (const bf16_t *)p.Khat;
    a.Vt = (const bf16_t *)vt;
    a.O = (bf16_t *)p.O;
    a.ents = (const Entry *)p.ents;
    a.counts = p.counts;
    a.Hq = p.Hq;
    a.Hkv = p.Hkv;
    a.n = p.n;
    a.n_pad = n_pad;
    a.W = p.W;
    a.rebase = p.rebase;
    const int g = p.Hq / p.Hkv;
    a.GH = (g % 4 == 0) ? 4 : (g % 2 == 0) ? 2 : 1;
    a.RT = kRows / a.GH;
    a.tiles = (p.n + a.RT - 1) / a.RT;
    a.hgroups = g / a.GH;
    a.scale_log2 = p.scale_log2;
    const size_t lds = (size_t)D * kRows * 2 + (size_t)2 * kTB * kRows * 4;
    static bool attr_done = false;
    if (!attr_done) {
        (void)hipFuncSetAttribute((const void *)prefill_mfma_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds);
        attr_done = true;
    }
    const size_t blocks = (size_t)units * a.tiles * a.hgroups;
    hipLaunchKernelGGL((prefill_mfma_kernel<D>), dim3((unsigned)blocks), dim3(512), lds, s, a);
}

int prefill_mfma_n_pad(int n) { return (n + 63) / 64 * 64; }

bool prefill_mfma_supported(const PrefillArgs &p) {
    return p.dtype == 1 && (p.d == 64 || p.d == 128) &&
           (size_t)p.B * p.Hkv * ((p.n + 63) / 64) * (p.Hq / p.Hkv) < ((size_t)1 << 31);
}

void launch_prefill_mfma(const PrefillArgs &p, void *vt, hipStream_t s) {
    const int n_pad = prefill_mfma_n_pad(p.n);
    if (p.d == 64)
        launch_d<64>(p, vt, n_pad, s);
    else
        launch_d<128>(p, vt, n_pad, s);
}

}  // namespace da
