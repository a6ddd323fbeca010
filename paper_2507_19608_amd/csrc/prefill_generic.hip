// Generic hybrid-attention prefill (Sec. III-B prefill stage; Eq. 4; Eq. 1): vector ALU only,
// any head_dim that is a multiple of 32 up to 256, fp32 or bf16 inputs, fp32 arithmetic.
//
// One wave per 64 consecutive query rows of one query head; lane = query row.  Every key
// column is wave-uniform, so its compacted (channel, delta) list, its raw key row and its value
// row are read through the scalar path and broadcast; the per-row operand q_i[c] comes from a
// transposed copy of the Q tile in LDS.  A row keeps its Eq. 4 running score in a register and
// its softmax state lane-locally (no cross-lane reductions anywhere).
#include "common.hpp"
#include "kernels.hpp"

namespace da {

template <typename T>
struct KArgs {
    const T *__restrict__ Q;
    const T *__restrict__ K;
    const T *__restrict__ V;
    const T *__restrict__ Khat;
    T *__restrict__ O;
    const EntryChunk *__restrict__ ents;
    const uint32_t *__restrict__ counts;
    int Hq, Hkv, n, W, rebase, sliding;
    int q_off, nq;   // query rows are positions q_off .. q_off + nq - 1 of the n keys
    float scale_log2;
};

template <typename T, int D>
__global__ __launch_bounds__(64) void prefill_generic_kernel(KArgs<T> a) {
    extern __shared__ __attribute__((aligned(16))) float qt[];   // [D][64]: qt[c * 64 + lane] = q_row(lane)[c]
    const int lane = threadIdx.x;
    const int tiles = (a.nq + 63) / 64;
    const int tile = tiles - 1 - (int)blockIdx.x;   // longest rows first
    const int i_first = a.q_off + tile * 64;        // position of the tile's first row
    const int h = blockIdx.y, b = blockIdx.z;
    const int g = a.Hq / a.Hkv;
    const int unit = b * a.Hkv + h / g;
    const int n = a.n, W = a.W;
    const int i = i_first + lane;
    const bool valid = i < n;
    const T *Qp = a.Q + ((size_t)(b * a.Hq + h) * a.nq) * D;
    const T *Kp = a.K + (size_t)unit * n * D;
    const T *Vp = a.V + (size_t)unit * n * D;
    const T *Hp = a.Khat + (size_t)unit * n * D;
    const EntryChunk *Ep = a.ents + (size_t)unit * n * (D / kGroup);
    const uint32_t *Cp = a.counts + (size_t)unit * n;

    for (int c = 0; c < D; ++c) qt[c * 64 + lane] = valid ? load_f32(Qp, (size_t)(i - a.q_off) * D + c) : 0.f;
    __syncthreads();

    const int i_last = min(n - 1, i_first + 63);            // last row of the tile
    // first exact column of row r: start of its square, or of its band (monotone in r either way)
    auto win_start = [&](int r) { return a.sliding ? max(r - W + 1, 0) : (r / W) * W; };
    const int win_first = win_start(i_first);               // window start of the tile's first row
    const int win_last = win_start(i_last);                 // window start of its last row
    const int my_win = valid ? win_start(i) : 0;

    float o[D];
#pragma unroll
    for (int c = 0; c < D; ++c) o[c] = 0.f;
    float m = -INFINITY, l = 0.f;
    // Eq. 4 running score of this row (unscaled).  A column's update is summed in binary32, the running score over
    // the columns in binary64: one add per column, and its rounding then does not grow with the prompt length
    // (in binary32 it reached 1e-4 of the output scale at ~1500 columns with fp32 inputs).
    double r = 0.0;

    constexpr int TB = 16;
    for (int jb = 0; jb <= i_last; jb += TB) {
        float s[TB];
#pragma unroll
        for (int jj = 0; jj < TB; ++jj) {
            const int j = jb + jj;   // wave-uniform
            float sc = -INFINITY;
            if (j <= i_last) {
                float approx = 0.f;
                if (j < win_last) {   // some row of the tile has this column outside its window
                    if (a.rebase) {
                        const T *hj = Hp + (size_t)j * D;
                        for (int c = 0; c < D; ++c) approx = fmaf(qt[c * 64 + lane], load_f32(hj, c), approx);
                    } else {
                        const uint32_t cnt = Cp[j];
                        const EntryChunk *e = Ep + (size_t)j * (D / kGroup);
                        float upd = 0.f;
                        for (uint32_t k = 0; k < cnt; k += kGroup) {
                            const EntryChunk ch = e[k / kGroup];
#pragma unroll
                            for (int u = 0; u < kGroup; ++u) upd = fmaf(qt[ch.chan[u] * 64 + lane], ch.delta[u], upd);
                        }
                        r += (double)upd;
                        approx = (float)r;
                    }
                }
                float exact = 0.f;
                if (j >= win_first) {  // some row of the tile has this column inside its window
                    const T *kj = Kp + (size_t)j * D;
                    for (int c = 0; c < D; ++c) exact = fmaf(qt[c * 64 + lane], load_f32(kj, c), exact);
                }
                const float pick = (j >= my_win) ? exact : approx;
                if (valid && j <= i) sc = pick * a.scale_log2;
            }
            s[jj] = sc;
        }
        float bm = s[0];
#pragma unroll
        for (int jj = 1; jj < TB; ++jj) bm = fmaxf(bm, s[jj]);
        const float m_new = fmaxf(m, bm);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = exp2f(m - m_use);
        l *= alpha;
#pragma unroll
        for (int c = 0; c < D; ++c) o[c] *= alpha;
#pragma unroll
        for (int jj = 0; jj < TB; ++jj) {
            const int j = jb + jj;
            if (j <= i_last) {
                const float p = exp2f(s[jj] - m_use);
                l += p;
                const T *vj = Vp + (size_t)j * D;
#pragma unroll
                for (int c = 0; c < D; ++c) o[c] = fmaf(p, load_f32(vj, c), o[c]);
            }
        }
        m = m_new;
    }
    if (valid) {
        const float inv = 1.f / l;
        T *Op = a.O + ((size_t)(b * a.Hq + h) * a.nq + (i - a.q_off)) * D;
#pragma unroll
        for (int c = 0; c < D; ++c) store_from_f32(Op, c, o[c] * inv);
    }
}

template <typename T, int D>
static void launch_one(const PrefillArgs &p, hipStream_t s) {
    KArgs<T> a;
    a.Q = (const T *)p.Q;
    a.K = (const T *)p.K;
    a.V = (const T *)p.V;
    a.Khat = (const T *)p.Khat;
    a.O = (T *)p.O;
    a.ents = (const EntryChunk *)p.ents;
    a.counts = p.counts;
    a.Hq = p.Hq;
    a.Hkv = p.Hkv;
    a.n = p.n;
    a.q_off = p.q_off;
    a.nq = p.nq;
    a.W = p.W;
    a.sliding = p.sliding;
    a.rebase = p.rebase;
    a.scale_log2 = p.scale_log2;
    const size_t lds = (size_t)D * 64 * sizeof(float);
    static std::atomic<uint64_t> lds_set;   // per instantiation, one bit per device
    ensure_dynamic_lds((const void *)prefill_generic_kernel<T, D>, (int)lds, lds_set);
    dim3 grid((p.nq + 63) / 64, p.Hq, p.B), block(64);
    hipLaunchKernelGGL((prefill_generic_kernel<T, D>), grid, block, lds, s, a);
}

template <typename T>
static bool launch_by_dim(const PrefillArgs &p, hipStream_t s) {
    switch (p.d) {
        case 32: launch_one<T, 32>(p, s); return true;
        case 64: launch_one<T, 64>(p, s); return true;
        case 96: launch_one<T, 96>(p, s); return true;
        case 128: launch_one<T, 128>(p, s); return true;
        case 160: launch_one<T, 160>(p, s); return true;
        case 192: launch_one<T, 192>(p, s); return true;
        case 224: launch_one<T, 224>(p, s); return true;
        case 256: launch_one<T, 256>(p, s); return true;
        default: return false;
    }
}

bool launch_prefill_generic(const PrefillArgs &p, hipStream_t s) {
    return p.dtype == 0 ? launch_by_dim<float>(p, s) : launch_by_dim<bf16_t>(p, s);
}

}  // namespace da
