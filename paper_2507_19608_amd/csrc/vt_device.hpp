// Re-ordering of value rows into the matrix-core operand order of the prefill kernels (shared by the stand-alone
// launch, the delta scan's first launch, which takes the re-order along, and the fused short-prompt kernel).
#pragma once
#include "common.hpp"

namespace da {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int kTB = 32;         // key columns per block of the prefill kernels

// V [unit][n][D] -> matrix-core operand order [unit][block of 32 keys][k-step ka][channel tile mt][lane][8]:
// lane l of operand (ka, mt) holds channel 32 mt + l % 32 at keys 16 ka + 4 (l / 32) + {0..3} and
// 16 ka + 8 + 4 (l / 32) + {0..3} of the block (the key order of the score tile's D registers).
// Keys beyond n are zero.  One block of 32 keys by `nt` threads (this one is number `lt`) that share `tile`
// ([kTB][D + 2] bf16); `sync` orders the tile's writes before its reads among those threads.
template <int D, int NT, typename Sync>
__device__ __forceinline__ void transpose_v_block(const bf16_t *__restrict__ Vp, u32x4 *__restrict__ Op, int t0, int n,
                                                  bf16_t (*tile)[D + 2], int lt, Sync sync) {
    constexpr int MT = D / 32;
    constexpr int kIn = kTB * (D / 8) / NT;                      // 16-byte loads per thread, 8 channels of one row each
    static_assert(kTB * (D / 8) % NT == 0 && (2 * MT * 64) % NT == 0, "thread count must divide the tile");
    u32x4 v[kIn];
#pragma unroll
    for (int i = 0; i < kIn; ++i) {                              // every load issued before the first is used
        const int idx = lt + i * NT, r = idx / (D / 8), c = (idx % (D / 8)) * 8;
        v[i] = u32x4{0u, 0u, 0u, 0u};
        if (t0 + r < n) v[i] = *(const u32x4 *)(Vp + (size_t)(t0 + r) * D + c);
    }
#pragma unroll
    for (int i = 0; i < kIn; ++i) {
        const int idx = lt + i * NT, r = idx / (D / 8), c = (idx % (D / 8)) * 8;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            tile[r][c + 2 * k] = (bf16_t)(v[i][k] & 0xffffu);
            tile[r][c + 2 * k + 1] = (bf16_t)(v[i][k] >> 16);
        }
    }
    sync();
#pragma unroll
    for (int i = 0; i < 2 * MT * 64 / NT; ++i) {
        const int idx = lt + i * NT;
        const int l = idx % 64, k = idx / 64, ka = k / MT, mt = k % MT;
        const int ch = mt * 32 + (l & 31), hf = l >> 5;
        u32x4 w;
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const int e = 2 * e2;
            const int key0 = 16 * ka + (e < 4 ? 4 * hf + e : 8 + 4 * hf + (e - 4));
            w[e2] = (uint32_t)tile[key0][ch] | ((uint32_t)tile[key0 + 1][ch] << 16);
        }
        Op[idx] = w;
    }
}

}  // namespace da
