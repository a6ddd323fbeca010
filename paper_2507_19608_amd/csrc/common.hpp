// Shared device helpers for the hybrid delta attention kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace da {

typedef unsigned short bf16_t;   // raw bfloat16 bits

constexpr int kWave = 64;
constexpr int kGroup = 8;        // compacted entry lists are padded to a multiple of this (one "chunk")

// Compacted delta entries of a key column are stored in chunks of kGroup entries: 8 channel
// indices (uint32) followed by 8 delta values (binary32), 64 bytes.  Unused slots hold channel 0
// with delta 0.  A column of head_dim d owns room for d / 8 chunks.
struct __attribute__((aligned(64))) EntryChunk {
    uint32_t chan[8];
    float delta[8];
};

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }
__device__ __forceinline__ float load_f32(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_f32(const bf16_t *p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void store_from_f32(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_from_f32(bf16_t *p, size_t i, float v) { p[i] = f32_to_bf16(v); }

// number of set bits of a 64-bit wave mask below this lane
__device__ __forceinline__ uint32_t lanes_below(uint64_t m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// Work-group barrier for hand-offs through LDS.  __syncthreads() is a fence over every address space: before
// its s_barrier a wave also waits for all of its outstanding global loads, so a prefetch issued ahead of the
// barrier is drained at it.  This one orders LDS traffic only; global loads stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// exclusive prefix sum over the 64 lanes; *total receives the wave sum
__device__ __forceinline__ uint32_t wave_exclusive_scan(uint32_t v, uint32_t *total) {
    const int lane = threadIdx.x & 63;
    uint32_t inc = v;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        const uint32_t o = __shfl_up(inc, s);
        if (lane >= s) inc += o;
    }
    *total = __shfl(inc, 63);
    return inc - v;
}

}  // namespace da
