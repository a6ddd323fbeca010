// Measurement aids behind the C ABI: a streaming-read kernel and arithmetic-rate kernels that give the rates this
// chip reaches on the access pattern and instruction forms of the library's own kernels.  Not part of the attention path.
#include "../../include/delta_attn.h"
#include "common.hpp"
#include "kernels.hpp"

using namespace da;

namespace {
typedef __attribute__((ext_vector_type(4))) uint32_t stream_u32x4;
// streaming read: a wave sums 16 pieces of 1 KiB; the (never true) comparison keeps the loads alive
__global__ __launch_bounds__(64) void stream_read_kernel(const stream_u32x4 *__restrict__ src, size_t pieces,
                                                         uint32_t *__restrict__ sink) {
    const size_t p0 = (size_t)blockIdx.x * 16;
    stream_u32x4 acc = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        stream_u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const size_t p = p0 + half * 8 + u;
            const size_t i = p * 64 + threadIdx.x;
            v[u] = i < pieces * 64 ? src[i] : stream_u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u && acc[0] == 0x7f4a7c15u && acc[1] == 0x12345678u) *sink = acc[2];
}
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;
typedef __attribute__((ext_vector_type(16))) float probe_f32x16;
// arithmetic-rate probes: every wave runs `iters` rounds of independent chains that depend on nothing in memory
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, float *__restrict__ sink) {
    probe_bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(0.001f * (float)((threadIdx.x + i) & 7));
        b[i] = (__bf16)(0.002f * (float)((threadIdx.x * 3 + i) & 7));
    }
    probe_f32x16 acc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[k][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[k][r];
    if (s == 12345.678f) *sink = s;
}

// kLiteral: the multiplier is an instruction literal (two register sources per multiply-add); otherwise all three
// operands are registers, as in the library's gather loop.  8 rounds per loop trip, so that the loop's own scalar
// instructions and branch do not show in the rate.
template <bool kLiteral>
__global__ __launch_bounds__(256) void fma_rate_kernel(int iters, float *__restrict__ sink) {
    float x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = 0.001f * (float)(threadIdx.x + i);
    const float m = 0.999f + 1e-6f * (float)(threadIdx.x & 1), c = 0.0001f * (float)(threadIdx.x & 3);
    for (int it = 0; it < iters; it += 8) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = kLiteral ? fmaf(x[i], 0.999f, c) : fmaf(x[i], m, c);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += x[i];
    if (s == 12345.678f) *sink = s;
}

// The multiply-add of the prefill kernel's gather loop: fp16 multiplicand widened inside the instruction, fp32
// multiplier and accumulator (v_fma_mix_f32).  Written as single instructions because the compiler would otherwise
// widen the loop-invariant fp16 values once, outside the loop, and time plain fp32 multiply-adds.
__global__ __launch_bounds__(256) void fma_mix_rate_kernel(int iters, float *__restrict__ sink) {
    float x[16];
    uint32_t qh[4];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = 0.001f * (float)(threadIdx.x + i);
#pragma unroll
    for (int i = 0; i < 4; ++i) qh[i] = 0x34003400u + ((threadIdx.x + i) & 15);   // two fp16 values near 0.25
    const float m = 0.999f + 1e-6f * (float)(threadIdx.x & 1);
    for (int it = 0; it < iters; it += 8) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                asm volatile("v_fma_mix_f32 %0, %1, %2, %0 op_sel_hi:[1,0,0]" : "+v"(x[i]) : "v"(qh[i & 3]), "v"(m));
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += x[i];
    if (s == 12345.678f) *sink = s;
}
}  // namespace

extern "C" {

da_status delta_attn_stream_read(const void *src, size_t bytes, uint32_t *sink, void *hip_stream) {
    if (!src || !sink || bytes == 0 || bytes % 1024 != 0) return DA_ERR_INVALID_ARG;
    const size_t pieces = bytes / 1024;                      // 1 KiB per wave-wide 128-bit load
    const size_t groups = (pieces + 15) / 16;
    if (groups > 0x7fffffffull) return DA_ERR_UNSUPPORTED;
    (void)hipGetLastError();
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)groups), dim3(64), 0, (hipStream_t)hip_stream,
                       (const stream_u32x4 *)src, pieces, sink);
    return launch_ok("stream_read") ? DA_OK : DA_ERR_HIP;
}

da_status delta_attn_rate_probe(int32_t kind, int32_t work_groups, int32_t iters, float *sink, double *flop,
                                void *hip_stream) {
    if (!sink || !flop || work_groups < 1 || iters < 1 || kind < 0 || kind > 3) return DA_ERR_INVALID_ARG;
    (void)hipGetLastError();
    const double waves = 4.0 * work_groups;
    if (kind == 0) {
        hipLaunchKernelGGL(mfma_rate_kernel, dim3(work_groups), dim3(256), 0, (hipStream_t)hip_stream, iters, sink);
        *flop = waves * iters * 4.0 * (2.0 * 32 * 32 * 16);
    } else {
        iters = (iters + 7) / 8 * 8;
        if (kind == 3)
            hipLaunchKernelGGL(fma_mix_rate_kernel, dim3(work_groups), dim3(256), 0, (hipStream_t)hip_stream, iters,
                               sink);
        else if (kind == 1)
            hipLaunchKernelGGL(fma_rate_kernel<true>, dim3(work_groups), dim3(256), 0, (hipStream_t)hip_stream, iters,
                               sink);
        else
            hipLaunchKernelGGL(fma_rate_kernel<false>, dim3(work_groups), dim3(256), 0, (hipStream_t)hip_stream, iters,
                               sink);
        *flop = waves * iters * 16.0 * 64.0 * 2.0;
    }
    return launch_ok("rate_probe") ? DA_OK : DA_ERR_HIP;
}

}  // extern "C"
