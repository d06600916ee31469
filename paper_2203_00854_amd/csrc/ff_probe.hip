// Calibration probes (diagnostics for the benchmark report, no part of the attention path):
// what this GPU sustains on a bare bf16 matrix-instruction loop and on a plain copy, so that
// roofline fractions can be quoted against measured as well as published peaks.
#include "ff_common.h"

namespace ff {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 probe_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float probe_f32x16;

// Every wavefront issues `iters` rounds of four independent 32x32x16 bf16 matrix instructions
// (four accumulators, so that no instruction waits for the one before it) on operands that never
// leave registers.  2 * 32 * 32 * 16 flop per instruction.
__global__ __launch_bounds__(512, 1) void k_probe_mfma(float* sink, int iters) {
    probe_bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(0.001f * (float)((threadIdx.x + i) & 7));
        b[i] = (__bf16)(0.002f * (float)((threadIdx.x + 3 * i) & 7));
    }
    probe_f32x16 c0, c1, c2, c3;
#pragma unroll
    for (int v = 0; v < 16; ++v) c0[v] = c1[v] = c2[v] = c3[v] = 0.f;
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) s += c0[v] + c1[v] + c2[v] + c3[v];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// dst[i] = src[i], 16 bytes per lane and step, grid-stride
__global__ __launch_bounds__(256) void k_probe_copy(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

constexpr int kProbeBlocks = 512, kProbeThreads = 512;     // two 8-wavefront blocks per compute unit of a 256-unit chip

}  // namespace ff

using namespace ff;

extern "C" {

size_t ff_probe_sink_bytes(void) { return (size_t)kProbeBlocks * kProbeThreads * sizeof(float); }

ff_status ff_probe_mfma(void* sink, int32_t iters, double* flop, void* hip_stream) {
    if (!sink || iters < 1 || !flop) return fail(FF_EINVAL, "ff_probe_mfma: bad argument");
    hipStream_t st = (hipStream_t)hip_stream;
    {
        Timed t(KK_PROBE_MFMA, st);
        hipLaunchKernelGGL(k_probe_mfma, dim3(kProbeBlocks), dim3(kProbeThreads), 0, st, (float*)sink, iters);
    }
    *flop = (double)kProbeBlocks * (kProbeThreads / 64) * (double)iters * 4.0 * (2.0 * 32 * 32 * 16);
    return check_launch("ff_probe_mfma");
}

ff_status ff_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
    if (!dst || !src || bytes < 16 || (bytes & 15u) || ((uintptr_t)dst & 15u) || ((uintptr_t)src & 15u))
        return fail(FF_EINVAL, "ff_probe_copy: pointers and size must be multiples of 16 bytes");
    hipStream_t st = (hipStream_t)hip_stream;
    {
        Timed t(KK_PROBE_COPY, st);
        hipLaunchKernelGGL(k_probe_copy, dim3(256 * 16), dim3(256), 0, st, (uint4*)dst, (const uint4*)src, bytes / 16);
    }
    return check_launch("ff_probe_copy");
}

}  // extern "C"
