// Calibration probes (diagnostics for the benchmark report, no part of the attention path):
// what this GPU sustains on a bare bf16 matrix-instruction loop, on a plain copy and on loops of single
// vector instructions, so that roofline fractions can be quoted against measured as well as published peaks.
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

// Every wavefront issues `iters` rounds of 16 independent vector instructions of one kind (16 registers, so
// that none waits for the one before it): what one SIMD spends per wavefront-wide instruction of that kind.
//   0: v_fma_f32   1: v_exp_f32   2: v_cvt_pk_bf16_f32 (two floats -> a bfloat16 pair)   3: v_dot2c_f32_bf16
template <int KIND>
__global__ __launch_bounds__(256) void k_probe_valu(float* sink, int iters, float seed) {
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf2;
    float r[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) r[i] = seed + (float)i * 0.001f + (float)threadIdx.x * 1e-6f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (KIND == 0) r[i] = __builtin_fmaf(r[i], 0.999f, 0.001f);
            else if (KIND == 1) r[i] = __builtin_amdgcn_exp2f(r[i]);
            else if (KIND == 2) {
                bf2 t;
                t[0] = (__bf16)r[i];
                t[1] = (__bf16)r[(i + 1) & 15];
                r[i] = __builtin_bit_cast(float, t);
            } else r[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, r[(i + 1) & 15]), __builtin_bit_cast(bf2, 0x3f803f80u), r[i], false);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += r[i];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Do matrix and vector instructions of one SIMD overlap?  Every wavefront issues `iters` rounds of four independent
// 32x32x16 bf16 matrix instructions with NV independent vector instructions (multiply-adds, or exponentials if EXP)
// spread evenly between them.
template <int NV, bool EXP>
__global__ __launch_bounds__(256) void k_probe_mix(float* sink, int iters, float seed) {
    probe_bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(0.001f * (float)((threadIdx.x + i) & 7));
        b[i] = (__bf16)(0.002f * (float)((threadIdx.x + 3 * i) & 7));
    }
    probe_f32x16 c[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) c[t][v] = 0.f;
    float r[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) r[i] = seed + (float)i * 0.001f + (float)threadIdx.x * 1e-6f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            c[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[t], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < NV / 4; ++i) {
                const int k = (t * (NV / 4) + i) & 15;
                r[k] = EXP ? __builtin_amdgcn_exp2f(r[k]) : __builtin_fmaf(r[k], 0.999f, 0.001f);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += r[i];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += c[t][v];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
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

ff_status ff_probe_valu(void* sink, int32_t kind, int32_t iters, double* wave_insts, void* hip_stream) {
    if (!sink || kind < 0 || kind > 7 || iters < 1 || !wave_insts) return fail(FF_EINVAL, "ff_probe_valu: bad argument");
    hipStream_t st = (hipStream_t)hip_stream;
    const int blocks = 1024;                                   // x 256 threads = the sink's size: eight wavefronts per SIMD of a 256-unit chip
    {
        Timed t(KK_PROBE_VALU, st);
        if (kind == 0) hipLaunchKernelGGL(k_probe_valu<0>, dim3(blocks), dim3(256), 0, st, (float*)sink, iters, 0.5f);
        else if (kind == 1) hipLaunchKernelGGL(k_probe_valu<1>, dim3(blocks), dim3(256), 0, st, (float*)sink, iters, 0.5f);
        else if (kind == 2) hipLaunchKernelGGL(k_probe_valu<2>, dim3(blocks), dim3(256), 0, st, (float*)sink, iters, 0.5f);
        else if (kind == 3) hipLaunchKernelGGL(k_probe_valu<3>, dim3(blocks), dim3(256), 0, st, (float*)sink, iters, 0.5f);
        else if (kind == 4) hipLaunchKernelGGL((k_probe_mix<0, false>), dim3(blocks), dim3(256), 0, st, (float*)sink, iters, 0.5f);
        else if (kind == 5) hipLaunchKernelGGL((k_probe_mix<16, false>), dim3(blocks), dim3(256), 0, st, (float*)sink, iters, 0.5f);
        else if (kind == 6) hipLaunchKernelGGL((k_probe_mix<32, false>), dim3(blocks), dim3(256), 0, st, (float*)sink, iters, 0.5f);
        else hipLaunchKernelGGL((k_probe_mix<16, true>), dim3(blocks), dim3(256), 0, st, (float*)sink, iters, 0.5f);
    }
    // kinds 0 .. 3: instructions of the kind; kinds 4 .. 7: rounds (of four matrix instructions each)
    *wave_insts = (double)blocks * 4.0 * (double)iters * (kind < 4 ? 16.0 : 1.0);
    return check_launch("ff_probe_valu");
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
