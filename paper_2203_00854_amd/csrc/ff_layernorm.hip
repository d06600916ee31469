// LayerNorm over the last axis (FastFold Section 5.2: the batch-reduction kernel for small
// hidden sizes).  The paper gives one warp per row with register-level reductions; on a
// 64-wide wavefront a 128- or 256-channel row fills only part of a wave with 16-byte
// loads, so a row is given to a power-of-two group of G <= 64 lanes and several rows share
// a wavefront.  The row stays in registers: one read and one write of HBM per element,
// mean and variance in float32 from two in-register passes.
#include "ff_common.h"

namespace ff {

template <typename T> struct Vec16;  // 16 bytes of T
template <> struct Vec16<float> { static constexpr int N = 4; };
template <> struct Vec16<bf16_t> { static constexpr int N = 8; };

template <typename T, int N> __device__ __forceinline__ void load16(const T* p, float (&v)[N]) {
    uint4 raw = *reinterpret_cast<const uint4*>(p);
    if constexpr (sizeof(T) == 4) {
        v[0] = __uint_as_float(raw.x); v[1] = __uint_as_float(raw.y);
        v[2] = __uint_as_float(raw.z); v[3] = __uint_as_float(raw.w);
    } else {
        const uint32_t r[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(r[i] << 16);
            v[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
        }
    }
}

template <typename T, int N> __device__ __forceinline__ void store16(T* p, const float (&v)[N]) {
    uint4 raw;
    if constexpr (sizeof(T) == 4) {
        raw.x = __float_as_uint(v[0]); raw.y = __float_as_uint(v[1]);
        raw.z = __float_as_uint(v[2]); raw.w = __float_as_uint(v[3]);
    } else {
        uint32_t r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = (uint32_t)f32_to_bf16(v[2 * i]) | ((uint32_t)f32_to_bf16(v[2 * i + 1]) << 16);
        raw.x = r[0]; raw.y = r[1]; raw.z = r[2]; raw.w = r[3];
    }
    *reinterpret_cast<uint4*>(p) = raw;
}

// Rows of c = chunks*N elements; a group of G lanes owns a row, lane g of the group holds
// 16-byte pieces g, g+G, ... (ITERS of them, the tail ones possibly past the row).
template <typename T, int ITERS>
__global__ __launch_bounds__(256) void k_layernorm_vec(const T* __restrict__ x, const T* __restrict__ gamma,
                                                        const T* __restrict__ beta, T* __restrict__ y,
                                                        int64_t rows, int c, int G, float eps) {
    constexpr int N = Vec16<T>::N;
    const int lane_in_group = threadIdx.x & (G - 1);
    const int groups_per_block = 256 / G;
    const int chunks = c / N;
    float gm[ITERS][N], bt[ITERS][N];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int ch = lane_in_group + it * G;
        if (ch < chunks) {
            load16<T, N>(gamma + (size_t)ch * N, gm[it]);
            load16<T, N>(beta + (size_t)ch * N, bt[it]);
        }
    }
    const float inv_c = 1.f / (float)c;
    for (int64_t row = (int64_t)blockIdx.x * groups_per_block + threadIdx.x / G; row < rows;
         row += (int64_t)gridDim.x * groups_per_block) {
        const T* xr = x + row * c;
        float v[ITERS][N];
        float s = 0.f;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            int ch = lane_in_group + it * G;
            if (ch < chunks) {
                load16<T, N>(xr + (size_t)ch * N, v[it]);
#pragma unroll
                for (int i = 0; i < N; ++i) s += v[it][i];
            }
        }
        for (int o = G >> 1; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        const float mean = s * inv_c;
        float q = 0.f;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            int ch = lane_in_group + it * G;
            if (ch < chunks) {
#pragma unroll
                for (int i = 0; i < N; ++i) {
                    float t = v[it][i] - mean;
                    q += t * t;
                }
            }
        }
        for (int o = G >> 1; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
        const float rstd = rsqrtf(q * inv_c + eps);
        T* yr = y + row * c;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            int ch = lane_in_group + it * G;
            if (ch < chunks) {
                float o[N];
#pragma unroll
                for (int i = 0; i < N; ++i) o[i] = (v[it][i] - mean) * rstd * gm[it][i] + bt[it][i];
                store16<T, N>(yr + (size_t)ch * N, o);
            }
        }
    }
}

// Any c: one wavefront per row, scalar accesses, the row is re-read from cache.
template <typename T>
__global__ __launch_bounds__(256) void k_layernorm_any(const T* __restrict__ x, const T* __restrict__ gamma,
                                                        const T* __restrict__ beta, T* __restrict__ y,
                                                        int64_t rows, int c, float eps) {
    const int lane = threadIdx.x & 63;
    const float inv_c = 1.f / (float)c;
    for (int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); row < rows; row += (int64_t)gridDim.x * 4) {
        const T* xr = x + row * c;
        float s = 0.f;
        for (int i = lane; i < c; i += 64) s += to_f32<T>(xr[i]);
        const float mean = wave_sum(s) * inv_c;
        float q = 0.f;
        for (int i = lane; i < c; i += 64) {
            float t = to_f32<T>(xr[i]) - mean;
            q += t * t;
        }
        const float rstd = rsqrtf(wave_sum(q) * inv_c + eps);
        T* yr = y + row * c;
        for (int i = lane; i < c; i += 64) {
            float t = (to_f32<T>(xr[i]) - mean) * rstd * to_f32<T>(gamma[i]) + to_f32<T>(beta[i]);
            yr[i] = from_f32<T>(t);
        }
    }
}

template <typename T>
static ff_status launch_t(const T* x, const T* g, const T* b, T* y, int64_t rows, int c, float eps, hipStream_t st) {
    constexpr int N = Vec16<T>::N;
    const bool aligned = (((uintptr_t)x | (uintptr_t)y | (uintptr_t)g | (uintptr_t)b) & 15u) == 0;
    const int chunks = c / N;
    if (aligned && c % N == 0 && chunks <= 256) {
        int G = 1;
        while (G < chunks && G < 64) G <<= 1;
        const int iters = (chunks + G - 1) / G;
        const int rows_per_block = 256 / G;
        int64_t blocks = (rows + rows_per_block - 1) / rows_per_block;
        const int64_t cap = 256 * 16;  // persistent-ish: every block loops over rows
        if (blocks > cap) blocks = cap;
        dim3 grid((unsigned)blocks), blk(256);
        if (iters == 1) hipLaunchKernelGGL((k_layernorm_vec<T, 1>), grid, blk, 0, st, x, g, b, y, rows, c, G, eps);
        else if (iters == 2) hipLaunchKernelGGL((k_layernorm_vec<T, 2>), grid, blk, 0, st, x, g, b, y, rows, c, G, eps);
        else hipLaunchKernelGGL((k_layernorm_vec<T, 4>), grid, blk, 0, st, x, g, b, y, rows, c, G, eps);
    } else {
        int64_t blocks = (rows + 3) / 4;
        if (blocks > 256 * 16) blocks = 256 * 16;
        hipLaunchKernelGGL((k_layernorm_any<T>), dim3((unsigned)blocks), dim3(256), 0, st, x, g, b, y, rows, c, eps);
    }
    return check_launch("ff_layernorm");
}

ff_status layernorm_launch(const void* x, const void* g, const void* b, void* y, int64_t rows, int c, float eps,
                           int dt, hipStream_t stream) {
    if (dt == FF_F32)
        return launch_t<float>((const float*)x, (const float*)g, (const float*)b, (float*)y, rows, c, eps, stream);
    return launch_t<bf16_t>((const bf16_t*)x, (const bf16_t*)g, (const bf16_t*)b, (bf16_t*)y, rows, c, eps, stream);
}

}  // namespace ff
