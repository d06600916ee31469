// Internal declarations shared by the libff translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ff.h"

namespace ff {

typedef uint16_t bf16_t;  // bfloat16 bit pattern

constexpr float kLog2e = 1.4426950408889634f;

// ---- scalar conversions -------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

// ---- wave64 reductions --------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---- the problem as the kernels see it ------------------------------------------------
// Every mode is "R independent batch rows, each a sequence of L tokens".  Token (r, l)
// of the mode lives at x + (r*sr + l*sl) * c; the mask entry of key (r, l) at mask[r*sr + l*sl].
struct Problem {
    int mode, dtype;
    int n_a, n_b, c, c_z, H, d;
    float eps;
    int R, L;          // batch rows, attended length
    int64_t sr, sl;    // token strides
    int Hd;            // H*d
    bool has_bias;
};

struct Workspace {
    float* bias;       // [H, L, L] float32, already multiplied by log2(e); NULL in column mode
    void* qkvg;        // layout is private to each kernel family
    void* o;           // gated context of one chunk
    float* stats;      // generic family: mean, rstd per token of one chunk
    void* prep;        // matrix-core family: prepared weights
    size_t total;      // bytes
    int chunk;         // batch rows per chunk the tensors above are sized for
};

// kernel kinds for the launch timer (ff_profile_* in the C ABI)
enum KernelKind { KK_PREP = 0, KK_BIAS, KK_PROJ, KK_ATTN, KK_OUT, KK_LAYERNORM, KK_GENERIC, KK_PROBE_MFMA, KK_PROBE_COPY,
                  KK_TM_PREP, KK_TM_PROJ, KK_TM_MUL, KK_TM_OUT, KK_GCA_KV, KK_GCA_SOFTMAX, KK_GCA_OUT,
                  KK_BWD_STATS, KK_BWD_DQ, KK_BWD_DKV, KK_BWD_DBIAS, KK_PROBE_VALU, KK_PROJ_ATTN, KK_COUNT };
void prof_begin(int kind, hipStream_t st);
void prof_end(int kind, hipStream_t st);
// brackets the launches issued in its scope with HIP events when the timer is on
struct Timed {
    int kind;
    hipStream_t st;
    Timed(int k, hipStream_t s) : kind(k), st(s) { prof_begin(k, s); }
    ~Timed() { prof_end(kind, st); }
};

// error plumbing (ff_api.hip)
ff_status fail(ff_status st, const char* fmt, ...);
ff_status check_launch(const char* what);

// ---- kernel families (each returns after enqueueing on `stream`) ---------------------
// generic float32 vector path (ff_generic.hip); T selected by p.dtype
size_t generic_workspace(const Problem& p, int chunk, Workspace* ws, void* base);
// once per call, before the chunks: the pair-bias tensor (and, for the matrix-core family, the
// prepared weights)
ff_status generic_prepare(const Problem& p, const ff_attn_weights& w, const void* x, const void* z,
                          const Workspace& ws, hipStream_t stream);
// the generic bias kernel writing into a [H][Lq][Lp] tensor (both families use it)
ff_status generic_bias_into(const Problem& p, const ff_attn_weights& w, const void* x, const void* z, float* bias,
                            int Lq, int Lp, hipStream_t stream);
// res: NULL, or a tensor laid out like out that is added to the module's output (may be out itself)
ff_status generic_chunk(const Problem& p, const ff_attn_weights& w, const void* x, const float* mask,
                        const void* res, void* out, const Workspace& ws, int r0, int rows, hipStream_t stream);

// bf16 matrix-core path (ff_mfma_*.hip)
bool mfma_supported(const Problem& p);
// whether `chunk` batch rows per launch are within the family's limits (else the generic family runs)
bool mfma_chunk_ok(const Problem& p, int chunk);
size_t mfma_workspace(const Problem& p, int chunk, Workspace* ws, void* base);
ff_status mfma_prepare(const Problem& p, const ff_attn_weights& w, const void* x, const void* z,
                       const Workspace& ws, hipStream_t stream);
ff_status mfma_chunk(const Problem& p, const ff_attn_weights& w, const void* x, const float* mask,
                     const void* res, void* out, const Workspace& ws, int r0, int rows, hipStream_t stream);

// compute units of the current device (queried once; 256 if the query fails); sizes the persistent grids
int compute_units();

// triangular multiplicative update (ff_trimul.hip), bf16 matrix-core kernels only
bool trimul_supported(int dtype, int cz, int c);
size_t trimul_workspace(int N, int cz, int c);
// residual: z is added to the module's output (out may then be z itself)
ff_status trimul_run(const ff_trimul_desc& d, const ff_trimul_weights& w, const void* z, const float* mask, bool residual,
                     void* out, void* ws, hipStream_t stream);

// global column attention of the extra-MSA stack (ff_global.hip), bf16 only
bool global_supported(const ff_global_desc& d);
size_t global_workspace(const ff_global_desc& d);
ff_status global_run(const ff_global_desc& d, const ff_global_weights& w, const void* m, const float* mask, void* out,
                     void* ws, hipStream_t stream);

// backward pass of the fused attention core (ff_attn_bwd.hip), bf16 only
bool core_backward_supported(const ff_core_desc& d);
size_t core_backward_workspace(const ff_core_desc& d);
ff_status core_backward_run(const ff_core_desc& d, const void* q, const void* k, const void* v, const void* g, const float* bias,
                            const float* mask, const void* dout, void* dq, void* dk, void* dv, void* dg, float* dbias,
                            void* ws, hipStream_t stream);

// LayerNorm (ff_layernorm.hip)
ff_status layernorm_launch(const void* x, const void* g, const void* b, void* y, int64_t rows, int c,
                           float eps, int dt, hipStream_t stream);

}  // namespace ff
