// Generic kernel family: every step of the gated attention in float32 vector arithmetic,
// for any shape and for both storage types.  It is the float32 path (no bfloat16 anywhere
// when T = float) and the fallback for bfloat16 shapes the matrix-core family does not
// take.  Steps follow FastFold Section 2.1 (projections, scaled dot product, softmax,
// product with V, output linear), Section 2.3 (axes, pair bias) and Section 5.2 (softmax
// with the mask and bias addends fused in; gate = bias + sigmoid + product).
//
// Workspace layout of this family, per chunk of `rows` batch rows, token t = rl*L + l:
//   stats [tokens][2]   float32 mean, 1/std of LayerNorm
//   qkvg  [tokens][4*Hd] T : q (times log2(e)/sqrt(d)), k, v, sigmoid gate
//   o     [tokens][Hd]   T : gate * context
//   bias  [H][L][L]      float32, times log2(e)
#include "ff_common.h"

namespace ff {

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t generic_workspace(const Problem& p, int chunk, Workspace* ws, void* base) {
    const size_t esz = p.dtype == FF_F32 ? 4 : 2;
    const size_t tokens = (size_t)chunk * p.L;
    size_t off = 0;
    char* b = (char*)base;
    ws->bias = nullptr;
    if (p.has_bias) {
        ws->bias = (float*)(b + off);
        off += align256((size_t)p.H * p.L * p.L * 4);
    }
    ws->prep = nullptr;
    ws->stats = (float*)(b + off);
    off += align256(tokens * 2 * 4);
    ws->qkvg = b + off;
    off += align256(tokens * 4 * p.Hd * esz);
    ws->o = b + off;
    off += align256(tokens * p.Hd * esz);
    ws->total = off;
    ws->chunk = chunk;
    return off;
}

// ---------------------------------------------------------------------------------------
// Bias: one wavefront per pair (q, k): LayerNorm of the source token, then H dot products.
// bias[h][q][k] = log2(e) * sum_c LN(src[(q*sq + k*sk)*c ...])_c * w_b[h][c]
template <typename T>
__global__ __launch_bounds__(256) void k_bias_generic(const T* __restrict__ src, int64_t sq, int64_t sk, int c,
                                                       const T* __restrict__ g, const T* __restrict__ b,
                                                       const T* __restrict__ wb, int H, int L, int Lq, int Lp, float eps,
                                                       float* __restrict__ bias) {
    const int lane = threadIdx.x & 63;
    const int64_t pair = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pair >= (int64_t)L * L) return;
    const int q = (int)(pair / L), k = (int)(pair % L);
    const T* v = src + ((int64_t)q * sq + (int64_t)k * sk) * c;
    float s = 0.f;
    for (int i = lane; i < c; i += 64) s += to_f32<T>(v[i]);
    const float mean = wave_sum(s) / (float)c;
    float qq = 0.f;
    for (int i = lane; i < c; i += 64) {
        float t = to_f32<T>(v[i]) - mean;
        qq += t * t;
    }
    const float rstd = rsqrtf(wave_sum(qq) / (float)c + eps);
    for (int h = 0; h < H; ++h) {
        float acc = 0.f;
        for (int i = lane; i < c; i += 64) {
            float xh = (to_f32<T>(v[i]) - mean) * rstd * to_f32<T>(g[i]) + to_f32<T>(b[i]);
            acc += xh * to_f32<T>(wb[(size_t)h * c + i]);
        }
        acc = wave_sum(acc);
        if (lane == 0) bias[((size_t)h * Lq + q) * Lp + k] = acc * kLog2e;
    }
}

// ---------------------------------------------------------------------------------------
// LayerNorm statistics of the tokens of one chunk: one wavefront per token.
template <typename T>
__global__ __launch_bounds__(256) void k_stats_generic(const T* __restrict__ x, int64_t sr, int64_t sl, int c, int L,
                                                        int r0, int tokens, float eps, float* __restrict__ stats) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= tokens) return;
    const int rl = t / L, l = t % L;
    const T* v = x + ((int64_t)(r0 + rl) * sr + (int64_t)l * sl) * c;
    float s = 0.f;
    for (int i = lane; i < c; i += 64) s += to_f32<T>(v[i]);
    const float mean = wave_sum(s) / (float)c;
    float q = 0.f;
    for (int i = lane; i < c; i += 64) {
        float u = to_f32<T>(v[i]) - mean;
        q += u * u;
    }
    q = wave_sum(q);
    if (lane == 0) {
        stats[2 * (size_t)t] = mean;
        stats[2 * (size_t)t + 1] = rsqrtf(q / (float)c + eps);
    }
}

// ---------------------------------------------------------------------------------------
// Tiled float32 GEMM, 64 tokens x 64 features per block, 4x4 outputs per thread.
//   PROJ = true : A = LayerNorm(x) on the fly (stats, gamma, beta), B rows from w_q|w_k|w_v|w_g,
//                 epilogue: q scaled, gate = sigmoid(acc + b_g); C -> qkvg[t][4Hd]
//   PROJ = false: A = o[t][Hd], B = w_o, epilogue + b_o, C -> out at the token's address.
struct GenericGemmArgs {
    const void* a;         // x (PROJ) or o
    int64_t sr, sl;        // token strides of x / out
    int L, r0, tokens;     // chunk geometry
    int K, N;              // contraction length, output features
    const float* stats;
    const void *ln_g, *ln_b;
    const void* w[4];      // PROJ: w_q, w_k, w_v, w_g ([Hd][K] each); else w[0] = w_o [N][K]
    const void* bvec;      // PROJ: b_g [Hd]; else b_o [N]
    int Hd;
    float qscale;
    void* cdst;            // qkvg or out
    const void* res;       // !PROJ: residual added to the output (laid out like out, may be out itself) or NULL
};

template <typename T, bool PROJ>
__global__ __launch_bounds__(256) void k_gemm_generic(GenericGemmArgs g) {
    __shared__ float As[16][64 + 1];
    __shared__ float Bs[16][64 + 1];
    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
    const int tx = tid & 15, ty = tid >> 4;   // thread owns tokens ty*4.., features tx*4..
    float acc[4][4] = {};
    // loader mapping: thread loads element (row = tid / 16 + 16*j, kk = tid % 16)
    const int lk = tid & 15, lrow = tid >> 4;
    for (int k0 = 0; k0 < g.K; k0 += 16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = lrow + 16 * j;
            const int t = t0 + row, kk = k0 + lk;
            float av = 0.f;
            if (t < g.tokens && kk < g.K) {
                if constexpr (PROJ) {
                    const int rl = t / g.L, l = t % g.L;
                    const T* xp = (const T*)g.a + ((int64_t)(g.r0 + rl) * g.sr + (int64_t)l * g.sl) * g.K;
                    const float mean = g.stats[2 * (size_t)t], rstd = g.stats[2 * (size_t)t + 1];
                    av = (to_f32<T>(xp[kk]) - mean) * rstd * to_f32<T>(((const T*)g.ln_g)[kk]) +
                         to_f32<T>(((const T*)g.ln_b)[kk]);
                } else {
                    av = to_f32<T>(((const T*)g.a)[(size_t)t * g.K + kk]);
                }
            }
            As[lk][row] = av;
            const int n = n0 + row;
            float bv = 0.f;
            if (n < g.N && kk < g.K) {
                if constexpr (PROJ) {
                    const T* wp = (const T*)g.w[n / g.Hd];
                    bv = to_f32<T>(wp[(size_t)(n % g.Hd) * g.K + kk]);
                } else {
                    bv = to_f32<T>(((const T*)g.w[0])[(size_t)n * g.K + kk]);
                }
            }
            Bs[lk][row] = bv;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int i = 0; i < 4; ++i) b[i] = Bs[kk][tx * 4 + i];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = t0 + ty * 4 + i;
        if (t >= g.tokens) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= g.N) continue;
            float v = acc[i][j];
            if constexpr (PROJ) {
                const int seg = n / g.Hd;
                if (seg == 0) v *= g.qscale;
                if (seg == 3) v = 1.f / (1.f + __expf(-(v + to_f32<T>(((const T*)g.bvec)[n - 3 * g.Hd]))));
                ((T*)g.cdst)[(size_t)t * g.N + n] = from_f32<T>(v);
            } else {
                v += to_f32<T>(((const T*)g.bvec)[n]);
                const int rl = t / g.L, l = t % g.L;
                const int64_t at = ((int64_t)(g.r0 + rl) * g.sr + (int64_t)l * g.sl) * g.N + n;
                // (the thread that stores an element is the one that read it: in place is safe)
                if (g.res) v += to_f32<T>(((const T*)g.res)[at]);
                ((T*)g.cdst)[at] = from_f32<T>(v);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Attention: one wavefront per (batch row, head, query).  Two sweeps over the keys: the
// first finds the maximum logit over unmasked keys, the second accumulates exp2(logit - max)
// and the weighted values; lane j owns keys j, j+64, ...  A query without any unmasked key
// gets zero context.  Output o = gate * context.
template <typename T, int D>
__global__ __launch_bounds__(256) void k_attn_generic(const T* __restrict__ qkvg, const float* __restrict__ bias,
                                                       const float* __restrict__ mask, int64_t sr, int64_t sl,
                                                       int r0, int rows, int L, int H, int d,
                                                       T* __restrict__ o) {
    __shared__ float qs[4][D];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t item = (int64_t)blockIdx.x * 4 + wv;      // ((rl*H + h)*L + q)
    const bool active = item < (int64_t)rows * H * L;
    const int qi = active ? (int)(item % L) : 0;
    const int h = active ? (int)((item / L) % H) : 0;
    const int rl = active ? (int)(item / ((int64_t)L * H)) : 0;
    const int Hd = H * d, N4 = 4 * Hd;
    const T* base = qkvg + (size_t)rl * L * N4;
    for (int e = lane; e < D; e += 64) qs[wv][e] = (e < d) ? to_f32<T>(base[(size_t)qi * N4 + h * d + e]) : 0.f;
    __syncthreads();
    if (!active) return;
    const float* brow = bias ? bias + ((size_t)h * L + qi) * L : nullptr;
    const float* mrow = mask ? mask + (int64_t)(r0 + rl) * sr : nullptr;
    const float ninf = -INFINITY;
    float m = ninf;
    for (int k = lane; k < L; k += 64) {
        if (mrow && mrow[(int64_t)k * sl] == 0.f) continue;
        const T* kp = base + (size_t)k * N4 + Hd + h * d;
        float s = 0.f;
        for (int e = 0; e < d; ++e) s += qs[wv][e] * to_f32<T>(kp[e]);
        if (brow) s += brow[k];
        m = fmaxf(m, s);
    }
    m = wave_max(m);
    float acc[D];
#pragma unroll
    for (int e = 0; e < D; ++e) acc[e] = 0.f;
    float sum = 0.f;
    if (m != ninf) {
        for (int k = lane; k < L; k += 64) {
            if (mrow && mrow[(int64_t)k * sl] == 0.f) continue;
            const T* kp = base + (size_t)k * N4 + Hd + h * d;
            float s = 0.f;
            for (int e = 0; e < d; ++e) s += qs[wv][e] * to_f32<T>(kp[e]);
            if (brow) s += brow[k];
            const float pr = exp2f(s - m);
            sum += pr;
            const T* vp = base + (size_t)k * N4 + 2 * Hd + h * d;
#pragma unroll
            for (int e = 0; e < D; ++e)
                if (e < d) acc[e] += pr * to_f32<T>(vp[e]);
        }
    }
    sum = wave_sum(sum);
    const float inv = sum > 0.f ? 1.f / sum : 0.f;
    T* op = o + ((size_t)rl * L + qi) * Hd + h * d;
    const T* gp = base + (size_t)qi * N4 + 3 * Hd + h * d;
#pragma unroll
    for (int e = 0; e < D; ++e) {
        const float tot = wave_sum(acc[e]);
        if (e < d && lane == (e & 63)) op[e] = from_f32<T>(tot * inv * to_f32<T>(gp[e]));
    }
}

// ---------------------------------------------------------------------------------------
template <typename T>
static ff_status bias_t(const Problem& p, const ff_attn_weights& w, const void* x, const void* z, float* bias, int Lq,
                        int Lp, hipStream_t st) {
    const int64_t pairs = (int64_t)p.L * p.L;
    const unsigned blocks = (unsigned)((pairs + 3) / 4);
    if (p.mode == FF_MSA_ROW)
        hipLaunchKernelGGL((k_bias_generic<T>), dim3(blocks), dim3(256), 0, st, (const T*)z, (int64_t)p.L, (int64_t)1,
                           p.c_z, (const T*)w.lnz_g, (const T*)w.lnz_b, (const T*)w.w_b, p.H, p.L, Lq, Lp, p.eps, bias);
    else
        hipLaunchKernelGGL((k_bias_generic<T>), dim3(blocks), dim3(256), 0, st, (const T*)x, p.sr, p.sl, p.c,
                           (const T*)w.ln_g, (const T*)w.ln_b, (const T*)w.w_b, p.H, p.L, Lq, Lp, p.eps, bias);
    return check_launch("bias (generic)");
}

template <typename T>
static ff_status chunk_t(const Problem& p, const ff_attn_weights& w, const void* x, const float* mask, const void* res,
                         void* out, const Workspace& ws, int r0, int rows, hipStream_t st) {
    const int tokens = rows * p.L;
    hipLaunchKernelGGL((k_stats_generic<T>), dim3((tokens + 3) / 4), dim3(256), 0, st, (const T*)x, p.sr, p.sl, p.c,
                       p.L, r0, tokens, p.eps, ws.stats);
    GenericGemmArgs g{};
    g.a = x; g.sr = p.sr; g.sl = p.sl; g.L = p.L; g.r0 = r0; g.tokens = tokens;
    g.K = p.c; g.N = 4 * p.Hd; g.stats = ws.stats; g.ln_g = w.ln_g; g.ln_b = w.ln_b;
    g.w[0] = w.w_q; g.w[1] = w.w_k; g.w[2] = w.w_v; g.w[3] = w.w_g; g.bvec = w.b_g; g.Hd = p.Hd;
    g.qscale = kLog2e / sqrtf((float)p.d);
    g.cdst = ws.qkvg;
    hipLaunchKernelGGL((k_gemm_generic<T, true>), dim3((tokens + 63) / 64, (g.N + 63) / 64), dim3(256), 0, st, g);

    const int64_t items = (int64_t)rows * p.H * p.L;
    const unsigned ablocks = (unsigned)((items + 3) / 4);
#define FF_ATTN(D)                                                                                              \
    hipLaunchKernelGGL((k_attn_generic<T, D>), dim3(ablocks), dim3(256), 0, st, (const T*)ws.qkvg, ws.bias, mask, \
                       p.sr, p.sl, r0, rows, p.L, p.H, p.d, (T*)ws.o)
    if (p.d <= 8) FF_ATTN(8);
    else if (p.d <= 16) FF_ATTN(16);
    else if (p.d <= 32) FF_ATTN(32);
    else if (p.d <= 64) FF_ATTN(64);
    else FF_ATTN(128);
#undef FF_ATTN

    GenericGemmArgs o{};
    o.a = ws.o; o.sr = p.sr; o.sl = p.sl; o.L = p.L; o.r0 = r0; o.tokens = tokens;
    o.K = p.Hd; o.N = p.c; o.w[0] = w.w_o; o.bvec = w.b_o; o.Hd = p.Hd; o.cdst = out; o.res = res;
    hipLaunchKernelGGL((k_gemm_generic<T, false>), dim3((tokens + 63) / 64, (o.N + 63) / 64), dim3(256), 0, st, o);
    return check_launch("attention chunk (generic)");
}

ff_status generic_prepare(const Problem& p, const ff_attn_weights& w, const void* x, const void* z,
                          const Workspace& ws, hipStream_t stream) {
    if (!p.has_bias) return FF_OK;
    return generic_bias_into(p, w, x, z, ws.bias, p.L, p.L, stream);
}

ff_status generic_bias_into(const Problem& p, const ff_attn_weights& w, const void* x, const void* z, float* bias,
                            int Lq, int Lp, hipStream_t stream) {
    return p.dtype == FF_F32 ? bias_t<float>(p, w, x, z, bias, Lq, Lp, stream)
                             : bias_t<bf16_t>(p, w, x, z, bias, Lq, Lp, stream);
}

ff_status generic_chunk(const Problem& p, const ff_attn_weights& w, const void* x, const float* mask,
                        const void* res, void* out, const Workspace& ws, int r0, int rows, hipStream_t stream) {
    return p.dtype == FF_F32 ? chunk_t<float>(p, w, x, mask, res, out, ws, r0, rows, stream)
                             : chunk_t<bf16_t>(p, w, x, mask, res, out, ws, r0, rows, stream);
}

}  // namespace ff
