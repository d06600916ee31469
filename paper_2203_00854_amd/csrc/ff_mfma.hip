// bfloat16 matrix-core kernel family for gfx950 (wave64, v_mfma_f32_32x32x16_bf16).
//
// Pipeline per chunk of batch rows (FastFold Sections 2.1, 2.3, 5.2):
//   k_pair_bias   LayerNorm + H dot products per pair, float32 bias tensor     (HBM bound)
//   k_gemm<PROJ>  LayerNorm fused as the prologue of the merged q|k|v|gate GEMM
//                 (Section 5.2 "merge GEMM"); epilogue scales q, applies bias+sigmoid
//                 to the gate, writes q,k,gate token-major and v transposed
//   k_attn        flash-style attention: S^T = K Q^T on the matrix cores with the
//                 bias tile as accumulator input, mask, online softmax in registers
//                 (the paper's fused scale+mask+bias softmax, Section 5.2, never
//                 materialising the score tensor of Section 3.2), O^T = V^T P^T,
//                 gate product in the epilogue
//   k_gemm<OUT>   output projection + b_o, scattered to the caller's layout
//
// Matrix-core operand layouts used throughout (wave64, 32x32x16, bf16 in, f32 out):
//   A (32 x 16): lane l holds row l%32, columns 8*(l/32) .. +7
//   B (16 x 32): lane l holds column l%32, rows 8*(l/32) .. +7
//   C/D (32 x 32): lane l holds column l%32, register v holds row 8*(v/4) + 4*(l/32) + v%4
// Computing S^T (keys x queries) instead of S puts one query in one lane, so the softmax
// statistics are lane-local except for one exchange between the two half-waves, and the
// exponentiated tile already has the B-operand layout of the second contraction once the
// key order inside a 32-key tile is permuted; the same permutation is applied when the K
// rows and the V^T columns are fetched, so no data is moved between the two contractions.
//
// Workspace layout of this family (Lp = L rounded up to 32, token p = rl*Lp + l):
//   bias [H][Lq][Lp] float32 (times log2 e), Lq = L rounded up to 64
//   q, k, g, o  [rows*Lp][Hd] bf16;  vt [rows][H][D][Lp] bf16 (pad keys hold zeros)
#include "ff_common.h"

namespace ff {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

union Frag {
    bf16x8 v;
    uint4 u;
    uint32_t w[4];
};

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    bf16x2 t;
    t[0] = (__bf16)a;
    t[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, t);
}
__device__ __forceinline__ float lo_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_f32(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ uint4 ldg16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ uint2 ldg8(const void* p) { return *reinterpret_cast<const uint2*>(p); }

// value of the other half-wave's lane (l ^ 32)
__device__ __forceinline__ float other_half(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    // r[0] = {lower half of v, lower half of v}, r[1] = {upper half, upper half}
    return (threadIdx.x & 32) ? __uint_as_float(r[0]) : __uint_as_float(r[1]);
}
// After the call lanes of the lower half hold (a of lower lane, a of upper lane) and lanes of
// the upper half hold (b of lower lane, b of upper lane): two 4-element groups that are
// adjacent in memory end up in one lane.
__device__ __forceinline__ void merge_halves(uint32_t& a, uint32_t& b) {
    auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    a = r[0];
    b = r[1];
}

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// ------------------------------------------------------------------------------------
struct MfmaWs {
    bf16_t *q, *k, *g, *vt, *o;
};

static MfmaWs split_ws(const Problem& p, int chunk, const Workspace& ws) {
    const size_t Lp = round_up(p.L, 32);
    const size_t n = (size_t)chunk * Lp * p.Hd;   // elements per tensor
    MfmaWs m;
    m.q = (bf16_t*)ws.qkvg;
    m.k = m.q + n;
    m.g = m.k + n;
    m.vt = m.g + n;
    m.o = (bf16_t*)ws.o;
    return m;
}

bool mfma_supported(const Problem& p) {
    if (p.dtype != FF_BF16) return false;
    if (p.c % 32 != 0 || p.c > 256) return false;
    if (p.Hd % 32 != 0 || p.Hd > 256) return false;
    if (p.d % 8 != 0 || p.d > 32) return false;
    if (p.L > 16384) return false;
    if (p.mode == FF_MSA_ROW && (p.c_z % 8 != 0)) return false;
    return true;
}

size_t mfma_workspace(const Problem& p, int chunk, Workspace* ws, void* base) {
    const size_t Lp = round_up(p.L, 32), Lq = round_up(p.L, 64);
    size_t off = 0;
    char* b = (char*)base;
    ws->bias = nullptr;
    if (p.has_bias) {
        ws->bias = (float*)(b + off);
        off += align256((size_t)p.H * Lq * Lp * 4);
    }
    const size_t n = (size_t)chunk * Lp * p.Hd * 2;
    ws->stats = nullptr;
    ws->qkvg = b + off;
    off += align256(4 * n);
    ws->o = b + off;
    off += align256(n);
    ws->total = off;
    ws->chunk = chunk;
    return off;
}

// ====================================================================================
// Pair bias.  A group of G lanes owns one pair (q, k): 16 bytes per lane, LayerNorm
// statistics and the H dot products by xor-shuffles inside the group.
//   bias[h][q][k] = log2(e) * sum_c LN(src[q,k,:])_c * w_b[h][c]
template <int HMAX>
__global__ __launch_bounds__(256) void k_pair_bias(const bf16_t* __restrict__ src, int64_t sq, int64_t sk, int c,
                                                    const bf16_t* __restrict__ gam, const bf16_t* __restrict__ bet,
                                                    const bf16_t* __restrict__ wb, int H, int L, int Lq, int Lp,
                                                    int G, float eps, float* __restrict__ bias) {
    const int lig = threadIdx.x & (G - 1);
    const int chunks = c >> 3;
    const bool has = lig < chunks;
    float wg[HMAX][8];      // w_b * gamma for this lane's 8 channels
    float cst[HMAX];        // sum_c beta_c * w_b[h][c]
#pragma unroll
    for (int h = 0; h < HMAX; ++h) {
        cst[h] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) wg[h][j] = 0.f;
    }
    if (has) {
        const uint4 gr = ldg16(gam + lig * 8), br = ldg16(bet + lig * 8);
        const uint32_t gw[4] = {gr.x, gr.y, gr.z, gr.w}, bw[4] = {br.x, br.y, br.z, br.w};
#pragma unroll
        for (int h = 0; h < HMAX; ++h) {
            if (h < H) {
                const uint4 wr = ldg16(wb + (size_t)h * c + lig * 8);
                const uint32_t ww[4] = {wr.x, wr.y, wr.z, wr.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    wg[h][2 * i] = lo_f32(ww[i]) * lo_f32(gw[i]);
                    wg[h][2 * i + 1] = hi_f32(ww[i]) * hi_f32(gw[i]);
                    cst[h] += lo_f32(ww[i]) * lo_f32(bw[i]) + hi_f32(ww[i]) * hi_f32(bw[i]);
                }
            }
        }
    }
#pragma unroll
    for (int h = 0; h < HMAX; ++h)
        for (int o = G >> 1; o > 0; o >>= 1) cst[h] += __shfl_xor(cst[h], o, 64);

    const int groups = 256 / G;
    const int64_t pairs = (int64_t)L * L;
    const float inv_c = 1.f / (float)c;
    for (int64_t pr = (int64_t)blockIdx.x * groups + threadIdx.x / G; pr < pairs; pr += (int64_t)gridDim.x * groups) {
        const int q = (int)(pr / L), k = (int)(pr - (int64_t)q * L);
        float v[8];
        float s = 0.f;
        if (has) {
            const uint4 r = ldg16(src + ((int64_t)q * sq + (int64_t)k * sk) * c + lig * 8);
            const uint32_t rw[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[2 * i] = lo_f32(rw[i]);
                v[2 * i + 1] = hi_f32(rw[i]);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) s += v[j];
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = 0.f;
        }
        for (int o = G >> 1; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        const float mean = s * inv_c;
        float qq = 0.f;
        if (has) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                v[j] -= mean;
                qq += v[j] * v[j];
            }
        }
        for (int o = G >> 1; o > 0; o >>= 1) qq += __shfl_xor(qq, o, 64);
        const float rstd = rsqrtf(qq * inv_c + eps);
        float mine = 0.f;
#pragma unroll
        for (int h = 0; h < HMAX; ++h) {
            if (h < H) {
                float a = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) a += v[j] * wg[h][j];
                for (int o = G >> 1; o > 0; o >>= 1) a += __shfl_xor(a, o, 64);
                if (lig == (h & (G - 1))) mine = (a * rstd + cst[h]) * kLog2e;
                if (G < HMAX && lig == (h & (G - 1)))   // fewer lanes than heads: write at once
                    bias[((size_t)h * Lq + q) * Lp + k] = mine;
            }
        }
        if (G >= HMAX && lig < H) bias[((size_t)lig * Lq + q) * Lp + k] = mine;
    }
}

// ====================================================================================
// GEMM with the whole contraction length (<= 256) resident: a wavefront owns 64 tokens
// (two 32-token tiles) as register-resident operand fragments and sweeps over 32-feature
// tiles of the weight matrix, which the block streams through LDS (double buffered).
struct GemmArgs {
    const bf16_t* src;     // PROJ: x (strided tokens); OUT: o [rows*Lp][K]
    int64_t sr, sl;        // token strides of x / out
    int r0, rows, L, Lp;
    int K;                 // contraction length (c for PROJ, Hd for OUT)
    const bf16_t *ln_g, *ln_b;
    float eps;
    const bf16_t* w[4];    // PROJ: w_q, w_k, w_v, w_g, each [Hd][K]; OUT: w[0] = w_o [N][K]
    const bf16_t* bvec;    // PROJ: b_g [Hd]; OUT: b_o [N]
    int Hd, H, D;
    float qscale;
    bf16_t *q, *k, *g, *vt;  // PROJ outputs
    bf16_t* out;             // OUT output [n_a][n_b][N], token (r,l) at (r*sr + l*sl)*N
    int N;                   // features in total (4*Hd or c)
    int tiles_per_split;     // 32-feature tiles per blockIdx.y
};

template <int KC, bool PROJ, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_gemm(GemmArgs a) {
    constexpr int NT = WAVES * 64;
    constexpr int PITCH = KC * 32 + 16;                 // bytes per weight row in LDS (padded)
    __shared__ __attribute__((aligned(16))) unsigned char s_w[2][32 * PITCH];
    __shared__ float s_g[PROJ ? KC * 16 : 1], s_b[PROJ ? KC * 16 : 1];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int K = a.K;
    const int tiles_m = a.rows * (a.Lp >> 5);

    if constexpr (PROJ) {
        for (int i = tid; i < KC * 16; i += NT) {
            s_g[i] = i < K ? bf16_to_f32(a.ln_g[i]) : 0.f;
            s_b[i] = i < K ? bf16_to_f32(a.ln_b[i]) : 0.f;
        }
    }

    // ---- weight tile loader: 32 rows x 2*KC 16-byte pieces, consecutive threads along a row
    constexpr int PIECES = 32 * 2 * KC;
    constexpr int PER_THREAD = (PIECES + NT - 1) / NT;
    const int ft_begin = blockIdx.y * a.tiles_per_split;
    int ft_end = ft_begin + a.tiles_per_split;
    if (ft_end > a.N / 32) ft_end = a.N / 32;
    uint4 wreg[PER_THREAD];
    auto load_w = [&](int ft) {
        // first row of this 32-feature tile (a tile never straddles two weight matrices: Hd % 32 == 0)
        const int sg = PROJ ? (ft * 32) / a.Hd : 0;
        const bf16_t* wt = a.w[sg] + (size_t)(ft * 32 - sg * a.Hd) * K;
#pragma unroll
        for (int j = 0; j < PER_THREAD; ++j) {
            const int i = tid + j * NT;
            const int f = i / (2 * KC), pc = i % (2 * KC);
            uint4 val = make_uint4(0, 0, 0, 0);
            if (i < PIECES && pc * 8 < K) val = ldg16(wt + (size_t)f * K + pc * 8);
            wreg[j] = val;
        }
    };
    auto store_w = [&](int buf) {
#pragma unroll
        for (int j = 0; j < PER_THREAD; ++j) {
            const int i = tid + j * NT;
            const int f = i / (2 * KC), pc = i % (2 * KC);
            if (i < PIECES) *reinterpret_cast<uint4*>(&s_w[buf][f * PITCH + pc * 16]) = wreg[j];
        }
    };
    if (ft_begin < ft_end) load_w(ft_begin);
    __syncthreads();   // s_g / s_b visible

    // ---- token operand fragments (with LayerNorm for PROJ)
    Frag xa[2][KC];
    bool tile_ok[2];
    int tok[2];        // padded token index of this lane
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        const int tg = (blockIdx.x * WAVES + wave) * 2 + tt;
        tile_ok[tt] = tg < tiles_m;
        const int p = tg * 32 + col;
        tok[tt] = p;
        const int rl = p / a.Lp, l = p - rl * a.Lp;
        const bool valid = tile_ok[tt] && l < a.L;
        const bf16_t* sp = PROJ ? a.src + ((int64_t)(a.r0 + rl) * a.sr + (int64_t)l * a.sl) * K
                                : a.src + (size_t)p * K;
#pragma unroll
        for (int s = 0; s < KC; ++s) {
            xa[tt][s].u = make_uint4(0, 0, 0, 0);
            if (valid && (16 * s + 8 * hf) < K) xa[tt][s].u = ldg16(sp + 16 * s + 8 * hf);
        }
        if constexpr (PROJ) {
            float sum = 0.f;
#pragma unroll
            for (int s = 0; s < KC; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i) sum += lo_f32(xa[tt][s].w[i]) + hi_f32(xa[tt][s].w[i]);
            sum += other_half(sum);
            const float mean = sum / (float)K;
            float sq = 0.f;
#pragma unroll
            for (int s = 0; s < KC; ++s) {
                if (16 * s + 8 * hf < K) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float d0 = lo_f32(xa[tt][s].w[i]) - mean, d1 = hi_f32(xa[tt][s].w[i]) - mean;
                        sq += d0 * d0 + d1 * d1;
                    }
                }
            }
            sq += other_half(sq);
            const float rstd = rsqrtf(sq / (float)K + a.eps);
#pragma unroll
            for (int s = 0; s < KC; ++s) {
                const int c0 = 16 * s + 8 * hf;
                if (valid && c0 < K) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float y0 = (lo_f32(xa[tt][s].w[i]) - mean) * rstd * s_g[c0 + 2 * i] + s_b[c0 + 2 * i];
                        const float y1 =
                            (hi_f32(xa[tt][s].w[i]) - mean) * rstd * s_g[c0 + 2 * i + 1] + s_b[c0 + 2 * i + 1];
                        xa[tt][s].w[i] = pack2(y0, y1);
                    }
                } else {
                    xa[tt][s].u = make_uint4(0, 0, 0, 0);
                }
            }
        }
    }

    if (ft_begin < ft_end) store_w(0);
    __syncthreads();

    for (int ft = ft_begin; ft < ft_end; ++ft) {
        const int buf = (ft - ft_begin) & 1;
        if (ft + 1 < ft_end) load_w(ft + 1);
        const int seg = PROJ ? (ft * 32) / a.Hd : 0;           // 0 q, 1 k, 2 v, 3 gate
        const bool tokens_by_features = PROJ && seg == 2;      // V: rows = tokens
        f32x16 acc[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tt][v] = 0.f;
        if (tokens_by_features) {
#pragma unroll
            for (int s = 0; s < KC; ++s) {
                Frag wf;
                wf.u = *reinterpret_cast<const uint4*>(&s_w[buf][col * PITCH + (2 * s + hf) * 16]);
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
                    acc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[tt][s].v, wf.v, acc[tt], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int s = 0; s < KC; ++s) {
                Frag wf;
                wf.u = *reinterpret_cast<const uint4*>(&s_w[buf][col * PITCH + (2 * s + hf) * 16]);
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
                    acc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, xa[tt][s].v, acc[tt], 0, 0, 0);
            }
        }

        // ---- epilogue
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            if (!tile_ok[tt]) continue;
            if (tokens_by_features) {
                // lane = feature (col), registers = tokens 8g + 4hf + e of the tile
                const int n = ft * 32 + col - 2 * a.Hd;
                const int h = n / a.D, e = n - h * a.D;
                const int p0 = tok[tt] - col;                      // first token of the tile
                const int rl = p0 / a.Lp, l0 = p0 - rl * a.Lp;
                uint32_t pk[8];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    pk[2 * g] = pack2(acc[tt][4 * g], acc[tt][4 * g + 1]);
                    pk[2 * g + 1] = pack2(acc[tt][4 * g + 2], acc[tt][4 * g + 3]);
                }
                merge_halves(pk[0], pk[2]);
                merge_halves(pk[1], pk[3]);
                merge_halves(pk[4], pk[6]);
                merge_halves(pk[5], pk[7]);
                // lower half: tokens 0..7 (pk0,pk1,pk2,pk3 -> a0 a1 | b0 b1) ; see merge_halves
                bf16_t* dst = a.vt + ((size_t)(rl * a.H + h) * a.D + e) * a.Lp + l0 + 8 * hf;
                *reinterpret_cast<uint4*>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                *reinterpret_cast<uint4*>(dst + 16) = make_uint4(pk[4], pk[5], pk[6], pk[7]);
            } else {
                // lane = token (col), registers = features 8g + 4hf + e of the tile
                const int p = tok[tt];
                const int rl = p / a.Lp, l = p - rl * a.Lp;
                const int nb = ft * 32;                            // first feature of the tile
                float bv[16];
                if (!PROJ || seg == 3) {
                    const bf16_t* bp = a.bvec + (PROJ ? nb - 3 * a.Hd : nb);
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const uint2 r = ldg8(bp + 8 * g + 4 * hf);
                        bv[4 * g] = lo_f32(r.x); bv[4 * g + 1] = hi_f32(r.x);
                        bv[4 * g + 2] = lo_f32(r.y); bv[4 * g + 3] = hi_f32(r.y);
                    }
                }
                float val[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float t = acc[tt][v];
                    if (PROJ) {
                        if (seg == 0) t *= a.qscale;
                        if (seg == 3) t = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-(t + bv[v]) * kLog2e));
                    } else {
                        t += bv[v];
                    }
                    val[v] = t;
                }
                uint32_t pk[8];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    pk[2 * g] = pack2(val[4 * g], val[4 * g + 1]);
                    pk[2 * g + 1] = pack2(val[4 * g + 2], val[4 * g + 3]);
                }
                merge_halves(pk[0], pk[2]);
                merge_halves(pk[1], pk[3]);
                merge_halves(pk[4], pk[6]);
                merge_halves(pk[5], pk[7]);
                if (l < a.L) {
                    bf16_t* dst;
                    if (PROJ) {
                        bf16_t* base = seg == 0 ? a.q : (seg == 1 ? a.k : a.g);
                        dst = base + (size_t)p * a.Hd + (nb - seg * a.Hd);
                    } else {
                        dst = a.out + ((int64_t)(a.r0 + rl) * a.sr + (int64_t)l * a.sl) * a.N + nb;
                    }
                    *reinterpret_cast<uint4*>(dst + 8 * hf) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                    *reinterpret_cast<uint4*>(dst + 16 + 8 * hf) = make_uint4(pk[4], pk[5], pk[6], pk[7]);
                }
            }
        }
        if (ft + 1 < ft_end) store_w(buf ^ 1);
        __syncthreads();
    }
}

// ====================================================================================
// Attention.  Block = 4 wavefronts = 4 batch rows, same head, same 64 queries: the bias
// tile [64 queries x 32 keys] is staged once per block in LDS and used by all four rows;
// K rows and V^T columns go straight from global memory into operand registers.
struct AttnArgs {
    const bf16_t *q, *k, *g, *vt;
    bf16_t* o;
    const float* bias;     // [H][Lq][Lp] or NULL
    const float* mask;     // caller's mask or NULL
    int64_t sr, sl;
    int r0, rows, L, Lp, Lq, H, Hd;
};

constexpr int kBiasPitch = 36;   // floats per LDS bias row (32 + 4 pad)

template <int D, bool HAS_BIAS>
__global__ __launch_bounds__(256) void k_attn(AttnArgs a) {
    constexpr int KS = (D + 15) / 16;   // 16-wide steps of the q.k contraction
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* s_bias = reinterpret_cast<float*>(smem);                                  // [2][64][kBiasPitch]
    uint32_t* s_mask = reinterpret_cast<uint32_t*>(smem + (HAS_BIAS ? 2 * 64 * kBiasPitch * 4 : 0));  // [4][Lp/32]

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int nt = a.Lp >> 5;
    const int rl_raw = blockIdx.z * 4 + wave;
    const bool row_ok = rl_raw < a.rows;
    const int rl = row_ok ? rl_raw : a.rows - 1;
    const int h = blockIdx.y;
    const int q0 = blockIdx.x * 64;

    // ---- key-validity bits of this wave's batch row, one word per 32-key tile
    {
        const float* mrow = a.mask ? a.mask + (int64_t)(a.r0 + rl) * a.sr : nullptr;
        for (int t = 0; t < nt; t += 2) {
            const int key = 32 * t + lane;
            bool valid = key < a.L;
            if (valid && mrow) valid = mrow[(int64_t)key * a.sl] != 0.f;
            const unsigned long long b = __ballot(valid);
            if (lane == 0) {
                s_mask[wave * nt + t] = (uint32_t)b;
                if (t + 1 < nt) s_mask[wave * nt + t + 1] = (uint32_t)(b >> 32);
            }
        }
    }

    // ---- Q operand fragments: B operand, lane = query, 8 consecutive e
    Frag qf[2][KS];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        int qi = q0 + 32 * j + col;
        if (qi > a.Lp - 1) qi = a.Lp - 1;
        const bf16_t* qp = a.q + ((size_t)rl * a.Lp + qi) * a.Hd + h * D;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            qf[j][s].u = make_uint4(0, 0, 0, 0);
            if (16 * s + 8 * hf < D) qf[j][s].u = ldg16(qp + 16 * s + 8 * hf);
        }
    }

    // ---- bias tile pipeline
    const int b_row = tid >> 3, b_c4 = tid & 7;     // thread loads rows b_row, b_row+32; floats 4*b_c4..+3
    const float* bias_h = HAS_BIAS ? a.bias + ((size_t)h * a.Lq + q0) * a.Lp : nullptr;
    float4 breg[2];
    auto load_bias = [&](int kt) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            breg[i] = *reinterpret_cast<const float4*>(bias_h + (size_t)(b_row + 32 * i) * a.Lp + 32 * kt + 4 * b_c4);
    };
    auto store_bias = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            *reinterpret_cast<float4*>(s_bias + ((size_t)buf * 64 + b_row + 32 * i) * kBiasPitch + 4 * b_c4) = breg[i];
    };
    if constexpr (HAS_BIAS) {
        load_bias(0);
        store_bias(0);
    }
    __syncthreads();

    // permuted key of S^T row m = col: rows 8g + 4b + e hold key 16*(g/2) + 8b + 4*(g%2) + e
    const int kperm = 16 * (col >> 4) + 8 * ((col >> 2) & 1) + 4 * ((col >> 3) & 1) + (col & 3);
    const bf16_t* kbase = a.k + (size_t)rl * a.Lp * a.Hd + h * D;
    const bf16_t* vbase = a.vt + ((size_t)(rl * a.H + h) * D + (col < D ? col : 0)) * a.Lp;

    f32x16 o_acc[2];
    float m_run[2], l_run[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        m_run[j] = -INFINITY;
        l_run[j] = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[j][v] = 0.f;
    }

    for (int kt = 0; kt < nt; ++kt) {
        const int buf = kt & 1;
        if constexpr (HAS_BIAS)
            if (kt + 1 < nt) load_bias(kt + 1);
        const uint32_t bits = __builtin_amdgcn_readfirstlane(s_mask[wave * nt + kt]);
        if (bits != 0u) {
            // K fragments: A operand, lane = (permuted) key, 8 consecutive e
            Frag kf[KS];
            const bf16_t* kp = kbase + (size_t)(32 * kt + kperm) * a.Hd;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                kf[s].u = make_uint4(0, 0, 0, 0);
                if (16 * s + 8 * hf < D) kf[s].u = ldg16(kp + 16 * s + 8 * hf);
            }
            // V^T fragments: A operand, lane = e, 8 consecutive (permuted = natural) keys
            Frag vf[2];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                vf[c].u = make_uint4(0, 0, 0, 0);
                if (col < D) vf[c].u = ldg16(vbase + 32 * kt + 16 * c + 8 * hf);
            }
            f32x16 s_acc[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if constexpr (HAS_BIAS) {
                    const float* br = s_bias + ((size_t)buf * 64 + 32 * j + col) * kBiasPitch + 8 * hf;
#pragma unroll
                    for (int c = 0; c < 2; ++c)
#pragma unroll
                        for (int i = 0; i < 2; ++i) {
                            const float4 t = *reinterpret_cast<const float4*>(br + 16 * c + 4 * i);
                            s_acc[j][8 * c + 4 * i] = t.x; s_acc[j][8 * c + 4 * i + 1] = t.y;
                            s_acc[j][8 * c + 4 * i + 2] = t.z; s_acc[j][8 * c + 4 * i + 3] = t.w;
                        }
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) s_acc[j][v] = 0.f;
                }
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    s_acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s].v, qf[j][s].v, s_acc[j], 0, 0, 0);
            }
            if (bits != 0xffffffffu) {
                // register v of this lane holds key 16*(v/8) + 8*hf + v%8 of the tile
                const uint32_t mine = bits >> (8 * hf);
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (!((mine >> (16 * (v >> 3) + (v & 7))) & 1u)) s_acc[j][v] = -INFINITY;
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                float tmax = s_acc[j][0];
#pragma unroll
                for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, s_acc[j][v]);
                tmax = fmaxf(tmax, other_half(tmax));
                const float m_new = fmaxf(m_run[j], tmax);
                const float m_use = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f(m_run[j] - m_use);
                m_run[j] = m_new;
                float psum = 0.f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float pv = __builtin_amdgcn_exp2f(s_acc[j][v] - m_use);
                    s_acc[j][v] = pv;
                    psum += pv;
                }
                l_run[j] = l_run[j] * alpha + psum;
                if (__any(alpha != 1.f)) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) o_acc[j][v] *= alpha;
                }
                Frag pf[2];
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int i = 0; i < 4; ++i) pf[c].w[i] = pack2(s_acc[j][8 * c + 2 * i], s_acc[j][8 * c + 2 * i + 1]);
#pragma unroll
                for (int c = 0; c < 2; ++c)
                    o_acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[c].v, pf[c].v, o_acc[j], 0, 0, 0);
            }
        }
        if constexpr (HAS_BIAS) {
            if (kt + 1 < nt) store_bias(buf ^ 1);
            __syncthreads();
        }
    }

    // ---- epilogue: normalise, gate, store.  o_acc[j]: lane = query, register v = e = 8*(v/4) + 4*hf + v%4
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const float l_tot = l_run[j] + other_half(l_run[j]);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        const int qi = q0 + 32 * j + col;
        if (row_ok && qi < a.L) {
            const size_t t = ((size_t)rl * a.Lp + qi) * a.Hd + h * D;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int e0 = 8 * g + 4 * hf;
                if (e0 < D) {
                    const uint2 gr = ldg8(a.g + t + e0);
                    uint2 ov;
                    ov.x = pack2(o_acc[j][4 * g] * inv * lo_f32(gr.x), o_acc[j][4 * g + 1] * inv * hi_f32(gr.x));
                    ov.y = pack2(o_acc[j][4 * g + 2] * inv * lo_f32(gr.y), o_acc[j][4 * g + 3] * inv * hi_f32(gr.y));
                    *reinterpret_cast<uint2*>(a.o + t + e0) = ov;
                }
            }
        }
    }
}

// ====================================================================================
// host side
ff_status mfma_bias(const Problem& p, const ff_attn_weights& w, const void* x, const void* z, const Workspace& ws,
                    hipStream_t st) {
    const int Lp = round_up(p.L, 32), Lq = round_up(p.L, 64);
    const bool row = p.mode == FF_MSA_ROW;
    const int c = row ? p.c_z : p.c;
    if (p.H > 8 || c > 512 || c % 8 != 0) return generic_bias_into(p, w, x, z, ws.bias, Lq, Lp, st);
    int G = 4;
    while (G * 8 < c) G <<= 1;
    const int groups = 256 / G;
    const int64_t pairs = (int64_t)p.L * p.L;
    int64_t blocks = (pairs + groups - 1) / groups;
    if (blocks > 256 * 32) blocks = 256 * 32;
    const bf16_t* src = (const bf16_t*)(row ? z : x);
    const int64_t sq = row ? p.L : p.sr, sk = row ? 1 : p.sl;
    const bf16_t* g = (const bf16_t*)(row ? w.lnz_g : w.ln_g);
    const bf16_t* b = (const bf16_t*)(row ? w.lnz_b : w.ln_b);
    if (p.H <= 4)
        hipLaunchKernelGGL((k_pair_bias<4>), dim3((unsigned)blocks), dim3(256), 0, st, src, sq, sk, c, g, b,
                           (const bf16_t*)w.w_b, p.H, p.L, Lq, Lp, G, p.eps, ws.bias);
    else
        hipLaunchKernelGGL((k_pair_bias<8>), dim3((unsigned)blocks), dim3(256), 0, st, src, sq, sk, c, g, b,
                           (const bf16_t*)w.w_b, p.H, p.L, Lq, Lp, G, p.eps, ws.bias);
    return check_launch("pair bias");
}

template <bool PROJ>
static void launch_gemm(const GemmArgs& a, int K, dim3 grid, hipStream_t st) {
    const int kc = K / 16;
    if (kc <= 2) hipLaunchKernelGGL((k_gemm<2, PROJ, 4>), grid, dim3(256), 0, st, a);
    else if (kc <= 4) hipLaunchKernelGGL((k_gemm<4, PROJ, 4>), grid, dim3(256), 0, st, a);
    else if (kc <= 8) hipLaunchKernelGGL((k_gemm<8, PROJ, 4>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((k_gemm<16, PROJ, 4>), grid, dim3(256), 0, st, a);
}

static int pick_split(int blocks_m, int tiles_n) {
    // enough blocks to fill 256 CUs twice, without recomputing the LayerNorm prologue too often
    int split = 1;
    while (blocks_m * split < 512 && split * 2 <= tiles_n && tiles_n % (split * 2) == 0 && split < 4) split *= 2;
    return split;
}

ff_status mfma_chunk(const Problem& p, const ff_attn_weights& w, const void* x, const float* mask, void* out,
                     const Workspace& ws, int r0, int rows, hipStream_t st) {
    const int Lp = round_up(p.L, 32), Lq = round_up(p.L, 64);
    MfmaWs m = split_ws(p, ws.chunk, ws);

    const int tiles_m = rows * (Lp / 32);
    const int blocks_m = (tiles_m + 7) / 8;           // 4 waves x 2 token tiles
    GemmArgs g{};
    g.src = (const bf16_t*)x; g.sr = p.sr; g.sl = p.sl; g.r0 = r0; g.rows = rows; g.L = p.L; g.Lp = Lp;
    g.K = p.c; g.ln_g = (const bf16_t*)w.ln_g; g.ln_b = (const bf16_t*)w.ln_b; g.eps = p.eps;
    g.w[0] = (const bf16_t*)w.w_q; g.w[1] = (const bf16_t*)w.w_k; g.w[2] = (const bf16_t*)w.w_v;
    g.w[3] = (const bf16_t*)w.w_g; g.bvec = (const bf16_t*)w.b_g;
    g.Hd = p.Hd; g.H = p.H; g.D = p.d; g.qscale = kLog2e / sqrtf((float)p.d);
    g.q = m.q; g.k = m.k; g.g = m.g; g.vt = m.vt; g.N = 4 * p.Hd;
    {
        const int tiles_n = g.N / 32;
        const int split = pick_split(blocks_m, tiles_n);
        g.tiles_per_split = tiles_n / split;
        launch_gemm<true>(g, p.c, dim3(blocks_m, split), st);
    }

    AttnArgs a{};
    a.q = m.q; a.k = m.k; a.g = m.g; a.vt = m.vt; a.o = m.o; a.bias = ws.bias; a.mask = mask;
    a.sr = p.sr; a.sl = p.sl; a.r0 = r0; a.rows = rows; a.L = p.L; a.Lp = Lp; a.Lq = Lq; a.H = p.H; a.Hd = p.Hd;
    {
        dim3 grid(Lq / 64, p.H, (rows + 3) / 4);
        const size_t mask_bytes = (size_t)4 * (Lp / 32) * 4;
        const size_t bias_bytes = (size_t)2 * 64 * kBiasPitch * 4;
#define FF_ATTN(DD)                                                                                          \
    do {                                                                                                     \
        if (p.has_bias) hipLaunchKernelGGL((k_attn<DD, true>), grid, dim3(256), bias_bytes + mask_bytes, st, a); \
        else hipLaunchKernelGGL((k_attn<DD, false>), grid, dim3(256), mask_bytes, st, a);                   \
    } while (0)
        if (p.d == 8) FF_ATTN(8);
        else if (p.d == 16) FF_ATTN(16);
        else if (p.d == 24) FF_ATTN(24);
        else FF_ATTN(32);
#undef FF_ATTN
    }

    GemmArgs o{};
    o.src = m.o; o.sr = p.sr; o.sl = p.sl; o.r0 = r0; o.rows = rows; o.L = p.L; o.Lp = Lp;
    o.K = p.Hd; o.w[0] = (const bf16_t*)w.w_o; o.bvec = (const bf16_t*)w.b_o;
    o.Hd = p.Hd; o.H = p.H; o.D = p.d; o.out = (bf16_t*)out; o.N = p.c;
    {
        const int tiles_n = o.N / 32;
        const int split = pick_split(blocks_m, tiles_n);
        o.tiles_per_split = tiles_n / split;
        launch_gemm<false>(o, p.Hd, dim3(blocks_m, split), st);
    }
    return check_launch("attention chunk (mfma)");
}

}  // namespace ff
