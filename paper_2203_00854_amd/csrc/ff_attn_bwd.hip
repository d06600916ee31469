// Backward pass of the fused attention core (FastFold Section 6.3 benchmarks the fused softmax forward and
// backward; Table 6 reports forward and backward per Evoformer layer), bf16 operands, float32 statistics and
// accumulators, gfx950 matrix cores.  Per batch row r and head h, with scale = 1 / sqrt(d):
//   S[i,j] = scale q[i].k[j] + bias[h,i,j] + M(mask[r,j]);  P = softmax_j S;  ctx[i] = sum_j P[i,j] v[j];  o = g * ctx
//   dg = do * ctx;  dctx = do * g;  dv[j] = sum_i P[i,j] dctx[i];  dP[i,j] = dctx[i].v[j];
//   dS[i,j] = P[i,j] (dP[i,j] - delta[i]),  delta[i] = dctx[i].ctx[i];
//   dq[i] = scale sum_j dS[i,j] k[j];  dk[j] = scale sum_i dS[i,j] q[i];  dbias[h,i,j] = sum_r dS[r,h,i,j]
//
// The score matrix is never stored (Section 3.2): as in the forward pass it is recomputed tile by tile.
// One wavefront per 32-query (or 32-key) tile:
//   k_bwd_transpose  position-contiguous copies [d][L] of q, k and v for the operands whose contraction runs over
//                positions (k_bwd_stats adds the one of dctx)
//   k_bwd_stats  forward recomputation with an online softmax: the logsumexp of every query (base 2), ctx,
//                dg, dctx and delta
//   k_bwd_dq     per query tile, over the key tiles: S^T = K Q^T and dP^T = V dctx^T (lane = query, so that
//                logsumexp and delta are lane-local), dS^T, dq^T += K^T dS^T
//   k_bwd_dkv    per key tile, over the query tiles: S = Q K^T and dP = dctx V^T (lane = key), P and dS,
//                dv^T += dctx^T P, dk^T += Q^T dS
//   k_bwd_dbias  per (head, query tile, key tile, chunk of batch rows): dS summed in registers over the rows of the
//                chunk, the chunks' partial sums added in a fixed order by a small second kernel (deterministic,
//                no atomics)
// Operands whose contraction runs over the head dim are 16-byte row loads; operands whose contraction runs
// over keys or queries ("transposed" fragments: lane = channel) are two 8-byte loads from the position-contiguous
// copies, taken in exactly the order in which the accumulator of the previous contraction leaves its values, so
// nothing moves between two contractions.
// Operand layouts of v_mfma_f32_32x32x16_bf16: A (32 x 16): lane l holds row l%32, columns 8*(l/32)..+7;
// B (16 x 32): lane l holds column l%32, rows 8*(l/32)..+7; D (32 x 32): lane l holds column l%32, register
// v holds row 8*(v/4) + 4*(l/32) + v%4.
#include "ff_common.h"

namespace ff {
namespace bwd {

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
__device__ __forceinline__ float other_half(float v) { return __shfl_xor(v, 32, 64); }

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

struct Args {
    const bf16_t *q, *k, *v, *g, *dout;      // [R][H][L][D]
    const float* bias;                       // [H][L][L] or NULL
    const float* mask;                       // [R][L] or NULL
    bf16_t *dq, *dk, *dv, *dg;               // [R][H][L][D]
    float* dbias;                            // [H][L][L] or NULL
    float* dbias_part;                       // workspace [row_chunks][H][L][L] (partial sums over the rows of a chunk)
    int row_chunks, rows_per_chunk;
    bf16_t* dctx;                            // workspace [R][H][L][D]
    bf16_t *qT, *kT, *vT, *dctxT;            // workspace [R][H][D][Lp]: position-contiguous copies for the transposed operands
    float *lse, *delta;                      // workspace [R*H][Lp]
    int R, H, L, Lp;
    float qscale2;                           // log2(e) / sqrt(D)
    float scale;                             // 1 / sqrt(D)
};

// Row fragments of the 32 positions n0 .. n0+31 of x [L][D] (x already offset to its (row, head)): lane (n, hf)
// holds channels 16 s + 8 hf .. + 7 of position n0 + col; zeros beyond L or D.
template <int D>
__device__ __forceinline__ void load_rows(Frag (&f)[(D + 15) / 16], const bf16_t* x, int n0, int L, int col, int hf) {
    constexpr int KS = (D + 15) / 16;
    const int n = n0 + col;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        f[s].u = make_uint4(0, 0, 0, 0);
        if (n < L && 16 * s + 8 * hf < D) f[s].u = *reinterpret_cast<const uint4*>(x + (size_t)n * D + 16 * s + 8 * hf);
    }
}

// Transposed fragments of the same 32 positions: lane (e, hf) holds x[n][e] for the eight positions that slot
// u = 0..7 of half hf of contraction step s meets, n0 + 16 s + 4 hf + (u < 4 ? u : u + 4): the order in which a
// 32 x 32 accumulator (register 8s + u of half hf) leaves its rows.  xT is the position-contiguous copy
// [D][Lp] of the (row, head) (zeros beyond L), so these are two 8-byte loads per step; zeros for e >= D.
template <int D>
__device__ __forceinline__ void load_cols(Frag (&f)[2], const bf16_t* xT, int n0, int Lp, int col, int hf) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        f[s].u = make_uint4(0, 0, 0, 0);
        if (col < D) {
            const bf16_t* p = xT + (size_t)col * Lp + n0 + 16 * s + 4 * hf;
            const uint2 lo = *reinterpret_cast<const uint2*>(p), hi = *reinterpret_cast<const uint2*>(p + 8);
            f[s].u = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
    }
}

// xT[(row, head)][e][n] = x[(row, head)][n][e] for q, k and v (blockIdx.y picks the tensor), zeros for n in [L, Lp).
// One wavefront per 32 positions: 16-byte row loads, 2-byte stores that are contiguous across the lanes.
template <int D>
__global__ __launch_bounds__(256) void k_bwd_transpose(Args a) {
    const int lane = threadIdx.x & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nt = a.Lp >> 5;
    const int task = blockIdx.x * 4 + wave;
    if (task >= a.R * a.H * nt) return;
    const int rh = task / nt, n0 = (task - rh * nt) * 32, n = n0 + col;
    const bf16_t* src = blockIdx.y == 0 ? a.q : (blockIdx.y == 1 ? a.k : a.v);
    bf16_t* dst = blockIdx.y == 0 ? a.qT : (blockIdx.y == 1 ? a.kT : a.vT);
    // lane (n, hf) takes channels 8 hf + 16 s .. + 7 of position n
#pragma unroll
    for (int s = 0; s < (D + 15) / 16; ++s) {
        const int e0 = 16 * s + 8 * hf;
        if (e0 < D) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (n < a.L) v = *reinterpret_cast<const uint4*>(src + ((size_t)rh * a.L + n) * D + e0);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                dst[((size_t)rh * D + e0 + 2 * i) * a.Lp + n] = (bf16_t)(w[i] & 0xffffu);
                dst[((size_t)rh * D + e0 + 2 * i + 1) * a.Lp + n] = (bf16_t)(w[i] >> 16);
            }
        }
    }
}

// registers 8s .. 8s+7 of an accumulator, rounded to bf16: the B operand of contraction step s over its rows
__device__ __forceinline__ void pack_rows(Frag (&f)[2], const f32x16& a) {
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) f[s].w[i] = pack2(a[8 * s + 2 * i], a[8 * s + 2 * i + 1]);
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 a;
#pragma unroll
    for (int v = 0; v < 16; ++v) a[v] = 0.f;
    return a;
}

constexpr int kTilePitch = 36;       // floats per row of a staged 32 x 32 bias tile (16-byte aligned rows, conflict-free reads)

// The bias tile [i0 .. i0+31][j0 .. j0+31] of head h, times log2(e), in the accumulator layout with lane = query:
// register v = key j0 + 8(v/4) + 4hf + v%4 of query i0 + col.  Read from memory in whole rows (a load instruction
// covers eight 128-byte rows) into the wavefront's own LDS tile and picked up from there; zeros without a bias
// or outside the matrix.
__device__ __forceinline__ void bias_tile_by_query(f32x16& b, const Args& a, int h, int i0, int j0, float* tile, int lane, int col, int hf) {
    if (!a.bias) {
        b = zero16();
        return;
    }
    const bool vec = (a.L & 3) == 0;
    const int c4 = (lane & 7) * 4;
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int row = 8 * n + (lane >> 3), i = i0 + row, j = j0 + c4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < a.L) {
            const float* p = a.bias + ((size_t)h * a.L + i) * a.L + j;
            if (vec && j + 3 < a.L) v = *reinterpret_cast<const float4*>(p);
            else {
                if (j < a.L) v.x = p[0];
                if (j + 1 < a.L) v.y = p[1];
                if (j + 2 < a.L) v.z = p[2];
                if (j + 3 < a.L) v.w = p[3];
            }
        }
        *reinterpret_cast<float4*>(tile + row * kTilePitch + c4) = v;
    }
    // (LDS operations of one wavefront are carried out in order and the compiler keeps a load behind a store that
    // may alias it, so the lanes see each other's rows without any wait; a fence here would also wait for the K and
    // V loads in flight and serialise the tiles)
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const float4 v = *reinterpret_cast<const float4*>(tile + col * kTilePitch + 8 * g + 4 * hf);
        b[4 * g] = v.x * kLog2e; b[4 * g + 1] = v.y * kLog2e; b[4 * g + 2] = v.z * kLog2e; b[4 * g + 3] = v.w * kLog2e;
    }
    __builtin_amdgcn_wave_barrier();
}

// Bit n of the result: key j0 + n may be attended to in batch row r (inside the sequence and not masked).
__device__ __forceinline__ uint32_t valid_keys(const Args& a, int r, int j0, int col) {
    const int j = j0 + col;
    const bool ok = j < a.L && (!a.mask || a.mask[(size_t)r * a.L + j] != 0.f);
    return (uint32_t)__ballot(ok);          // (lanes 32 .. 63 repeat lanes 0 .. 31: the low word is enough)
}

// S^T tile in base-2 logits for the wavefront's queries (lane = query i, register v = key j0 + 8(v/4) + 4hf + v%4):
// acc * qscale2 + bias tile, -inf for keys that are masked or beyond L (and for queries beyond L).
__device__ __forceinline__ void logits_by_query(f32x16& s, const f32x16& b, uint32_t keys, bool query_ok, float qscale2, int hf) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int n = 8 * (v >> 2) + (v & 3);
        const bool ok = query_ok && ((keys >> (n + 4 * hf)) & 1u);
        s[v] = ok ? s[v] * qscale2 + b[v] : -INFINITY;
    }
}

// the same with lane = key j and register v = query i0 + 8(v/4) + 4hf + v%4
__device__ __forceinline__ void logits_by_key(f32x16& s, const Args& a, int r, int h, int i0, int j, int hf) {
    const bool key_ok = j < a.L && (!a.mask || a.mask[(size_t)r * a.L + j] != 0.f);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = i0 + 8 * (v >> 2) + 4 * hf + (v & 3);
        const bool ok = key_ok && i < a.L;
        const float b = (a.bias && ok) ? a.bias[((size_t)h * a.L + i) * a.L + j] * kLog2e : 0.f;
        s[v] = ok ? s[v] * a.qscale2 + b : -INFINITY;
    }
}

// ====================================================================================
template <int D>
__global__ __launch_bounds__(256) void k_bwd_stats(Args a) {
    constexpr int KS = (D + 15) / 16;
    const int lane = threadIdx.x & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nt = a.Lp >> 5;
    const int task = blockIdx.x * 4 + wave;
    if (task >= a.R * a.H * nt) return;
    const int rh = task / nt, i0 = (task - rh * nt) * 32, r = rh / a.H, h = rh - r * a.H, i = i0 + col;
    const size_t base = (size_t)rh * a.L * D;
    __shared__ __attribute__((aligned(16))) float s_tile[4 * 32 * kTilePitch];
    float* tile = s_tile + wave * 32 * kTilePitch;
    Frag qf[KS];
    load_rows<D>(qf, a.q + base, i0, a.L, col, hf);

    float m = -INFINITY, l = 0.f;
    f32x16 ctx = zero16();          // ctx^T: lane = query, register v = channel 8(v/4) + 4hf + v%4
    for (int j0 = 0; j0 < a.L; j0 += 32) {
        Frag kf[KS], vt[2], pf[2];
        load_rows<D>(kf, a.k + base, j0, a.L, col, hf);
        load_cols<D>(vt, a.vT + (size_t)rh * D * a.Lp, j0, a.Lp, col, hf);
        const uint32_t keys = valid_keys(a, r, j0, col);
        f32x16 bt;
        bias_tile_by_query(bt, a, h, i0, j0, tile, lane, col, hf);
        f32x16 s = zero16();
#pragma unroll
        for (int t = 0; t < KS; ++t) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t].v, qf[t].v, s, 0, 0, 0);
        logits_by_query(s, bt, keys, i < a.L, a.qscale2, hf);
        float tmax = s[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, s[v]);
        tmax = fmaxf(tmax, other_half(tmax));
        const float m_new = fmaxf(m, tmax);
        // (nothing valid so far: every weight of the tile is zero and nothing is rescaled)
        const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m - m_new);
        float lt = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            s[v] = m_new == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(s[v] - m_new);
            lt += s[v];
            ctx[v] *= alpha;
        }
        l = l * alpha + lt;
        m = m_new;
        pack_rows(pf, s);
#pragma unroll
        for (int t = 0; t < 2; ++t) ctx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt[t].v, pf[t].v, ctx, 0, 0, 0);
    }
    const float l_tot = l + other_half(l);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    // a query without unmasked keys: logsumexp = +inf makes every recomputed weight exp2(s - inf) = 0
    const float lse = l_tot > 0.f ? m + __builtin_amdgcn_logf(l_tot) : INFINITY;

    float dl = 0.f;
    if (i >= a.L) {         // pad queries: zeros in the position-contiguous copy of dctx
#pragma unroll
        for (int gq = 0; gq < 4; ++gq)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (8 * gq + 4 * hf + e < D) a.dctxT[((size_t)rh * D + 8 * gq + 4 * hf + e) * a.Lp + i] = 0;
    }
    if (i < a.L) {
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int e0 = 8 * gq + 4 * hf;
            if (e0 < D) {
                const size_t off = base + (size_t)i * D + e0;
                const uint2 dov = *reinterpret_cast<const uint2*>(a.dout + off);
                const uint2 gv = *reinterpret_cast<const uint2*>(a.g + off);
                const float d_o[4] = {lo_f32(dov.x), hi_f32(dov.x), lo_f32(dov.y), hi_f32(dov.y)};
                const float gg[4] = {lo_f32(gv.x), hi_f32(gv.x), lo_f32(gv.y), hi_f32(gv.y)};
                float dgv[4], dc[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float c = ctx[4 * gq + e] * inv;
                    dgv[e] = d_o[e] * c;
                    // delta uses the very dctx values the other kernels read (rounded to bf16)
                    dc[e] = lo_f32(pack2(d_o[e] * gg[e], 0.f));
                    dl += dc[e] * c;
                }
                *reinterpret_cast<uint2*>(a.dg + off) = make_uint2(pack2(dgv[0], dgv[1]), pack2(dgv[2], dgv[3]));
                *reinterpret_cast<uint2*>(a.dctx + off) = make_uint2(pack2(dc[0], dc[1]), pack2(dc[2], dc[3]));
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    a.dctxT[((size_t)rh * D + e0 + e) * a.Lp + i] = (bf16_t)(pack2(dc[e], 0.f) & 0xffffu);
            }
        }
    }
    dl += other_half(dl);
    if (hf == 0) {       // (Lp slots per (row, head): queries beyond L get a defined value too)
        a.lse[(size_t)rh * a.Lp + i] = i < a.L ? lse : INFINITY;
        a.delta[(size_t)rh * a.Lp + i] = dl;
    }
}

// ====================================================================================
template <int D>
__global__ __launch_bounds__(256) void k_bwd_dq(Args a) {
    constexpr int KS = (D + 15) / 16;
    const int lane = threadIdx.x & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nt = a.Lp >> 5;
    const int task = blockIdx.x * 4 + wave;
    if (task >= a.R * a.H * nt) return;
    const int rh = task / nt, i0 = (task - rh * nt) * 32, r = rh / a.H, h = rh - r * a.H, i = i0 + col;
    const size_t base = (size_t)rh * a.L * D;
    __shared__ __attribute__((aligned(16))) float s_tile[4 * 32 * kTilePitch];
    float* tile = s_tile + wave * 32 * kTilePitch;
    Frag qf[KS], dcf[KS];
    load_rows<D>(qf, a.q + base, i0, a.L, col, hf);
    load_rows<D>(dcf, a.dctx + base, i0, a.L, col, hf);
    const float lse = a.lse[(size_t)rh * a.Lp + i], delta = a.delta[(size_t)rh * a.Lp + i];

    f32x16 dq = zero16();           // dq^T: lane = query, register = channel
    for (int j0 = 0; j0 < a.L; j0 += 32) {
        Frag kf[KS], vf[KS], kt[2], dsf[2];
        load_rows<D>(kf, a.k + base, j0, a.L, col, hf);
        load_rows<D>(vf, a.v + base, j0, a.L, col, hf);
        load_cols<D>(kt, a.kT + (size_t)rh * D * a.Lp, j0, a.Lp, col, hf);
        const uint32_t keys = valid_keys(a, r, j0, col);
        f32x16 bt;
        bias_tile_by_query(bt, a, h, i0, j0, tile, lane, col, hf);
        f32x16 s = zero16(), dp = zero16();
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t].v, qf[t].v, s, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t].v, dcf[t].v, dp, 0, 0, 0);
        }
        logits_by_query(s, bt, keys, i < a.L, a.qscale2, hf);
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = __builtin_amdgcn_exp2f(s[v] - lse) * (dp[v] - delta);
        pack_rows(dsf, s);
#pragma unroll
        for (int t = 0; t < 2; ++t) dq = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt[t].v, dsf[t].v, dq, 0, 0, 0);
    }
    if (i < a.L) {
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int e0 = 8 * gq + 4 * hf;
            if (e0 < D)
                *reinterpret_cast<uint2*>(a.dq + base + (size_t)i * D + e0) =
                    make_uint2(pack2(dq[4 * gq] * a.scale, dq[4 * gq + 1] * a.scale),
                               pack2(dq[4 * gq + 2] * a.scale, dq[4 * gq + 3] * a.scale));
        }
    }
}

// ====================================================================================
template <int D>
__global__ __launch_bounds__(256) void k_bwd_dkv(Args a) {
    constexpr int KS = (D + 15) / 16;
    const int lane = threadIdx.x & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nt = a.Lp >> 5;
    const int task = blockIdx.x * 4 + wave;
    if (task >= a.R * a.H * nt) return;
    const int rh = task / nt, j0 = (task - rh * nt) * 32, r = rh / a.H, h = rh - r * a.H, j = j0 + col;
    const size_t base = (size_t)rh * a.L * D;
    Frag kf[KS], vf[KS];
    load_rows<D>(kf, a.k + base, j0, a.L, col, hf);
    load_rows<D>(vf, a.v + base, j0, a.L, col, hf);

    f32x16 dk = zero16(), dv = zero16();     // dk^T, dv^T: lane = key, register = channel
    for (int i0 = 0; i0 < a.L; i0 += 32) {
        Frag qf[KS], dcf[KS], qt[2], dct[2], pf[2], dsf[2];
        load_rows<D>(qf, a.q + base, i0, a.L, col, hf);
        load_rows<D>(dcf, a.dctx + base, i0, a.L, col, hf);
        load_cols<D>(qt, a.qT + (size_t)rh * D * a.Lp, i0, a.Lp, col, hf);
        load_cols<D>(dct, a.dctxT + (size_t)rh * D * a.Lp, i0, a.Lp, col, hf);
        f32x16 s = zero16(), dp = zero16();      // lane = key, register v = query i0 + 8(v/4) + 4hf + v%4
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[t].v, kf[t].v, s, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dcf[t].v, vf[t].v, dp, 0, 0, 0);
        }
        logits_by_key(s, a, r, h, i0, j, hf);
        const float* lp = a.lse + (size_t)rh * a.Lp + i0 + 4 * hf;
        const float* dp_ = a.delta + (size_t)rh * a.Lp + i0 + 4 * hf;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const float4 l4 = *reinterpret_cast<const float4*>(lp + 8 * gq);
            const float4 d4 = *reinterpret_cast<const float4*>(dp_ + 8 * gq);
            const float ls[4] = {l4.x, l4.y, l4.z, l4.w}, ds_[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float p = __builtin_amdgcn_exp2f(s[4 * gq + e] - ls[e]);
                s[4 * gq + e] = p;
                dp[4 * gq + e] = p * (dp[4 * gq + e] - ds_[e]);
            }
        }
        pack_rows(pf, s);
        pack_rows(dsf, dp);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            dv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dct[t].v, pf[t].v, dv, 0, 0, 0);
            dk = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt[t].v, dsf[t].v, dk, 0, 0, 0);
        }
    }
    if (j < a.L) {
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int e0 = 8 * gq + 4 * hf;
            if (e0 < D) {
                const size_t off = base + (size_t)j * D + e0;
                *reinterpret_cast<uint2*>(a.dv + off) = make_uint2(pack2(dv[4 * gq], dv[4 * gq + 1]), pack2(dv[4 * gq + 2], dv[4 * gq + 3]));
                *reinterpret_cast<uint2*>(a.dk + off) = make_uint2(pack2(dk[4 * gq] * a.scale, dk[4 * gq + 1] * a.scale),
                                                                   pack2(dk[4 * gq + 2] * a.scale, dk[4 * gq + 3] * a.scale));
            }
        }
    }
}

// ====================================================================================
template <int D>
__global__ __launch_bounds__(256) void k_bwd_dbias(Args a) {
    constexpr int KS = (D + 15) / 16;
    const int lane = threadIdx.x & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nt = a.Lp >> 5;
    const int task = blockIdx.x * 4 + wave;
    if (task >= a.row_chunks * a.H * nt * nt) return;
    const int chunk = task / (a.H * nt * nt), t2 = task - chunk * a.H * nt * nt;
    const int h = t2 / (nt * nt), rem = t2 - h * nt * nt, i0 = (rem / nt) * 32, j0 = (rem - (rem / nt) * nt) * 32;
    const int r_begin = chunk * a.rows_per_chunk;
    const int r_end = r_begin + a.rows_per_chunk < a.R ? r_begin + a.rows_per_chunk : a.R;
    const int i = i0 + col;
    __shared__ __attribute__((aligned(16))) float s_tile[4 * 32 * kTilePitch];
    f32x16 bt;
    bias_tile_by_query(bt, a, h, i0, j0, s_tile + wave * 32 * kTilePitch, lane, col, hf);
    f32x16 acc = zero16();          // lane = query i, register v = key j0 + 8(v/4) + 4hf + v%4
    for (int r = r_begin; r < r_end; ++r) {
        const int rh = r * a.H + h;
        const size_t base = (size_t)rh * a.L * D;
        Frag qf[KS], dcf[KS], kf[KS], vf[KS];
        load_rows<D>(qf, a.q + base, i0, a.L, col, hf);
        load_rows<D>(dcf, a.dctx + base, i0, a.L, col, hf);
        load_rows<D>(kf, a.k + base, j0, a.L, col, hf);
        load_rows<D>(vf, a.v + base, j0, a.L, col, hf);
        const float lse = a.lse[(size_t)rh * a.Lp + i], delta = a.delta[(size_t)rh * a.Lp + i];
        const uint32_t keys = valid_keys(a, r, j0, col);
        f32x16 s = zero16(), dp = zero16();
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t].v, qf[t].v, s, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t].v, dcf[t].v, dp, 0, 0, 0);
        }
        logits_by_query(s, bt, keys, i < a.L, a.qscale2, hf);
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] += __builtin_amdgcn_exp2f(s[v] - lse) * (dp[v] - delta);
    }
    if (i < a.L) {
        float* out = a.row_chunks > 1 ? a.dbias_part + (size_t)chunk * a.H * a.L * a.L : a.dbias;
        float* drow = out + ((size_t)h * a.L + i) * a.L;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int j = j0 + 8 * (v >> 2) + 4 * hf + (v & 3);
            if (j < a.L) drow[j] = acc[v];
        }
    }
}

// dbias = sum over the row chunks of the partial sums, in chunk order (deterministic)
__global__ __launch_bounds__(256) void k_bwd_dbias_reduce(Args a) {
    const size_t n = (size_t)a.H * a.L * a.L;
    for (size_t x = (size_t)blockIdx.x * 256 + threadIdx.x; x < n; x += (size_t)gridDim.x * 256) {
        float t = 0.f;
        for (int c = 0; c < a.row_chunks; ++c) t += a.dbias_part[(size_t)c * n + x];
        a.dbias[x] = t;
    }
}

}  // namespace bwd

bool core_backward_supported(const ff_core_desc& d) {
    return d.dtype == FF_BF16 && (d.head_dim == 8 || d.head_dim == 16 || d.head_dim == 32);
}

// Row chunks of the bias gradient: enough (head, tile, tile, chunk) wavefronts to fill the chip, at least 8 rows each.
static int dbias_chunks(const ff_core_desc& d) {
    const int nt = (d.length + 31) / 32;
    const long tasks = (long)d.heads * nt * nt;
    int chunks = (int)((4096 + tasks - 1) / tasks);
    if (chunks > d.rows / 8) chunks = d.rows / 8;
    return chunks < 1 ? 1 : chunks;
}

size_t core_backward_workspace(const ff_core_desc& d) {
    const size_t Lp = bwd::round_up(d.length, 32), rh = (size_t)d.rows * d.heads;
    const int chunks = dbias_chunks(d);
    return 2 * bwd::align256(rh * Lp * 4) + bwd::align256(rh * d.length * d.head_dim * 2) +
           4 * bwd::align256(rh * d.head_dim * Lp * 2) +
           (chunks > 1 ? bwd::align256((size_t)chunks * d.heads * d.length * d.length * 4) : 0);
}

ff_status core_backward_run(const ff_core_desc& d, const void* q, const void* k, const void* v, const void* g, const float* bias,
                            const float* mask, const void* dout, void* dq, void* dk, void* dv, void* dg, float* dbias,
                            void* ws, hipStream_t st) {
    using namespace bwd;
    Args a{};
    a.q = (const bf16_t*)q; a.k = (const bf16_t*)k; a.v = (const bf16_t*)v; a.g = (const bf16_t*)g; a.dout = (const bf16_t*)dout;
    a.bias = bias; a.mask = mask; a.dq = (bf16_t*)dq; a.dk = (bf16_t*)dk; a.dv = (bf16_t*)dv; a.dg = (bf16_t*)dg; a.dbias = dbias;
    a.R = d.rows; a.H = d.heads; a.L = d.length; a.Lp = round_up(d.length, 32);
    const size_t rh = (size_t)d.rows * d.heads;
    char* p = (char*)ws;
    a.lse = (float*)p; p += align256(rh * a.Lp * 4);
    a.delta = (float*)p; p += align256(rh * a.Lp * 4);
    a.dctx = (bf16_t*)p; p += align256(rh * d.length * d.head_dim * 2);
    const size_t tbytes = align256(rh * d.head_dim * a.Lp * 2);
    a.qT = (bf16_t*)p; p += tbytes;
    a.kT = (bf16_t*)p; p += tbytes;
    a.vT = (bf16_t*)p; p += tbytes;
    a.dctxT = (bf16_t*)p; p += tbytes;
    a.row_chunks = bias ? dbias_chunks(d) : 1;
    a.rows_per_chunk = (d.rows + a.row_chunks - 1) / a.row_chunks;
    a.dbias_part = a.row_chunks > 1 ? (float*)p : nullptr;
    a.qscale2 = kLog2e / sqrtf((float)d.head_dim);
    a.scale = 1.f / sqrtf((float)d.head_dim);
    const int nt = a.Lp / 32;
    const dim3 g1((unsigned)((rh * nt + 3) / 4)), g2((unsigned)(((size_t)a.row_chunks * d.heads * nt * nt + 3) / 4));
#define FF_BWD(KERNEL, GRID, KIND)                                                                       \
    do {                                                                                                 \
        Timed t(KIND, st);                                                                               \
        if (d.head_dim == 8) hipLaunchKernelGGL((KERNEL<8>), GRID, dim3(256), 0, st, a);                 \
        else if (d.head_dim == 16) hipLaunchKernelGGL((KERNEL<16>), GRID, dim3(256), 0, st, a);          \
        else hipLaunchKernelGGL((KERNEL<32>), GRID, dim3(256), 0, st, a);                                \
    } while (0)
    const dim3 gt(g1.x, 3);
    FF_BWD(k_bwd_transpose, gt, KK_BWD_STATS);
    FF_BWD(k_bwd_stats, g1, KK_BWD_STATS);
    FF_BWD(k_bwd_dq, g1, KK_BWD_DQ);
    FF_BWD(k_bwd_dkv, g1, KK_BWD_DKV);
    if (bias) {
        FF_BWD(k_bwd_dbias, g2, KK_BWD_DBIAS);
        if (a.row_chunks > 1) {
            Timed t(KK_BWD_DBIAS, st);
            hipLaunchKernelGGL(k_bwd_dbias_reduce, dim3(1024), dim3(256), 0, st, a);
        }
    }
#undef FF_BWD
    return check_launch("attention core backward");
}

}  // namespace ff
