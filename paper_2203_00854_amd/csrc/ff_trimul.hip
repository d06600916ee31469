// Triangular multiplicative update of the pair stack (FastFold Section 2.3, Figure 3; the left / right
// projections and their gates merged into one GEMM as in Section 5.2), bf16, gfx950 matrix cores.
//
//   zn = LayerNorm_in(z);  a = mask * sigmoid(zn W_ag^T + b_ag) * (zn W_ap^T + b_ap);  b likewise;
//   g = sigmoid(zn W_g^T + b_g)
//   outgoing t[i,j,:] = sum_k a[i,k,:] * b[j,k,:];   incoming t[i,j,:] = sum_k a[k,i,:] * b[k,j,:]
//   out = g * (LayerNorm_out(t) W_o^T + b_o)   (+ z in the residual form)
//
// Four launches per call:
//   k_tm_prep  folds the LayerNorm gains into the weights: W' = bf16(W * gamma), S = rowsum(W'),
//              Cn = W beta + bias, so that LN(x) W^T + bias = rstd * (x W'^T - mean * S + Cn / rstd): the
//              matrix cores read the raw activations, and S, Cn of a row (as bfloat16 pairs) are one more
//              contraction step against the token's -mean and 1 / rstd (token_side)
//   k_tm_proj  one merged GEMM over the 4c features of the left and right side.  A projection tile is
//              contracted together with its gate tile (features x tokens), so that the lane that holds a
//              projection value also holds its gate value; a and b leave channel-major, [c][N][Np], which makes every
//              channel a dense N x N matrix for the next kernel.  The incoming form is the outgoing form
//              on the transposed view of z (strides), so a[c][i][k] then holds a of pair (k, i).
//   k_tm_mul   per channel t_c = A_c B_c^T: a batched N x N x N contraction, 128 x 128 or 256 x 256 tiles through
//              LDS; t leaves as [i][channel][j]
//   k_tm_out   LayerNorm over the channels of t (read as 2-byte loads straight into operand fragments), output
//              projection; the output gate g is computed here, from z, in float32 (it never exists in
//              memory), then the product and the optional residual
//
// Matrix-core operand layouts (wave64, v_mfma_f32_32x32x16_bf16): A (32 x 16): lane l holds row l%32,
// columns 8*(l/32)..+7; B (16 x 32): lane l holds column l%32, rows 8*(l/32)..+7; D (32 x 32): lane l
// holds column l%32, register v holds row 8*(v/4) + 4*(l/32) + v%4.
#include "ff_common.h"

namespace ff {
namespace tm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

union Frag {
    bf16x8 v;
    uint4 u;
    uint32_t w[4];
};

__device__ __forceinline__ uint32_t pack2(float a, float b) {   // a -> low half (first element)
    bf16x2 t;
    t[0] = (__bf16)a;
    t[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, t);
}
// After the call lanes of the lower half hold (a of lower lane, a of upper lane) and lanes of the upper half hold
// (b of lower lane, b of upper lane)
__device__ __forceinline__ void merge_halves(uint32_t& a, uint32_t& b) {
    auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    a = r[0];
    b = r[1];
}
__device__ __forceinline__ float lo_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_f32(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// LayerNorm statistics of the token whose K channels lie in the fragments of the two lanes (col, hf = 0 | 1),
// channels beyond K being zero: mean, 1 / sqrt(var + eps) and sqrt(var + eps), float32.  Sum and sum of squares
// come from the packed pairs directly (two-element dot products with float32 accumulation: the squares of
// bfloat16 values are exact in float32), the variance as E[x^2] - mean^2: its rounding error is about
// 2^-22 (1 + mean^2 / variance), far below what the bfloat16 tokens themselves carry.
template <int KC>
__device__ __forceinline__ void token_stats(const Frag (&xa)[KC], int K, float eps, float& mean, float& rstd, float& istd) {
    const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
    float sum = 0.f, sq = 0.f;
#pragma unroll
    for (int s = 0; s < KC; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bf16x2 w = __builtin_bit_cast(bf16x2, xa[s].w[i]);
            sum = __builtin_amdgcn_fdot2_f32_bf16(w, ones, sum, false);
            sq = __builtin_amdgcn_fdot2_f32_bf16(w, w, sq, false);
        }
    sum += __shfl_xor(sum, 32, 64);
    sq += __shfl_xor(sq, 32, 64);
    const float rk = 1.f / (float)K;
    mean = sum * rk;
    const float ve = fmaxf(sq * rk - mean * mean, 0.f) + eps;
    rstd = rsqrtf(ve);
    istd = ve * rstd;
}

// LayerNorm followed by a projection with folded weights W' (row sums S, offsets C) is rstd (W' x - mean S + C / rstd):
// the matrix cores take the tokens as stored, and the two corrections are ONE MORE contraction step.  Its weight
// side (a row's eight slots, written by k_tm_prep) is S S S' C C C' 0 0 with S + S' = the row sum as a bfloat16 pair
// (hi, lo) and C likewise; its token side, built here, holds -mean and 1 / rstd split the same way in the order
// hi lo hi: the three largest of the four partial products, 16 significant bits.  The upper half of the
// wavefront (slots 8 .. 15 of the step) holds zeros.
__device__ __forceinline__ void split2(float v, float& hi, float& lo) {
    hi = __uint_as_float(pack2(0.f, v) & 0xffff0000u);
    lo = v - hi;
}
__device__ __forceinline__ Frag token_side(float mean, float istd, int hf) {
    float m_hi, m_lo, r_hi, r_lo;
    split2(-mean, m_hi, m_lo);
    split2(istd, r_hi, r_lo);
    Frag xe;
    xe.w[0] = hf ? 0u : pack2(m_hi, m_lo);
    xe.w[1] = hf ? 0u : pack2(m_hi, r_hi);
    xe.w[2] = hf ? 0u : pack2(r_lo, r_hi);
    xe.w[3] = 0u;
    return xe;
}

// ====================================================================================
// Weight preparation, one wavefront per output row.
//   rows [0, 64 * n_pairs): the merged projection in the order k_tm_proj sweeps it.  Pair p < G (G = c / 32):
//     rows 64p .. +31 = left projection of channels 32p .. +31, rows 64p + 32 .. +63 = their gate;
//     pairs G .. 2G - 1 the right side.
//   then the output projection (LayerNorm_out folded in) and the output gate (LayerNorm_in folded in), c_z rows each.
struct TmPrepArgs {
    const bf16_t *w_ap, *b_ap, *w_ag, *b_ag, *w_bp, *b_bp, *w_bg, *b_bg, *w_g, *b_g, *ln_g, *ln_b;
    const bf16_t *w_o, *b_o, *lno_g, *lno_b;
    bf16_t *wp1, *wp3, *wp4;       // [64 n_pairs][Kp1], [cz][Kp3], [cz][Kp1]
    bf16_t *ext1, *ext3, *ext4;    // [rows][8]: the extra contraction step of every row (see token_side)
    int cz, c, G, n_pairs, Kp1, Kp3;
};

__global__ __launch_bounds__(256) void k_tm_prep(TmPrepArgs a) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int rows1 = 64 * a.n_pairs;
    if (n >= rows1 + 2 * a.cz) return;
    const bf16_t *wrow = nullptr, *gamma, *beta;
    float bias = 0.f;
    int K, Kp;
    bf16_t *dst, *ext;
    if (n < rows1) {
        const int p = n >> 6, half = (n >> 5) & 1, j = n & 31;
        K = a.cz; Kp = a.Kp1; gamma = a.ln_g; beta = a.ln_b;
        dst = a.wp1 + (size_t)n * Kp; ext = a.ext1 + (size_t)n * 8;
        const bool left = p < a.G;
        const int ch = 32 * (left ? p : p - a.G) + j;
        const bf16_t* w = left ? (half ? a.w_ag : a.w_ap) : (half ? a.w_bg : a.w_bp);
        const bf16_t* b = left ? (half ? a.b_ag : a.b_ap) : (half ? a.b_bg : a.b_bp);
        wrow = w + (size_t)ch * K;
        bias = bf16_to_f32(b[ch]);
    } else if (n < rows1 + a.cz) {
        const int f = n - rows1;
        K = a.c; Kp = a.Kp3; gamma = a.lno_g; beta = a.lno_b;
        dst = a.wp3 + (size_t)f * Kp; ext = a.ext3 + (size_t)f * 8;
        wrow = a.w_o + (size_t)f * K;
        bias = bf16_to_f32(a.b_o[f]);
    } else {
        const int f = n - rows1 - a.cz;
        K = a.cz; Kp = a.Kp1; gamma = a.ln_g; beta = a.ln_b;
        dst = a.wp4 + (size_t)f * Kp; ext = a.ext4 + (size_t)f * 8;
        wrow = a.w_g + (size_t)f * K;
        bias = bf16_to_f32(a.b_g[f]);
    }
    float sum = 0.f, cst = 0.f;
    for (int k = lane; k < Kp; k += 64) {
        float r = 0.f;
        if (k < K) {
            const float w = bf16_to_f32(wrow[k]);
            r = bf16_to_f32(f32_to_bf16(w * bf16_to_f32(gamma[k])));
            cst += w * bf16_to_f32(beta[k]);
        }
        dst[k] = f32_to_bf16(r);
        sum += r;
    }
    sum = wave_sum(sum);
    cst = wave_sum(cst);
    if (lane == 0) {
        const float C = cst + bias;
        const bf16_t s_hi = f32_to_bf16(sum), s_lo = f32_to_bf16(sum - bf16_to_f32(s_hi));
        const bf16_t c_hi = f32_to_bf16(C), c_lo = f32_to_bf16(C - bf16_to_f32(c_hi));
        ext[0] = s_hi; ext[1] = s_hi; ext[2] = s_lo; ext[3] = c_hi; ext[4] = c_hi; ext[5] = c_lo;
        ext[6] = f32_to_bf16(0.f); ext[7] = f32_to_bf16(0.f);
    }
}

// ====================================================================================
// Merged projection.  Block = 8 wavefronts, each owning one 32-token tile (tokens of one row of the view)
// as register-resident operand fragments and sweeping the prepared weight matrix 64 rows (a "pair") at a
// time; the matrix is resident in LDS (row pitch padded by 16 bytes: conflict-free operand reads).
struct TmProjArgs {
    const bf16_t* z;
    int64_t sr, sl;          // token (r, l) of the view at z + (r*sr + l*sl) * K; the same index addresses mask
    const float* mask;       // or NULL
    int N, Np, K, C, cz, G, n_pairs;
    int ppb;                 // pairs per block: blockIdx.y takes pairs [blockIdx.y * ppb, + ppb)
    float eps;
    const bf16_t* wp;        // [64 n_pairs][16 KC]
    const bf16_t* ext;       // [64 n_pairs][8]
    bf16_t *a, *b;           // [C][N][Np]
};

template <int KC>
__global__ __launch_bounds__(512, 2) void k_tm_proj(TmProjArgs p) {
    constexpr int PITCH = KC * 32 + 16;                 // bytes per weight row in LDS
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* s_w = smem;       // [64 ppb][PITCH]: the block's share of the folded weights, a row's extra step in its last 16 bytes
    const int pr_first = blockIdx.y * p.ppb;
    constexpr int OPITCH = 80;                          // bytes per channel row of a staged output half-tile [16][32]

    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tpr = p.Np >> 5;                          // token tiles per row
    const int tiles_m = p.N * tpr;
    // the wavefront's own staging area (only it reads or writes there; its LDS operations complete in order)
    unsigned char* s_o = smem + (size_t)64 * p.ppb * PITCH + wave * (16 * OPITCH);

    // The block's share of the folded weight matrix (all of it, at most 512 rows of 256 bytes, for large inputs;
    // a quarter for small ones, which need the blocks) stays in LDS for the life of the block, which works through
    // token tiles blockIdx.x * 8 + wave, + 8 * gridDim.x, ...: after this one barrier the wavefronts run
    // independently, so that one wavefront's matrix instructions overlap another's epilogue arithmetic on the
    // same SIMD, and the weights are read from L2 once per block, not once per 256 tokens.
    for (int id = tid; id < 64 * p.ppb * (2 * KC + 1); id += 512) {
        const int row = id / (2 * KC + 1), pc = id - row * (2 * KC + 1);
        const bf16_t* src = pc < 2 * KC ? p.wp + (size_t)(64 * pr_first + row) * (16 * KC) + pc * 8
                                        : p.ext + (size_t)(64 * pr_first + row) * 8;
        *reinterpret_cast<uint4*>(s_w + row * PITCH + pc * 16) = *reinterpret_cast<const uint4*>(src);
    }
    __syncthreads();                                    // (the only barrier)

    const size_t plane = (size_t)p.N * p.Np;

    for (int tg = blockIdx.x * 8 + wave; tg < tiles_m; tg += gridDim.x * 8) {
        const int r = tg / tpr, l0 = (tg - r * tpr) * 32, l = l0 + col;
        const bool valid = l < p.N;
        const int64_t tok = (int64_t)r * p.sr + (int64_t)(valid ? l : 0) * p.sl;
        Frag xa[KC];
        {
            const bf16_t* zp = p.z + tok * p.K;
#pragma unroll
            for (int s = 0; s < KC; ++s) {
                xa[s].u = make_uint4(0, 0, 0, 0);
                if (valid && 16 * s + 8 * hf < p.K) xa[s].u = *reinterpret_cast<const uint4*>(zp + 16 * s + 8 * hf);
            }
        }
        const float mval = valid ? (p.mask ? p.mask[tok] : 1.f) : 0.f;
        float mean, rstd, istd;
        token_stats<KC>(xa, p.K, p.eps, mean, rstd, istd);
        const Frag xe = token_side(mean, istd, hf);
        const float nrl = -kLog2e * rstd;               // sigmoid(rstd t) = 1 / (1 + exp2(nrl t))
        const float rm = rstd * mval;

        for (int pl = 0; pl < p.ppb; ++pl) {
            const int pr = pr_first + pl;
            const unsigned char* st = s_w + (size_t)pl * 64 * PITCH;
            f32x16 acc0, acc1;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc0[v] = acc1[v] = 0.f;
            // features x tokens: the lane owns one token (its statistics are in its registers); register v holds
            // channel 8 (v / 4) + 4 hf + v % 4 of the pair's 32, the projection in acc0 and the gate in acc1
#pragma unroll
            for (int s = 0; s < KC; ++s) {
                Frag w0, w1;
                w0.u = *reinterpret_cast<const uint4*>(st + col * PITCH + (2 * s + hf) * 16);
                w1.u = *reinterpret_cast<const uint4*>(st + (32 + col) * PITCH + (2 * s + hf) * 16);
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w0.v, xa[s].v, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1.v, xa[s].v, acc1, 0, 0, 0);
            }
            {
                Frag w0, w1;                            // - mean S + C / rstd (the same 16 bytes for both halves: the token side's upper half is zero)
                w0.u = *reinterpret_cast<const uint4*>(st + col * PITCH + 2 * KC * 16);
                w1.u = *reinterpret_cast<const uint4*>(st + (32 + col) * PITCH + 2 * KC * 16);
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w0.v, xe.v, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1.v, xe.v, acc1, 0, 0, 0);
            }
            const bool left = pr < p.G;
            const int ch0 = 32 * (left ? pr : pr - p.G);
            // A lane holds ONE position of 16 channels, and the channel rows of a and b lie a whole plane apart:
            // 16 channels at a time the results are turned in LDS into rows [channel][32 positions] and leave as
            // 16-byte pieces, a store instruction writing 16 channel rows of 64 contiguous bytes (2-byte stores,
            // one channel row per half-wave and instruction, took a quarter of the kernel's time).
            bf16_t* dst = (left ? p.a : p.b) + (size_t)(ch0 + (lane >> 2)) * plane + (size_t)r * p.Np + l0 + 8 * (lane & 3);
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                for (int gg = 0; gg < 2; ++gg) {
                    const int g = 2 * hh + gg;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float gate = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(nrl * acc1[4 * g + e]));
                        *reinterpret_cast<bf16_t*>(s_o + (8 * gg + 4 * hf + e) * OPITCH + col * 2) =
                            (bf16_t)(pack2(acc0[4 * g + e] * rm * gate, 0.f) & 0xffffu);
                    }
                }
                const uint4 v = *reinterpret_cast<const uint4*>(s_o + (lane >> 2) * OPITCH + (lane & 3) * 16);
                *reinterpret_cast<uint4*>(dst + (size_t)(16 * hh) * plane) = v;
            }
        }
    }
}

// ====================================================================================
// t_c[i][j] = sum_k A_c[i][k] B_c[j][k] for every channel c: block = WI x WJ wavefronts, each TI x TJ accumulator tiles
// (block tile 128 x 128 with 2 x 2 wavefronts of 64 x 64, or 256 x 256 with 2 x 4 wavefronts of 128 x 64), the
// contraction in chunks of 64 through double-buffered LDS.
// Blocks are handed to the 8 XCDs round-robin; channel c goes to XCD c % 8 with all of its tiles, so a
// channel's operands live in one L2.
struct TmMulArgs {
    const bf16_t *a, *b;     // [C][N][Np]
    bf16_t* x;               // [N][C][Np]
    int N, Np, C, tiles_i, tiles_j;     // block tiles along i and along j
};

constexpr int kMulPitch = 144;                          // bytes per 64-element row in LDS (128 + 16 padding)

// Block tile (32 WI TI) x (32 WJ TJ) of one channel: WI x WJ wavefronts, each TI x TJ accumulator tiles of 32 x 32.
// Per contraction step a wavefront reads TI + TJ operand fragments from LDS for TI TJ matrix instructions: the
// LDS read rate is what bounds this kernel (1 KiB per instruction at 2 x 2), hence 4 x 2 tiles per wavefront (and a
// 256 x 256 block tile, eight wavefronts, all of LDS) where the matrix is large enough to fill the chip with those.
template <int WI, int WJ, int TI, int TJ>
struct MulShape {
    static constexpr int NT = 64 * WI * WJ, BI = 32 * WI * TI, BJ = 32 * WJ * TJ;
    static constexpr int RSTEP = NT / 8;                 // rows between the pieces of one thread
    static_assert(BI * 8 / NT == 4 && BJ * 8 / NT == 4, "four 16-byte pieces per thread, operand and chunk");
    static constexpr int STAGE_A = BI * kMulPitch, STAGE_B = BJ * kMulPitch;
    static constexpr size_t SMEM = 2 * (size_t)(STAGE_A + STAGE_B);      // two operands, two buffers
    static_assert((size_t)WI * WJ * 32 * TI * kMulPitch <= SMEM, "the output tiles of all wavefronts fit in LDS");
};

template <int WI, int WJ, int TI, int TJ>
__global__ __launch_bounds__(64 * WI * WJ, 2) void k_tm_mul(TmMulArgs p) {
    using Sh = MulShape<WI, WJ, TI, TJ>;
    constexpr int PITCH = kMulPitch, BI = Sh::BI, BJ = Sh::BJ, RSTEP = Sh::RSTEP;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* s_a = smem;                          // [2][STAGE_A]
    unsigned char* s_b = smem + 2 * Sh::STAGE_A;        // [2][STAGE_B]
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wi = wave / WJ, wj = wave % WJ;
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3, t2 = p.tiles_i * p.tiles_j;
    const int ch = (idx / t2) * 8 + xcd, tile = idx % t2;
    if (ch >= p.C) return;                              // (whole block)
    const int i0 = (tile / p.tiles_j) * BI, j0 = (tile % p.tiles_j) * BJ;
    const size_t plane = (size_t)p.N * p.Np;
    const bf16_t* ac = p.a + (size_t)ch * plane;
    const bf16_t* bc = p.b + (size_t)ch * plane;

    // this thread's four pieces of each operand chunk: rows tid/8 + RSTEP n, piece tid%8 (16 bytes = 8 positions of k)
    // (named registers and macros: arrays captured by a lambda end up in scratch memory)
    const int prow = tid >> 3, pc = tid & 7;
    const bool a_ok0 = i0 + prow < p.N, a_ok1 = i0 + prow + RSTEP < p.N, a_ok2 = i0 + prow + 2 * RSTEP < p.N,
               a_ok3 = i0 + prow + 3 * RSTEP < p.N;
    const bool b_ok0 = j0 + prow < p.N, b_ok1 = j0 + prow + RSTEP < p.N, b_ok2 = j0 + prow + 2 * RSTEP < p.N,
               b_ok3 = j0 + prow + 3 * RSTEP < p.N;
    const size_t rstep = (size_t)RSTEP * p.Np;
    const bf16_t* ap = ac + (size_t)(a_ok0 ? i0 + prow : 0) * p.Np + pc * 8;     // rows + RSTEP n: ap + n * rstep (guarded)
    const bf16_t* bp = bc + (size_t)(b_ok0 ? j0 + prow : 0) * p.Np + pc * 8;
    const int sdst = prow * PITCH + pc * 16;
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    uint4 ra0 = zero4, ra1 = zero4, ra2 = zero4, ra3 = zero4, rb0 = zero4, rb1 = zero4, rb2 = zero4, rb3 = zero4;
#define fetch(KCH)                                                                                     \
    do {                                                                                               \
        const int k0_ = (KCH) * 64;                                                                    \
        const bool k_ok_ = k0_ + pc * 8 < p.Np;   /* Np is a multiple of 32: the last chunk may be half there */ \
        ra0 = zero4;                                                                                   \
        if (a_ok0 && k_ok_) ra0 = *reinterpret_cast<const uint4*>(ap + k0_);                           \
        ra1 = zero4;                                                                                   \
        if (a_ok1 && k_ok_) ra1 = *reinterpret_cast<const uint4*>(ap + rstep + k0_);                   \
        ra2 = zero4;                                                                                   \
        if (a_ok2 && k_ok_) ra2 = *reinterpret_cast<const uint4*>(ap + 2 * rstep + k0_);               \
        ra3 = zero4;                                                                                   \
        if (a_ok3 && k_ok_) ra3 = *reinterpret_cast<const uint4*>(ap + 3 * rstep + k0_);               \
        rb0 = zero4;                                                                                   \
        if (b_ok0 && k_ok_) rb0 = *reinterpret_cast<const uint4*>(bp + k0_);                           \
        rb1 = zero4;                                                                                   \
        if (b_ok1 && k_ok_) rb1 = *reinterpret_cast<const uint4*>(bp + rstep + k0_);                   \
        rb2 = zero4;                                                                                   \
        if (b_ok2 && k_ok_) rb2 = *reinterpret_cast<const uint4*>(bp + 2 * rstep + k0_);               \
        rb3 = zero4;                                                                                   \
        if (b_ok3 && k_ok_) rb3 = *reinterpret_cast<const uint4*>(bp + 3 * rstep + k0_);               \
    } while (0)
#define stash(BUF)                                                                           \
    do {                                                                                     \
        unsigned char* da_ = s_a + (BUF) * Sh::STAGE_A + sdst;                               \
        unsigned char* db_ = s_b + (BUF) * Sh::STAGE_B + sdst;                               \
        *reinterpret_cast<uint4*>(da_) = ra0;                                                \
        *reinterpret_cast<uint4*>(da_ + RSTEP * PITCH) = ra1;                                \
        *reinterpret_cast<uint4*>(da_ + 2 * RSTEP * PITCH) = ra2;                            \
        *reinterpret_cast<uint4*>(da_ + 3 * RSTEP * PITCH) = ra3;                            \
        *reinterpret_cast<uint4*>(db_) = rb0;                                                \
        *reinterpret_cast<uint4*>(db_ + RSTEP * PITCH) = rb1;                                \
        *reinterpret_cast<uint4*>(db_ + 2 * RSTEP * PITCH) = rb2;                            \
        *reinterpret_cast<uint4*>(db_ + 3 * RSTEP * PITCH) = rb3;                            \
    } while (0)

    f32x16 acc[TJ][TI];     // [j tile][i tile]: lane = i, registers = j
#pragma unroll
    for (int tj = 0; tj < TJ; ++tj)
#pragma unroll
        for (int ti = 0; ti < TI; ++ti)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tj][ti][v] = 0.f;

    const int nk = (p.Np + 63) >> 6;
    fetch(0);
    stash(0);
    if (nk > 1) {
        fetch(1);
        stash(1);
    }
    __syncthreads();
    // chunk kc + 2 travels to registers while the matrix cores work on chunk kc, and takes over its LDS half
    // after the barrier
    for (int kc = 0; kc < nk; ++kc) {
        const bool more = kc + 2 < nk;
        if (more) fetch(kc + 2);
        const unsigned char* sa = s_a + (kc & 1) * Sh::STAGE_A + (wi * 32 * TI + col) * PITCH + hf * 16;
        const unsigned char* sb = s_b + (kc & 1) * Sh::STAGE_B + (wj * 32 * TJ + col) * PITCH + hf * 16;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            Frag af[TI], bf[TJ];
#pragma unroll
            for (int ti = 0; ti < TI; ++ti) af[ti].u = *reinterpret_cast<const uint4*>(sa + ti * 32 * PITCH + kk * 32);
#pragma unroll
            for (int tj = 0; tj < TJ; ++tj) bf[tj].u = *reinterpret_cast<const uint4*>(sb + tj * 32 * PITCH + kk * 32);
#pragma unroll
            for (int tj = 0; tj < TJ; ++tj)
#pragma unroll
                for (int ti = 0; ti < TI; ++ti)
                    acc[tj][ti] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[tj].v, af[ti].v, acc[tj][ti], 0, 0, 0);
        }
        __syncthreads();
        if (more) stash(kc & 1);
    }
#undef fetch
#undef stash

    // t leaves as [i][channel][j]: the channels of a row i lie close together, which is what the LayerNorm over
    // the channels in k_tm_out reads (128 short segments inside half a megabyte instead of one per 8 MiB plane).
    // A lane holds 8-byte pieces of 32 TI different rows i, rows that lie C Np elements apart: stored like that every
    // instruction would touch 64 lines.  The wavefront's tile is therefore gathered in LDS (free after the
    // last barrier of the loop; each wavefront uses its own part, and a wavefront's LDS operations complete in
    // order) and leaves as row segments of 64 TJ bytes, 16 bytes per lane.
    {
        static_assert(TJ == 2, "a row of the wavefront's tile is 64 elements: eight 16-byte pieces");
        unsigned char* s_o = smem + wave * (32 * TI * PITCH);
#pragma unroll
        for (int ti = 0; ti < TI; ++ti)
#pragma unroll
            for (int tj = 0; tj < TJ; ++tj)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<uint2*>(s_o + (32 * ti + col) * PITCH + (32 * tj + 8 * g + 4 * hf) * 2) =
                        make_uint2(pack2(acc[tj][ti][4 * g], acc[tj][ti][4 * g + 1]), pack2(acc[tj][ti][4 * g + 2], acc[tj][ti][4 * g + 3]));
        bf16_t* xc = p.x + (size_t)ch * p.Np;
        const size_t xrow = (size_t)p.C * p.Np;
        const int pcj = lane & 7, j = j0 + wj * 32 * TJ + pcj * 8;
#pragma unroll
        for (int n = 0; n < 4 * TI; ++n) {
            const int row = 8 * n + (lane >> 3), i = i0 + wi * 32 * TI + row;
            const uint4 v = *reinterpret_cast<const uint4*>(s_o + row * PITCH + pcj * 16);
            if (i < p.N && j < p.Np) *reinterpret_cast<uint4*>(xc + (size_t)i * xrow + j) = v;
        }
    }
}

// ====================================================================================
// out[i][j][:] = g[i][j][:] * (LayerNorm_out(t[:, i, j]) W_o^T + b_o) (+ z[i][j][:]),
// g[i][j][:] = sigmoid(LayerNorm_in(z[i][j][:]) W_g^T + b_g).
// Block = 8 wavefronts, both folded weight matrices resident in LDS, each wavefront working through 32-token
// tiles (i, j0 .. j0 + 31); features x tokens on the matrix cores (the lane owns a token) for both GEMMs, so the
// gate meets the projected value in the same lane and register.  Results leave the accumulators as 8-byte pieces
// of 32 different tokens; the output tile [32 tokens][cz], one contiguous block of out, is gathered in the
// wavefront's own LDS area and stored 16 bytes per lane.
struct TmOutArgs {
    const bf16_t* x;         // [N][C][Np]
    const bf16_t* z;         // [N*N][cz]
    bf16_t* out;             // [N*N][cz]; may be z itself when residual
    int residual;
    int N, Np, C, cz;
    int wave_bytes;          // LDS area of a wavefront: 32 * (2 cz + 16)
    float eps;
    const bf16_t *wp, *wg;   // [cz][16 KC], [cz][16 KZ]
    const bf16_t *ext, *extg;  // [cz][8] each: the rows' extra contraction step
};

template <int KC, int KZ>
__global__ __launch_bounds__(512) void k_tm_out(TmOutArgs p) {
    constexpr int PC = KC * 32 + 16, PZ = KZ * 32 + 16;     // bytes per weight row in LDS (padded: conflict-free operand reads)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* s_wo = smem;                             // [cz][PC]
    unsigned char* s_wg = smem + (size_t)p.cz * PC;         // [cz][PZ]
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // (only this wavefront reads or writes its area; a wavefront's LDS operations complete in order)
    unsigned char* s_x = s_wg + (size_t)p.cz * PZ + (size_t)wave * p.wave_bytes;
    const int tpr = p.Np >> 5, tiles_m = p.N * tpr, n_ft = p.cz >> 5, nwaves = gridDim.x * 8;
    const int PO = 2 * p.cz + 16;                           // bytes per token row of the staged output tile
    int t = blockIdx.x * 8 + wave;

    // (a row's extra contraction step - see token_side - sits in the 16 bytes that pad it)
    for (int id = tid; id < p.cz * (2 * KC + 1); id += 512) {
        const int row = id / (2 * KC + 1), pc = id - row * (2 * KC + 1);
        const bf16_t* src = pc < 2 * KC ? p.wp + (size_t)row * (16 * KC) + pc * 8 : p.ext + (size_t)row * 8;
        *reinterpret_cast<uint4*>(s_wo + row * PC + pc * 16) = *reinterpret_cast<const uint4*>(src);
    }
    for (int id = tid; id < p.cz * (2 * KZ + 1); id += 512) {
        const int row = id / (2 * KZ + 1), pc = id - row * (2 * KZ + 1);
        const bf16_t* src = pc < 2 * KZ ? p.wg + (size_t)row * (16 * KZ) + pc * 8 : p.extg + (size_t)row * 8;
        *reinterpret_cast<uint4*>(s_wg + row * PZ + pc * 16) = *reinterpret_cast<const uint4*>(src);
    }
    __syncthreads();                                        // (the only barrier)

    for (; t < tiles_m; t += nwaves) {
        const int i = t / tpr, j0 = (t - i * tpr) * 32;
        Frag za[KZ], xa[KC];
        {
            const int j = j0 + col;
            const bf16_t* zp = p.z + ((size_t)i * p.N + (j < p.N ? j : 0)) * p.cz;
#pragma unroll
            for (int s = 0; s < KZ; ++s) {
                za[s].u = make_uint4(0, 0, 0, 0);
                if (16 * s + 8 * hf < p.cz) za[s].u = *reinterpret_cast<const uint4*>(zp + 16 * s + 8 * hf);
            }
            // t is [i][channel][j]: the eight channels of an operand fragment are eight 2-byte loads, each of
            // them 64 contiguous bytes across the half-wave (turning the tile in LDS instead, 16-byte loads and
            // 2-byte LDS reads, measured the same)
            const bf16_t* xp = p.x + (size_t)i * p.C * p.Np + j;
#pragma unroll
            for (int s = 0; s < KC; ++s) {
                xa[s].u = make_uint4(0, 0, 0, 0);
                if (16 * s + 8 * hf < p.C) {
                    const bf16_t* xc = xp + (size_t)(16 * s + 8 * hf) * p.Np;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        xa[s].w[e] = (uint32_t)xc[(size_t)(2 * e) * p.Np] | ((uint32_t)xc[(size_t)(2 * e + 1) * p.Np] << 16);
                }
            }
        }
        float mean_z, rstd_z, istd_z, mean, rstd, istd;
        token_stats<KZ>(za, p.cz, p.eps, mean_z, rstd_z, istd_z);
        token_stats<KC>(xa, p.C, p.eps, mean, rstd, istd);
        const Frag xe = token_side(mean, istd, hf), ze = token_side(mean_z, istd_z, hf);
        const float nrl = -kLog2e * rstd_z;                 // sigmoid(rstd_z t) = 1 / (1 + exp2(nrl t))

#pragma unroll
        for (int ft = 0; ft < KZ / 2; ++ft) {               // (unrolled: the residual below picks registers by ft)
            if (ft >= n_ft) break;
            f32x16 acc, accg;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = accg[v] = 0.f;
            const unsigned char* wrow = s_wo + (ft * 32 + col) * PC + hf * 16;
            const unsigned char* grow = s_wg + (ft * 32 + col) * PZ + hf * 16;
#pragma unroll
            for (int s = 0; s < KC; ++s) {
                Frag wf;
                wf.u = *reinterpret_cast<const uint4*>(wrow + 32 * s);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, xa[s].v, acc, 0, 0, 0);
            }
#pragma unroll
            for (int s = 0; s < KZ; ++s) {
                Frag gf;
                gf.u = *reinterpret_cast<const uint4*>(grow + 32 * s);
                accg = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gf.v, za[s].v, accg, 0, 0, 0);
            }
            {
                Frag wf, gf;                                // - mean S + C / rstd of either projection
                wf.u = *reinterpret_cast<const uint4*>(s_wo + (ft * 32 + col) * PC + 2 * KC * 16);
                gf.u = *reinterpret_cast<const uint4*>(s_wg + (ft * 32 + col) * PZ + 2 * KZ * 16);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, xe.v, acc, 0, 0, 0);
                accg = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gf.v, ze.v, accg, 0, 0, 0);
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int f0 = ft * 32 + 8 * g + 4 * hf;
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o[e] = acc[4 * g + e] * rstd * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(nrl * accg[4 * g + e]));
                if (p.residual) {
                    // z[token][f0 .. f0 + 3] is in the registers of the token's two lanes: channels 16 s + 8 h' + u of
                    // fragment s belong to half h'; the lane wants words 2 hf, 2 hf + 1 of fragment 2 ft + g / 2 of half
                    // g % 2, its own or the other half's (one exchange per fragment word serves both halves)
                    const int sz = 2 * ft + (g >> 1);        // (a constant: the loop over ft is unrolled)
                    uint32_t a0 = za[sz].w[0], b0 = za[sz].w[2], a1 = za[sz].w[1], b1 = za[sz].w[3];
                    merge_halves(a0, b0);
                    merge_halves(a1, b1);
                    const uint32_t r0 = (g & 1) ? b0 : a0, r1 = (g & 1) ? b1 : a1;
                    o[0] += lo_f32(r0); o[1] += hi_f32(r0); o[2] += lo_f32(r1); o[3] += hi_f32(r1);
                }
                *reinterpret_cast<uint2*>(s_x + col * PO + f0 * 2) = make_uint2(pack2(o[0], o[1]), pack2(o[2], o[3]));
            }
            __builtin_amdgcn_sched_barrier(0);              // (keeps the next feature tile's weight reads out of this one: registers)
        }
        // the tile is 32 cz contiguous elements of out (tokens j0 .. j0 + 31 of row i): 16 bytes per lane
        {
            const int ppr = p.cz >> 3;                      // 16-byte pieces per token
            unsigned char* ob = reinterpret_cast<unsigned char*>(p.out + ((size_t)i * p.N + j0) * p.cz);
#pragma unroll
            for (int n = 0; n < KZ; ++n) {
                const int id = lane + 64 * n, row = id / ppr, pc = id - row * ppr;
                if (id < 32 * ppr) {
                    const uint4 v = *reinterpret_cast<const uint4*>(s_x + row * PO + pc * 16);
                    if (j0 + row < p.N) *reinterpret_cast<uint4*>(ob + (size_t)id * 16) = v;
                }
            }
        }
    }
}

// ====================================================================================
struct TmWs {
    bf16_t *wp1, *wp3, *wp4, *ext1, *ext3, *ext4, *a, *b, *x;
    size_t total;
};

static int kc_for(int K) { return K <= 32 ? 2 : (K <= 64 ? 4 : 8); }

static TmWs tm_carve(int N, int cz, int c, void* base) {
    const int Np = round_up(N, 32), G = c / 32, n_pairs = 2 * G;
    const int Kp1 = 16 * kc_for(cz), Kp3 = 16 * kc_for(c);
    char* b = (char*)base;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* p = b + off;
        off += align256(bytes);
        return p;
    };
    TmWs w;
    w.wp1 = (bf16_t*)take((size_t)64 * n_pairs * Kp1 * 2);
    w.wp3 = (bf16_t*)take((size_t)cz * Kp3 * 2);
    w.wp4 = (bf16_t*)take((size_t)cz * Kp1 * 2);
    w.ext1 = (bf16_t*)take((size_t)64 * n_pairs * 8 * 2);
    w.ext3 = (bf16_t*)take((size_t)cz * 8 * 2);
    w.ext4 = (bf16_t*)take((size_t)cz * 8 * 2);
    const size_t plane = (size_t)c * N * Np * 2;
    w.a = (bf16_t*)take(plane);
    w.b = (bf16_t*)take(plane);
    w.x = (bf16_t*)take(plane);
    w.total = off;
    return w;
}

}  // namespace tm

bool trimul_supported(int dtype, int cz, int c) {
    return dtype == FF_BF16 && cz % 32 == 0 && c % 32 == 0 && cz >= 32 && c >= 32 && cz <= 128 && c <= 128;
}

size_t trimul_workspace(int N, int cz, int c) { return tm::tm_carve(N, cz, c, nullptr).total; }

ff_status trimul_run(const ff_trimul_desc& d, const ff_trimul_weights& w, const void* z, const float* mask, bool residual,
                     void* out, void* ws, hipStream_t st) {
    using namespace tm;
    const int N = d.n, cz = d.c_z, c = d.c, Np = round_up(N, 32), G = c / 32, n_pairs = 2 * G;
    const int kc1 = kc_for(cz), kc3 = kc_for(c);
    const TmWs m = tm_carve(N, cz, c, ws);
    {
        TmPrepArgs a{};
        a.w_ap = (const bf16_t*)w.w_ap; a.b_ap = (const bf16_t*)w.b_ap; a.w_ag = (const bf16_t*)w.w_ag; a.b_ag = (const bf16_t*)w.b_ag;
        a.w_bp = (const bf16_t*)w.w_bp; a.b_bp = (const bf16_t*)w.b_bp; a.w_bg = (const bf16_t*)w.w_bg; a.b_bg = (const bf16_t*)w.b_bg;
        a.w_g = (const bf16_t*)w.w_g; a.b_g = (const bf16_t*)w.b_g; a.ln_g = (const bf16_t*)w.ln_g; a.ln_b = (const bf16_t*)w.ln_b;
        a.w_o = (const bf16_t*)w.w_o; a.b_o = (const bf16_t*)w.b_o; a.lno_g = (const bf16_t*)w.lno_g; a.lno_b = (const bf16_t*)w.lno_b;
        a.wp1 = m.wp1; a.wp3 = m.wp3; a.wp4 = m.wp4; a.ext1 = m.ext1; a.ext3 = m.ext3; a.ext4 = m.ext4;
        a.cz = cz; a.c = c; a.G = G; a.n_pairs = n_pairs; a.Kp1 = 16 * kc1; a.Kp3 = 16 * kc3;
        const int rows = 64 * n_pairs + 2 * cz;
        Timed t(KK_TM_PREP, st);
        hipLaunchKernelGGL(k_tm_prep, dim3((rows + 3) / 4), dim3(256), 0, st, a);
    }
    {
        TmProjArgs a{};
        a.z = (const bf16_t*)z;
        a.sr = d.incoming ? 1 : N; a.sl = d.incoming ? N : 1;
        a.mask = mask; a.N = N; a.Np = Np; a.K = cz; a.C = c; a.cz = cz; a.G = G; a.n_pairs = n_pairs; a.eps = d.ln_eps;
        a.wp = m.wp1; a.ext = m.ext1; a.a = m.a; a.b = m.b;
        const int tiles_m = N * (Np / 32);
        int blocks = (tiles_m + 7) / 8;
        // Large inputs: one persistent block per compute unit with all weights in its LDS.  Small ones (fewer than
        // four token tiles per wavefront slot of the chip) split the pairs in two over blockIdx.y, so that two
        // blocks fit a compute unit: x is then read twice, the second time from L2 (N_res = 256: 28.7 -> 26.3 us,
        // 384: 57 -> 51 us; a split in four loses again, 30 and 58 us).
        const int split = (blocks < 4 * 256 && n_pairs % 2 == 0) ? 2 : 1;
        a.ppb = n_pairs / split;
        const int per_cu = split;
        if (blocks > compute_units() * per_cu) blocks = compute_units() * per_cu;
        const dim3 grid(blocks, split);
        // weights (with their extra step), one staged output half-tile [16][32] per wavefront
        auto smem = [&](int kc) { return (size_t)64 * a.ppb * (kc * 32 + 16) + (size_t)8 * 16 * 80; };
        hipError_t attr = hipSuccess;
        Timed t(KK_TM_PROJ, st);
#define FF_TM_PROJ(KCV)                                                                                          \
    do {                                                                                                         \
        static const hipError_t once = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tm_proj<KCV>),      \
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); \
        attr = once;                                                                                             \
        if (once == hipSuccess) hipLaunchKernelGGL((k_tm_proj<KCV>), grid, dim3(512), smem(KCV), st, a);         \
    } while (0)
        if (kc1 == 2) FF_TM_PROJ(2);
        else if (kc1 == 4) FF_TM_PROJ(4);
        else FF_TM_PROJ(8);
#undef FF_TM_PROJ
        if (attr != hipSuccess) return fail(FF_EHIP, "k_tm_proj: dynamic LDS limit: %s", hipGetErrorString(attr));
    }
    {
        TmMulArgs a{};
        a.a = m.a; a.b = m.b; a.x = m.x; a.N = N; a.Np = Np; a.C = c;
        hipError_t attr = hipSuccess;
        Timed t(KK_TM_MUL, st);
#define FF_TM_MUL(WI, WJ, TI, TJ)                                                                                \
    do {                                                                                                         \
        using Sh = tm::MulShape<WI, WJ, TI, TJ>;                                                                 \
        static const hipError_t once = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tm_mul<WI, WJ, TI, TJ>), \
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)Sh::SMEM); \
        attr = once;                                                                                             \
        a.tiles_i = (N + Sh::BI - 1) / Sh::BI;                                                                   \
        a.tiles_j = (N + Sh::BJ - 1) / Sh::BJ;                                                                   \
        const int blocks = 8 * ((c + 7) / 8) * a.tiles_i * a.tiles_j;                                            \
        if (once == hipSuccess) hipLaunchKernelGGL((k_tm_mul<WI, WJ, TI, TJ>), dim3(blocks), dim3(Sh::NT), Sh::SMEM, st, a); \
    } while (0)
        // 256 x 256 block tiles once they fill the chip several times over (c channels x (N / 256)^2 blocks, one per CU)
        if ((int64_t)c * ((N + 255) / 256) * ((N + 255) / 256) >= 4 * compute_units() && N % 256 == 0) FF_TM_MUL(2, 4, 4, 2);
        else FF_TM_MUL(2, 2, 2, 2);
#undef FF_TM_MUL
        if (attr != hipSuccess) return fail(FF_EHIP, "k_tm_mul: dynamic LDS limit: %s", hipGetErrorString(attr));
    }
    {
        TmOutArgs a{};
        a.x = m.x; a.z = (const bf16_t*)z; a.out = (bf16_t*)out; a.residual = residual ? 1 : 0;
        a.N = N; a.Np = Np; a.C = c; a.cz = cz; a.eps = d.ln_eps;
        a.wp = m.wp3; a.wg = m.wp4; a.ext = m.ext3; a.extg = m.ext4;
        const int tiles_m = N * (Np / 32);
        int blocks = (tiles_m + 7) / 8;
        if (blocks > compute_units()) blocks = compute_units();     // one block of eight wavefronts per compute unit
        const dim3 grid(blocks);
        a.wave_bytes = 32 * (2 * cz + 16);
        const size_t smem = (size_t)cz * (kc3 * 32 + 16) + (size_t)cz * (kc1 * 32 + 16) + (size_t)8 * a.wave_bytes;
        hipError_t attr = hipSuccess;
        Timed t(KK_TM_OUT, st);
#define FF_TM_OUT(KCV, KZV)                                                                                          \
    do {                                                                                                             \
        static const hipError_t once = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tm_out<KCV, KZV>),      \
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); \
        attr = once;                                                                                                 \
        if (once == hipSuccess) hipLaunchKernelGGL((k_tm_out<KCV, KZV>), grid, dim3(512), smem, st, a);             \
    } while (0)
#define FF_TM_OUT_Z(KCV)              \
    do {                              \
        if (kc1 == 2) FF_TM_OUT(KCV, 2);      \
        else if (kc1 == 4) FF_TM_OUT(KCV, 4); \
        else FF_TM_OUT(KCV, 8);               \
    } while (0)
        if (kc3 == 2) FF_TM_OUT_Z(2);
        else if (kc3 == 4) FF_TM_OUT_Z(4);
        else FF_TM_OUT_Z(8);
#undef FF_TM_OUT_Z
#undef FF_TM_OUT
        if (attr != hipSuccess) return fail(FF_EHIP, "k_tm_out: dynamic LDS limit: %s", hipGetErrorString(attr));
    }
    return check_launch("triangle multiplication");
}

}  // namespace ff
