// Global column attention of the extra-MSA stack (FastFold Table 1: N_extra_seq 1024 / 5120; Section 6.2 lists
// the extra MSA among the optional modules; the algorithm is AlphaFold's published MSA column global
// self-attention), bf16, gfx950.  Per residue column i, with mn = LayerNorm(m):
//   qbar[i] = mean over unmasked s of mn[s,i];  q[i,h] = (W_q qbar[i])[h] / sqrt(d);  k[s,i] = W_k mn[s,i];
//   v[s,i] = W_v mn[s,i] (one shared head);  P[i,h,:] = softmax_s(q[i,h] . k[s,i]) over unmasked s;
//   o[i,h] = sum_s P[i,h,s] v[s,i];  out[s,i] = W_o (sigmoid(W_g mn[s,i] + b_g) * o[i]) + b_o
//
// The module is linear in N_seq and moves far more bytes than it computes: two reads of m and one write of
// out bound it (HBM).  Three launches:
//   (prep_row)     the LayerNorm gain folded into the weights (W' = bf16(W * gamma), C = W beta (+ bias)), W_o in the
//                  operand order of the last contraction and, for the gate rows, the row sums of W' and the
//                  offsets C as bfloat16 pairs (one more contraction step of the gate GEMM): what the second and
//                  third launch need of it is written by the last blocks of the first launch, one wavefront per
//                  row; the key / value blocks fold their own [W_q | W_k | W_v] on their way into LDS
//   k_gca_kv       one block per (32 residues, group of sequences), its four wavefronts each a range of consecutive
//                  sequences: a tile = the 32 c contiguous elements of one sequence's residues, asked for as whole
//                  lines and turned into operand fragments through LDS, normalised (masked tokens as zeros) and
//                  contracted with W_q' (tokens x features, never cleared between sequences: the accumulator IS the
//                  sum over the sequences, the query average's numerator) and with W_k' | W_v' (features x tokens:
//                  k, v of a token leave as bf16, four sequences at a time through LDS so that
//                  kv[residue][sequence] is written in whole lines; the mask goes along as one byte per token,
//                  by column); partial query sums and counts go to the workspace
//   k_gca_softmax  one block per column, a thread per sequence with all heads in registers: q from the partial
//                  sums, one sweep over k and v (a reference per thread and head that follows the maximum lazily,
//                  exponentials, denominators, weighted sums of v; the next sequences' k, v are on their way
//                  meanwhile), o[i] normalised
//   k_gca_out      a wavefront keeps one tile of 32 residues and walks over the sequences (o[i] read once): gate
//                  GEMM on the tokens as they are (LayerNorm's mean and scale enter through the extra contraction
//                  step and the factor of the exponential), sigmoid, times o[i] (the gated tile is already the B
//                  operand of the output GEMM because W_o was stored in the matching order), output GEMM with
//                  b_o as one more step, the output tile through LDS
// Operand layouts of v_mfma_f32_32x32x16_bf16 as in ff_trimul.hip.
#include "ff_common.h"

namespace ff {
namespace gca {

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
__device__ __forceinline__ float sigmoid(float t) {
    return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-t * kLog2e));
}
__device__ __forceinline__ float pick(const float4& q, int e) { return e == 0 ? q.x : (e == 1 ? q.y : (e == 2 ? q.z : q.w)); }

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Blocks per residue tile of k_gca_kv (four wavefronts each, every wavefront a range of consecutive sequences): also
// the number of partial query sums per residue that k_gca_softmax adds up.  Three blocks per compute unit at 5120
// sequences x 384 residues (as many as its LDS lets be resident), at least eight sequences per wavefront (more
// groups: 5120 sequences 79 -> 86 us with 80, 95 us with 128; 1024 sequences unchanged with 64).
static int kv_groups(int n_seq) {
    int g = n_seq / 32;
    return g < 1 ? 1 : (g > 64 ? 64 : g);
}
// A tile (32 tokens of c channels, contiguous in m) is asked for as whole lines: lane l of request j asks for
// the 16-byte piece 64 j + l of the tile (asked for in the operand layout - lane = token, 16 bytes of its 2 c -
// every request would touch 32 lines for a quarter of each, which holds the reads of m near 3.7 TB/s).  The
// pieces reach the operand layout through the wavefront's own LDS area [32 tokens][2 c + 16 bytes] (only this
// wavefront touches it; its LDS operations complete in order).  Tokens past the end of the residues repeat the
// last valid one.
template <int KC>
struct TileFetch {
    int goff[KC];      // element offset of the lane's piece of request j within the tile
    int woff[KC];      // byte offset of that piece in the LDS area, or -1: no such piece (c < 16 KC)
    __device__ __forceinline__ void init(int c, int lane, int valid_tokens) {
        const int ppt = c >> 3, pitch = 2 * c + 16;
#pragma unroll
        for (int j = 0; j < KC; ++j) {
            const int P = 64 * j + lane;
            const bool act = P < 32 * ppt;
            const int t = act ? P / ppt : 0, w = act ? P - t * ppt : 0;
            const int tt = t < valid_tokens ? t : valid_tokens - 1;
            goff[j] = tt * c + 8 * w;
            woff[j] = act ? t * pitch + 16 * w : -1;
        }
    }
    __device__ __forceinline__ void fetch(Frag (&raw)[KC], const bf16_t* tile) const {
#pragma unroll
        for (int j = 0; j < KC; ++j) raw[j].u = *reinterpret_cast<const uint4*>(tile + goff[j]);
    }
    // raw pieces -> xa: eight channels 16 q + 8 hf .. of token col per step q (zeros beyond c)
    __device__ __forceinline__ void to_operands(const Frag (&raw)[KC], Frag (&xa)[KC], unsigned char* area, int c, int col, int hf) const {
        const int pitch = 2 * c + 16;
#pragma unroll
        for (int j = 0; j < KC; ++j) {
            uint32_t a = raw[j].w[0], b = raw[j].w[1], cc = raw[j].w[2], d = raw[j].w[3];
            asm volatile("" : "+v"(a), "+v"(b), "+v"(cc), "+v"(d));   // (keeps the pieces in registers from load to store)
            if (woff[j] >= 0) *reinterpret_cast<uint4*>(area + woff[j]) = make_uint4(a, b, cc, d);
        }
#pragma unroll
        for (int q = 0; q < KC; ++q) {
            xa[q].u = make_uint4(0, 0, 0, 0);
            if (16 * q + 8 * hf < c) xa[q].u = *reinterpret_cast<const uint4*>(area + col * pitch + (2 * q + hf) * 16);
        }
    }
};

// Statistics of the lane's token (which stays as it is): mean, 1 / sqrt(variance + eps) and sqrt(variance + eps).
// Sum and sum of squares come from the packed pairs directly (a two-element dot product with float32
// accumulation per pair: the squares of bfloat16 values are exact in float32), the variance as
// E[x^2] - mean^2: its rounding error is about 2^-22 (1 + mean^2 / variance), far below what the bfloat16
// tokens themselves carry.
template <int KC>
__device__ __forceinline__ void statistics(const Frag (&xa)[KC], int K, float eps, float& mean, float& rstd, float& istd) {
    const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
    float sum = 0.f, sq = 0.f;
#pragma unroll
    for (int s = 0; s < KC; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {                    // (channels beyond K are zero)
            const bf16x2 w = __builtin_bit_cast(bf16x2, xa[s].w[i]);
            sum = __builtin_amdgcn_fdot2_f32_bf16(w, ones, sum, false);
            sq = __builtin_amdgcn_fdot2_f32_bf16(w, w, sq, false);
        }
    sum += __shfl_xor(sum, 32, 64);
    sq += __shfl_xor(sq, 32, 64);
    const float rk = 1.f / (float)K;
    mean = sum * rk;
    const float var = fmaxf(sq * rk - mean * mean, 0.f);
    const float ve = var + eps;
    rstd = rsqrtf(ve);
    istd = ve * rstd;                                // sqrt(variance + eps)
}
// Normalised operand fragments of the lane's token: xn = bf16((x - mean) * rstd) (the LayerNorm gain and
// offset live in the folded weights), or zeros if !keep.
template <int KC>
__device__ __forceinline__ void normalise(Frag (&xa)[KC], int K, int hf, float eps, bool keep) {
    float mean, rstd, istd;
    statistics<KC>(xa, K, eps, mean, rstd, istd);
    if (!keep) rstd = 0.f;
    const float off = -mean * rstd;
#pragma unroll
    for (int s = 0; s < KC; ++s) {
        const bool in = 16 * s + 8 * hf < K;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a = lo_f32(xa[s].w[i]) * rstd + off, b = hi_f32(xa[s].w[i]) * rstd + off;
            xa[s].w[i] = in ? pack2(a, b) : 0u;
        }
    }
}
// v = hi + lo with hi, lo bfloat16 (hi the nearest, lo the nearest to the rest): 16 significant bits in two operand slots
__device__ __forceinline__ void split2(float v, float& hi, float& lo) {
    hi = __uint_as_float(pack2(0.f, v) & 0xffff0000u);
    lo = v - hi;
}

// ====================================================================================
struct PrepArgs {
    const bf16_t *w_q, *w_k, *w_v, *w_g, *b_g, *w_o, *b_o, *ln_g, *ln_b;
    bf16_t *wq, *wkv, *wg, *wo;       // [Hd][Kp], [32][Kp], [Hd][Kp], [c][Hd] (operand order)
    float *Cq, *Ckv, *Co;             // [Hd], [32], [c]
    bf16_t* gext;                     // [Hd][8]: the gate rows' extra contraction step (see k_gca_out)
    int c, Hd, d, Kp;
};

// One wavefront per row n of the three folded matrices (rows [0, Hd): W_q', [Hd, Hd + 32): W_k' | W_v',
// [Hd + 32, 2 Hd + 32): W_g'); the c rows after them copy W_o and b_o.  Run by the last blocks of the k_gca_kv launch
// for what the later kernels need (C_q, W_g', W_o: the key / value blocks fold their own weights).
__device__ __forceinline__ void prep_row(const PrepArgs& a, int n, int lane) {
    const int rows_fold = 2 * a.Hd + 32;
    if (n < rows_fold) {
        const bf16_t* wrow = nullptr;
        float bias = 0.f;
        bf16_t* dst;
        float* Cd = nullptr;
        bf16_t* ext = nullptr;
        if (n < a.Hd) {
            wrow = a.w_q + (size_t)n * a.c; dst = a.wq + (size_t)n * a.Kp; Cd = a.Cq + n;
        } else if (n < a.Hd + 32) {
            const int r = n - a.Hd;               // rows 0 .. d-1: keys, 16 .. 16+d-1: values, others zero
            if (r < a.d) wrow = a.w_k + (size_t)r * a.c;
            else if (r >= 16 && r < 16 + a.d) wrow = a.w_v + (size_t)(r - 16) * a.c;
            dst = a.wkv + (size_t)r * a.Kp; Cd = a.Ckv + r;
        } else {
            const int f = n - a.Hd - 32;
            wrow = a.w_g + (size_t)f * a.c; bias = bf16_to_f32(a.b_g[f]);
            dst = a.wg + (size_t)f * a.Kp; ext = a.gext + (size_t)f * 8;
        }
        float cst = 0.f, rowsum = 0.f;
        for (int k = lane; k < a.Kp; k += 64) {
            float r = 0.f;
            if (wrow && k < a.c) {
                const float w = bf16_to_f32(wrow[k]);
                r = w * bf16_to_f32(a.ln_g[k]);
                cst += w * bf16_to_f32(a.ln_b[k]);
            }
            const bf16_t rb = f32_to_bf16(r);
            dst[k] = rb;
            rowsum += bf16_to_f32(rb);                // of the rounded entries: what the matrix unit multiplies with
        }
        cst = wave_sum(cst);
        rowsum = wave_sum(rowsum);
        if (lane == 0) {
            if (Cd) *Cd = cst + bias;
            if (ext) {
                // slots of the extra step: S S_ S' C C_ C' 0 0 with S = hi(rowsum), S' = lo(rowsum), C likewise; the
                // token side holds -mean and 1 / rstd split the same way (hi, lo, hi): the three largest of the four products
                const float C = cst + bias;
                const bf16_t s_hi = f32_to_bf16(rowsum), s_lo = f32_to_bf16(rowsum - bf16_to_f32(s_hi));
                const bf16_t c_hi = f32_to_bf16(C), c_lo = f32_to_bf16(C - bf16_to_f32(c_hi));
                ext[0] = s_hi; ext[1] = s_hi; ext[2] = s_lo; ext[3] = c_hi; ext[4] = c_hi; ext[5] = c_lo;
                ext[6] = f32_to_bf16(0.f); ext[7] = f32_to_bf16(0.f);
            }
        }
        return;
    }
    const int co = n - rows_fold;
    if (co >= a.c) return;
    // Slot u of half hf of contraction step (T, j) of the output GEMM holds gated feature
    // 32T + 16j + 4hf + (u < 4 ? u : u + 4): that is where the gate GEMM's accumulator leaves it.
    for (int x = lane; x < a.Hd; x += 64) {
        const int T = x >> 5, j = (x >> 4) & 1, hf = (x >> 3) & 1, u = x & 7;
        const int f = 32 * T + 16 * j + 4 * hf + (u < 4 ? u : u + 4);
        a.wo[(size_t)co * a.Hd + x] = a.w_o[(size_t)co * a.Hd + f];
    }
    if (lane == 0) a.Co[co] = bf16_to_f32(a.b_o[co]);
}

// ====================================================================================
struct KvArgs {
    const bf16_t* m;         // [S][R][c]
    const float* mask;       // [S][R] or NULL
    int S, R, c, Hd, d, groups;
    float eps;
    const bf16_t *w_q, *w_k, *w_v, *ln_g, *ln_b;   // the caller's weights: [Hd][c], [d][c], [d][c], [c], [c]
    PrepArgs prep;           // for the blocks behind the kv_blocks key / value blocks
    int kv_blocks;
    bf16_t* kv;              // [R][S][2d]: k then v of a token
    unsigned char* keepT;    // [R][S]: 1 = the token takes part (the mask, by column); written only if mask != NULL
    float* qpart;            // [R][groups][Hd]
    float* cntpart;          // [R][groups]
};

// Block = one residue tile (32 residues) and one group of sequences; its four wavefronts walk over the sequences
// s = 4 group + wave, + 4 groups, ...: a tile is 32 c contiguous elements of m (the tokens of the next sequence are
// requested before this one is worked on), and k | v of its 32 tokens 32 x 2d contiguous elements of kv.  The query
// sums need no arithmetic of their own: the accumulator of the tokens x features contraction with W_q' simply is
// not cleared between sequences (lane = feature, register = residue).  At the end the block adds the four
// wavefronts' sums in LDS and writes one partial sum per residue and feature.
template <int KC, int D, int NQT>      // NQT = H d / 32: 32-feature tiles of the query projection
__global__ __launch_bounds__(256) void k_gca_kv(KvArgs p) {
    constexpr int PITCH = KC * 32 + 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* s_wq = smem;                                  // [Hd][PITCH]
    unsigned char* s_wkv = smem + (size_t)p.Hd * PITCH;          // [32][PITCH]
    float* s_red = reinterpret_cast<float*>(smem);               // [4][32][Hd + 1]: the wavefronts' query sums and counts, after the loop
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if ((int)blockIdx.x >= p.kv_blocks) {
        // what the softmax and the output kernel need of the weights (rows of W_q' for C_q, W_g', W_o): it depends
        // on nothing, so it rides in this launch instead of one of its own
        const int n = ((int)blockIdx.x - p.kv_blocks) * 4 + wave;
        prep_row(p.prep, n < p.Hd ? n : n + 32, lane);
        return;
    }
    const int tpr = (p.R + 31) >> 5;
    const int rt = blockIdx.x % tpr, grp = blockIdx.x / tpr;
    const int per = (p.S + 4 * p.groups - 1) / (4 * p.groups);       // consecutive sequences per wavefront
    const int s_lo = (4 * grp + wave) * per, s_hi = s_lo + per < p.S ? s_lo + per : p.S;
    const int i_raw = rt * 32 + col;
    const bool valid = i_raw < p.R;
    const int i = valid ? i_raw : p.R - 1;
    constexpr int REC = 4 * D, BP = 4 * REC + 16;  // bytes of a token's k | v; bytes per residue row of the batch in LDS
    // k | v of four consecutive sequences are gathered per residue in the wavefront's own LDS area and leave as whole
    // 128-byte (d = 8) runs of kv[residue][sequence]: stored straight from the accumulators they would be 8-byte
    // pieces of 32 different lines per instruction (only this wavefront touches the area; its LDS operations
    // complete in order)
    unsigned char* s_b = smem + (size_t)(p.Hd + 32) * PITCH + (size_t)wave * 32 * BP;
    // the wavefront's area for the incoming tile [32 tokens][2 c + 16]
    unsigned char* s_in = smem + (size_t)(p.Hd + 32) * PITCH + (size_t)4 * 32 * BP + (size_t)wave * 32 * (2 * p.c + 16);
    // ... and for the keep flags of the batch [32 residues][4 sequences]
    unsigned char* s_keep = smem + (size_t)(p.Hd + 32) * PITCH + (size_t)4 * 32 * BP + (size_t)4 * 32 * (2 * p.c + 16) + wave * 128;
    TileFetch<KC> tf;
    tf.init(p.c, lane, p.R - rt * 32 < 32 ? p.R - rt * 32 : 32);

    // the first tokens are requested before the weights are copied: both are on their way together
    Frag xn[KC];
    float mkn = 1.f;
    {
        const int s0 = s_lo < p.S ? s_lo : 0;
        tf.fetch(xn, p.m + ((size_t)s0 * p.R + rt * 32) * p.c);
        if (p.mask) mkn = p.mask[(size_t)s0 * p.R + i];
    }
    // The block folds the LayerNorm gain into its own copy of [W_q | W_k | W_v] (W' = bf16(W gamma), eight channels
    // per thread and step; rows Hd .. Hd + 31: keys in 0 .. d - 1, values in 16 .. 16 + d - 1, the others zero) and
    // forms the key / value offsets C = W beta from the pieces' partial sums in a fixed order.
    float* s_part = reinterpret_cast<float*>(s_keep + (4 - wave) * 128);      // [32][2 KC] (behind the four wavefronts' flag areas)
    float* s_ckv = s_part + 32 * 2 * KC;                                        // [32]
    for (int id = tid; id < (p.Hd + 32) * 2 * KC; id += 256) {
        const int row = id / (2 * KC), pc = id - row * (2 * KC), r = row - p.Hd;
        const bf16_t* src = row < p.Hd ? p.w_q + (size_t)row * p.c
                                       : (r < p.d ? p.w_k + (size_t)r * p.c : ((r >= 16 && r < 16 + p.d) ? p.w_v + (size_t)(r - 16) * p.c : nullptr));
        uint4 out = make_uint4(0, 0, 0, 0);
        float cst = 0.f;
        if (src && 8 * pc < p.c) {
            const uint4 w8 = *reinterpret_cast<const uint4*>(src + 8 * pc);
            const uint4 g8 = *reinterpret_cast<const uint4*>(p.ln_g + 8 * pc);
            const uint4 b8 = *reinterpret_cast<const uint4*>(p.ln_b + 8 * pc);
            const uint32_t ww[4] = {w8.x, w8.y, w8.z, w8.w}, gw[4] = {g8.x, g8.y, g8.z, g8.w}, bw[4] = {b8.x, b8.y, b8.z, b8.w};
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o[e] = pack2(lo_f32(ww[e]) * lo_f32(gw[e]), hi_f32(ww[e]) * hi_f32(gw[e]));
                cst += lo_f32(ww[e]) * lo_f32(bw[e]) + hi_f32(ww[e]) * hi_f32(bw[e]);
            }
            out = make_uint4(o[0], o[1], o[2], o[3]);
        }
        *reinterpret_cast<uint4*>(smem + row * PITCH + pc * 16) = out;
        if (r >= 0) s_part[r * 2 * KC + pc] = cst;
    }
    __syncthreads();
    if (tid < 32) {
        float t = 0.f;
#pragma unroll
        for (int pc = 0; pc < 2 * KC; ++pc) t += s_part[tid * 2 * KC + pc];
        s_ckv[tid] = t;
    }
    __syncthreads();

    f32x16 qacc[NQT];                            // tokens x features, summed over the wavefront's sequences
#pragma unroll
    for (int T = 0; T < NQT; ++T)
#pragma unroll
        for (int v = 0; v < 16; ++v) qacc[T][v] = 0.f;
    float cnt = 0.f;                             // unmasked sequences of the lane's residue
    // offsets of the lane's key / value rows (read once)
    const float4 ckv0 = *reinterpret_cast<const float4*>(s_ckv + 4 * hf), ckv1 = *reinterpret_cast<const float4*>(s_ckv + 8 + 4 * hf);
    const float4 ckv2 = *reinterpret_cast<const float4*>(s_ckv + 16 + 4 * hf), ckv3 = *reinterpret_cast<const float4*>(s_ckv + 24 + 4 * hf);

    for (int s = s_lo; s < s_hi; ++s) {
        Frag xa[KC];
        tf.to_operands(xn, xa, s_in, p.c, col, hf);
        const bool keep = valid && mkn != 0.f;
        {
            const int sn = s + 1 < s_hi ? s + 1 : s;               // (the last round asks for its own tokens again)
            tf.fetch(xn, p.m + ((size_t)sn * p.R + rt * 32) * p.c);
            if (p.mask) mkn = p.mask[(size_t)sn * p.R + i];
        }
        normalise<KC>(xa, p.c, hf, p.eps, keep);
        cnt += keep ? 1.f : 0.f;
#pragma unroll
        for (int T = 0; T < NQT; ++T) {
#pragma unroll
            for (int q = 0; q < KC; ++q) {
                Frag wf;
                wf.u = *reinterpret_cast<const uint4*>(s_wq + (32 * T + col) * PITCH + (2 * q + hf) * 16);
                qacc[T] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[q].v, wf.v, qacc[T], 0, 0, 0);
            }
        }
        // keys and values: features x tokens, the lane owns a token; rows 0 .. D-1 keys, 16 .. 16+D-1 values
        {
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int q = 0; q < KC; ++q) {
                Frag wf;
                wf.u = *reinterpret_cast<const uint4*>(s_wkv + col * PITCH + (2 * q + hf) * 16);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, xa[q].v, acc, 0, 0, 0);
            }
            const int b = (s - s_lo) & 3;
            const bool last = s + 1 == s_hi;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int row = 8 * g + 4 * hf;                  // rows row .. row + 3 of the tile
                const bool is_v = row >= 16;
                const int e0 = is_v ? row - 16 : row;            // first key / value channel of the group
                if (e0 < D) {
                    const float4 c4 = g == 0 ? ckv0 : (g == 1 ? ckv1 : (g == 2 ? ckv2 : ckv3));
                    *reinterpret_cast<uint2*>(s_b + col * BP + b * REC + ((is_v ? D : 0) + e0) * 2) =
                        make_uint2(pack2(acc[4 * g] + c4.x, acc[4 * g + 1] + c4.y), pack2(acc[4 * g + 2] + c4.z, acc[4 * g + 3] + c4.w));
                }
            }
            if (p.mask && hf == 0) s_keep[col * 4 + b] = keep ? 1 : 0;
            if (b == 3 || last) {
                // nb sequences s - b .. s of 32 residues: 16-byte pieces, a residue's nb records are contiguous in kv
                const int ppr = (b + 1) * (REC / 16);            // pieces per residue
                unsigned char* kvb = reinterpret_cast<unsigned char*>(p.kv) + ((size_t)(rt * 32) * p.S + (s - b)) * REC;
                for (int id = lane; id < 32 * ppr; id += 64) {
                    const int r = id / ppr, pc = id - r * ppr;
                    const uint4 v = *reinterpret_cast<const uint4*>(s_b + r * BP + pc * 16);
                    if (rt * 32 + r < p.R) *reinterpret_cast<uint4*>(kvb + (size_t)r * p.S * REC + pc * 16) = v;
                }
                if (p.mask) {
                    const int nb = b + 1;
                    for (int id = lane; id < 32 * nb; id += 64) {
                        const int r = id / nb, j = id - r * nb;
                        if (rt * 32 + r < p.R) p.keepT[(size_t)(rt * 32 + r) * p.S + (s - b) + j] = s_keep[r * 4 + j];
                    }
                }
            }
        }
    }
    // the block's partial sums: wavefront w leaves [residue][feature] (and the count in column Hd) in its part of LDS
    // (the sums take the place of the weights and the k | v batches, which every wavefront is done with by now)
    __syncthreads();
    const int RP = p.Hd + 1;
    float* red = s_red + (size_t)wave * 32 * RP;
#pragma unroll
    for (int T = 0; T < NQT; ++T)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[(8 * (v >> 2) + 4 * hf + (v & 3)) * RP + 32 * T + col] = qacc[T][v];
    if (hf == 0) red[col * RP + p.Hd] = cnt;
    __syncthreads();
    for (int id = tid; id < 32 * RP; id += 256) {
        const int r = id / RP, f = id - r * RP;
        const float t = s_red[id] + s_red[32 * RP + id] + s_red[2 * 32 * RP + id] + s_red[3 * 32 * RP + id];
        const int ir = rt * 32 + r;
        if (ir < p.R) {
            if (f < p.Hd) p.qpart[((size_t)ir * p.groups + grp) * p.Hd + f] = t;
            else p.cntpart[(size_t)ir * p.groups + grp] = t;
        }
    }
}

// ====================================================================================
struct SmArgs {
    const bf16_t* kv;        // [R][S][2d]
    const unsigned char* keepT;   // [R][S] (1 = takes part) or NULL: every token takes part
    const float *qpart, *cntpart, *Cq;
    float* o;                // [R][Hd]
    int S, R, Hd, H, nchunk;
    float qscale;            // log2(e) / sqrt(d)
};

// Sums (or maxima) of N per-lane values over the 64 lanes, N a power of two up to 64.  Instead of N butterflies
// of six exchanges each, every exchange step halves the number of values a lane still carries (the lane keeps
// one half of its values and hands the other half to its partner), N - 1 exchanges in all (plus the plain
// butterfly over the remaining steps when N < 64).  Afterwards v[0] of lane l is the result for value index
// l >> log2(64 / N).  Exchanges go through the LDS crossbar, which is what bounds this kernel otherwise.
template <int N, int n, bool MAX>
__device__ __forceinline__ void wave_reduce_scatter_step(float (&v)[N], int lane, int o) {
    if constexpr (n > 1) {
        const bool up = (lane & o) != 0;
#pragma unroll
        for (int f = 0; f < n / 2; ++f) {
            const float send = up ? v[f] : v[f + n / 2];
            const float keep = up ? v[f + n / 2] : v[f];
            const float recv = __shfl_xor(send, o, 64);
            v[f] = MAX ? fmaxf(keep, recv) : keep + recv;
        }
        wave_reduce_scatter_step<N, n / 2, MAX>(v, lane, o >> 1);
    } else {
        for (; o > 0; o >>= 1) {
            const float recv = __shfl_xor(v[0], o, 64);
            v[0] = MAX ? fmaxf(v[0], recv) : v[0] + recv;
        }
    }
}
template <int N, bool MAX>
__device__ __forceinline__ void wave_reduce_scatter(float (&v)[N], int lane) {
    static_assert(N >= 1 && N <= 64 && (N & (N - 1)) == 0, "a power of two up to 64");
    wave_reduce_scatter_step<N, N, MAX>(v, lane, 32);
}

// Block = one column, NT threads; a thread takes the sequences s = tid, tid + NT, ... and holds all H heads:
// k and v of a sequence are read ONCE (one sweep: every thread keeps a reference per head - at most kSlack below
// the largest logit it has met - and rescales its own partial sums when the reference moves, so no pass over the
// logits precedes the exponentials), the H
// denominators and H x D weighted sums live in registers (hence H and D as template parameters), and the
// block combines the threads' partial results, each brought to the common maximum, through shuffles and LDS.
template <int H, int D, int NT>
__global__ __launch_bounds__(NT) void k_gca_softmax(SmArgs p) {
    constexpr int HD = H * D, NW = NT / 64, PW = HD + 2 * H;
    constexpr float kSlack = 8.f;                 // (logits are in units of log 2)
    __shared__ float s_q[HD];
    __shared__ float s_red[NW * PW];              // per wavefront: weighted sums, denominators, maxima
    __shared__ __attribute__((aligned(16))) float s_part[4 * NT];   // the threads' partial query sums
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, i = blockIdx.x;
    // U sequences at a time: their loads (k, v and the keep flag, none of which depends on another) are all in
    // flight together; k and v of a masked sequence exist (finite) and are simply not used.  The first batch is
    // asked for here, before the partial sums: the two round trips to memory overlap.
    constexpr int U = 64 / (2 * D);
    static_assert(D % 8 == 0, "k and v of a token are read in 16-byte pieces");
    const bf16_t* kvc = p.kv + (size_t)i * p.S * (2 * D);
    // (the next U sequences are asked for before this batch is worked on; sequences past the end ask for the last
    // one again and count as masked; nothing is done with a loaded value before its batch's turn, so that no wait
    // for it precedes the work on the batch before)
    uint4 kvn[U][2 * D / 8];
    unsigned char keepn[U];
    const unsigned char* keepc = p.keepT ? p.keepT + (size_t)i * p.S : nullptr;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int s = tid + u * NT, sc = s < p.S ? s : p.S - 1;
        const uint4* kp = reinterpret_cast<const uint4*>(kvc + (size_t)sc * (2 * D));
#pragma unroll
        for (int e8 = 0; e8 < 2 * D / 8; ++e8) kvn[u][e8] = kp[e8];
        keepn[u] = 1;
        if (keepc) keepn[u] = keepc[sc];
    }
    // partial counts and query sums of the column's chunks: spread over the lanes / the threads so that the loads
    // do not queue behind each other (a column of 5120 sequences has 20 chunks)
    float cnt = 0.f;
    for (int j = lane; j < p.nchunk; j += 64) cnt += p.cntpart[(size_t)i * p.nchunk + j];
    cnt = wave_sum(cnt);
    if (cnt == 0.f) {                              // no unmasked sequence: zero context (uniform over the block)
        if (tid < HD) p.o[(size_t)i * HD + tid] = 0.f;
        return;
    }
    {
        // the column's partial query sums [groups][HD], contiguous: 16 bytes per thread and step, four steps'
        // loads in flight together; a thread always meets the same four features, threads tid % (HD / 4) apart
        // share them and are added up through LDS
        constexpr int QP = HD / 4, G = NT / QP;    // 16-byte pieces per partial sum; threads per piece
        const float4* qp = reinterpret_cast<const float4*>(p.qpart + (size_t)i * p.nchunk * HD);
        const int n = p.nchunk * QP;
        float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int id = tid; id < n; id += 4 * NT) {
            float4 t0 = make_float4(0.f, 0.f, 0.f, 0.f), t1 = t0, t2 = t0, t3 = t0;
            t0 = qp[id];
            if (id + NT < n) t1 = qp[id + NT];
            if (id + 2 * NT < n) t2 = qp[id + 2 * NT];
            if (id + 3 * NT < n) t3 = qp[id + 3 * NT];
            q.x += (t0.x + t1.x) + (t2.x + t3.x); q.y += (t0.y + t1.y) + (t2.y + t3.y);
            q.z += (t0.z + t1.z) + (t2.z + t3.z); q.w += (t0.w + t1.w) + (t2.w + t3.w);
        }
        static_assert(NT % QP == 0, "whole groups of threads per piece");
        float4* s_q4 = reinterpret_cast<float4*>(s_part);
        s_q4[tid] = q;                              // [G][QP] pieces
        __syncthreads();
        if (tid < HD) {
            float t = 0.f;
#pragma unroll
            for (int gg = 0; gg < G; ++gg) t += s_part[(gg * QP + (tid >> 2)) * 4 + (tid & 3)];
            s_q[tid] = (t / cnt + p.Cq[tid]) * p.qscale;
        }
    }
    __syncthreads();
    float mx[H], den[H], o[HD];
#pragma unroll
    for (int h = 0; h < H; ++h) { mx[h] = -INFINITY; den[h] = 0.f; }
#pragma unroll
    for (int f = 0; f < HD; ++f) o[f] = 0.f;
    for (int s0 = tid; s0 < p.S; s0 += U * NT) {
        uint4 kv4[U][2 * D / 8];
        float mk[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            mk[u] = s0 + u * NT < p.S && keepn[u] ? 1.f : 0.f;
#pragma unroll
            for (int e8 = 0; e8 < 2 * D / 8; ++e8) kv4[u][e8] = kvn[u][e8];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = s0 + (U + u) * NT, sc = s < p.S ? s : p.S - 1;
            const uint4* kp = reinterpret_cast<const uint4*>(kvc + (size_t)sc * (2 * D));
#pragma unroll
            for (int e8 = 0; e8 < 2 * D / 8; ++e8) kvn[u][e8] = kp[e8];
            if (keepc) keepn[u] = keepc[sc];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (mk[u] == 0.f) continue;
            float k[D], v[D];
#pragma unroll
            for (int e8 = 0; e8 < D / 8; ++e8) {
                const uint4 k8 = kv4[u][e8], v8 = kv4[u][D / 8 + e8];
                const uint32_t kw[4] = {k8.x, k8.y, k8.z, k8.w}, vw[4] = {v8.x, v8.y, v8.z, v8.w};
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    k[8 * e8 + 2 * w] = lo_f32(kw[w]); k[8 * e8 + 2 * w + 1] = hi_f32(kw[w]);
                    v[8 * e8 + 2 * w] = lo_f32(vw[w]); v[8 * e8 + 2 * w + 1] = hi_f32(vw[w]);
                }
            }
#pragma unroll
            for (int h = 0; h < H; ++h) {
                float l = 0.f;
#pragma unroll
                for (int e = 0; e < D; ++e) l += s_q[h * D + e] * k[e];
                // mx is the thread's reference for the exponentials, not the exact maximum: it moves (and the sums
                // are rescaled) only when a logit exceeds it by more than kSlack, so that after a thread's first
                // sequences almost no step pays for the rescaling; weights stay below 2^kSlack
                if (l > mx[h] + kSlack) {
                    const float a = __builtin_amdgcn_exp2f(mx[h] - l);      // 0 for the thread's first sequence
                    mx[h] = l;
                    den[h] *= a;
#pragma unroll
                    for (int e = 0; e < D; ++e) o[h * D + e] *= a;
                }
                const float w = __builtin_amdgcn_exp2f(l - mx[h]);
                den[h] += w;
#pragma unroll
                for (int e = 0; e < D; ++e) o[h * D + e] += w * v[e];
            }
        }
    }
    // bring the lanes of a wavefront to its maximum (a lane without any sequence has -inf and all-zero sums)
    {
        float M[H];
#pragma unroll
        for (int h = 0; h < H; ++h) M[h] = mx[h];
        wave_reduce_scatter<H, true>(M, lane);            // lane l: maximum of head l / (64 / H)
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const float Mh = __shfl(M[0], h * (64 / H), 64);
            const float sc = mx[h] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mx[h] - Mh);
            den[h] *= sc;
#pragma unroll
            for (int e = 0; e < D; ++e) o[h * D + e] *= sc;
        }
        if ((lane & (64 / H - 1)) == 0) s_red[wave * PW + HD + H + lane / (64 / H)] = M[0];
        wave_reduce_scatter<H, false>(den, lane);
        if ((lane & (64 / H - 1)) == 0) s_red[wave * PW + HD + lane / (64 / H)] = den[0];
    }
    if constexpr (HD <= 64) {
        wave_reduce_scatter<HD, false>(o, lane);
        if ((lane & (64 / HD - 1)) == 0) s_red[wave * PW + lane / (64 / HD)] = o[0];
    } else {
        static_assert(HD == 128, "the weighted sums are reduced 64 at a time");
        float o1[64], o2[64];
#pragma unroll
        for (int f = 0; f < 64; ++f) { o1[f] = o[f]; o2[f] = o[64 + f]; }
        wave_reduce_scatter<64, false>(o1, lane);
        wave_reduce_scatter<64, false>(o2, lane);
        s_red[wave * PW + lane] = o1[0];
        s_red[wave * PW + 64 + lane] = o2[0];
    }
    __syncthreads();
    if (tid < HD) {
        const int h = tid / D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, s_red[w * PW + HD + H + h]);      // finite: cnt > 0
        float so = 0.f, sd = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float mw = s_red[w * PW + HD + H + h];
            const float sc = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - M);
            so += s_red[w * PW + tid] * sc;
            sd += s_red[w * PW + HD + h] * sc;
        }
        p.o[(size_t)i * HD + tid] = so / sd;
    }
}

// ====================================================================================
struct OutArgs {
    const bf16_t* m;         // [S][R][c]
    bf16_t* out;             // [S][R][c]
    const float* o;          // [R][Hd]
    int S, R, c, Hd;
    float eps;
    const bf16_t *wg, *wo;   // folded gate weights (pitch 16 KC); W_o in operand order [c][Hd]
    const bf16_t* gext;      // [Hd][8]: row sums and offsets of the gate rows as one more contraction step
    const float* Co;         // [c] output bias
};

template <int KC, int NGT>       // contraction steps of the gate GEMM (c / 16, rounded up to 2, 4, 8); gate tiles H d / 32
__global__ __launch_bounds__(256) void k_gca_out(OutArgs p) {
    constexpr int PITCH = KC * 32 + 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int po = p.Hd * 2 + 16;                                // bytes per row of W_o in LDS
    // the 16 bytes that pad a row of either matrix hold one more contraction step: for a gate row its row sum S and
    // offset C as S S S' C C C' 0 0 (hi, hi, lo), for a row of W_o its bias as b 0 ... 0
    unsigned char* s_wg = smem;                                  // [Hd][PITCH]
    unsigned char* s_wo = smem + (size_t)p.Hd * PITCH;           // [c][po]
    const int pt = p.c * 2 + 16;                                 // bytes per token row of the staged output tile
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // the wavefront's own staging area for one output tile [32 tokens][c]: results leave the accumulators as 8-byte
    // pieces of 32 different tokens; written to memory like that every store instruction would touch 32 lines, so
    // they are gathered here and leave as whole contiguous kilobytes (only this wavefront reads or writes the area;
    // a wavefront's LDS operations complete in order)
    unsigned char* s_tile = s_wo + (size_t)p.c * po + (size_t)wave * 32 * pt;
    for (int id = tid; id < p.Hd * (2 * KC + 1); id += 256) {
        const int row = id / (2 * KC + 1), pc = id - row * (2 * KC + 1);
        const bf16_t* src = pc < 2 * KC ? p.wg + (size_t)row * (16 * KC) + pc * 8 : p.gext + (size_t)row * 8;
        *reinterpret_cast<uint4*>(s_wg + row * PITCH + pc * 16) = *reinterpret_cast<const uint4*>(src);
    }
    const int opr = p.Hd >> 3;                                   // 16-byte pieces per row of W_o
    for (int id = tid; id < p.c * (opr + 1); id += 256) {
        const int row = id / (opr + 1), pc = id - row * (opr + 1);
        uint4 v = make_uint4(f32_to_bf16(p.Co[row]), 0, 0, 0);
        if (pc < opr) v = *reinterpret_cast<const uint4*>(p.wo + (size_t)row * p.Hd + pc * 8);
        *reinterpret_cast<uint4*>(s_wo + row * po + pc * 16) = v;
    }
    __syncthreads();

    // a tile = 32 consecutive residues of one sequence: 32 c contiguous elements of m and of out.  A wavefront
    // keeps ONE residue tile and walks over the sequences: the attended vectors o[i] of its 32 residues are the
    // same for every sequence, so they are read once, and the tokens of the next sequence are on their way while
    // this one is worked on.
    const int tpr = (p.R + 31) >> 5;             // residue tiles per sequence
    const int n_ct = p.c >> 5;                   // output tiles (at most 4)
    const int gw = blockIdx.x * 4 + wave, ng = (gridDim.x * 4) / tpr;      // ng >= 1: wavefronts per residue tile
    const int rt = gw % tpr, sg = gw / tpr;
    if (sg >= ng || sg >= p.S) return;           // (no barrier after this point)
    const int i_raw = rt * 32 + col;
    const bool valid = i_raw < p.R;
    const int i = valid ? i_raw : p.R - 1;
    float4 o4[NGT][4];
    {
        const float* oi = p.o + (size_t)i * p.Hd;
#pragma unroll
        for (int T = 0; T < NGT; ++T)
#pragma unroll
            for (int g = 0; g < 4; ++g) o4[T][g] = *reinterpret_cast<const float4*>(oi + 32 * T + 8 * g + 4 * hf);
    }
    Frag one;                                    // token side of the bias step: a one in slot 0 of the first half
    one.u = make_uint4(hf ? 0u : 0x3f80u, 0u, 0u, 0u);
    TileFetch<KC> tf;
    tf.init(p.c, lane, p.R - rt * 32 < 32 ? p.R - rt * 32 : 32);
    Frag xn[KC];
    tf.fetch(xn, p.m + ((size_t)sg * p.R + rt * 32) * p.c);
    for (int s = sg; s < p.S; s += ng) {
        // (the incoming tile passes through the area that later stages the output tile)
        Frag xa[KC];
        tf.to_operands(xn, xa, s_tile, p.c, col, hf);
        {
            const int sn = s + ng < p.S ? s + ng : s;        // (the last round fetches its own tokens again)
            tf.fetch(xn, p.m + ((size_t)sn * p.R + rt * 32) * p.c);
        }
        // The tokens enter the gate GEMM as they are.  With W' the folded weights, S their row sums and C the
        // offsets, LayerNorm followed by the projection is rstd (W' x - mean S + C / rstd): the two corrections are
        // one more contraction step whose token side holds -mean and 1 / rstd (each as hi + lo bfloat16, slots
        // hi lo hi against the row's hi hi lo), and rstd rides in the factor of the exponential.
        float mean, rstd, istd;
        statistics<KC>(xa, p.c, p.eps, mean, rstd, istd);
        Frag xe;
        {
            float m_hi, m_lo, r_hi, r_lo;
            split2(-mean, m_hi, m_lo);
            split2(istd, r_hi, r_lo);
            xe.w[0] = hf ? 0u : pack2(m_hi, m_lo);
            xe.w[1] = hf ? 0u : pack2(m_hi, r_hi);
            xe.w[2] = hf ? 0u : pack2(r_lo, r_hi);
            xe.w[3] = 0u;
        }
        const float nrl = -kLog2e * rstd;            // sigmoid(rstd a) = 1 / (1 + exp2(nrl a))

        // gate: features x tokens; value of feature 32T + 8g + 4hf + e in register 4g + e, times o[i][feature];
        // registers 8j .. 8j+7 of tile T packed are the B operand of contraction step 2T + j of the output GEMM
        Frag gf[2 * NGT];
#pragma unroll
        for (int T = 0; T < NGT; ++T) {
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int q = 0; q < KC; ++q) {
                Frag wf;
                wf.u = *reinterpret_cast<const uint4*>(s_wg + (32 * T + col) * PITCH + (2 * q + hf) * 16);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, xa[q].v, acc, 0, 0, 0);
            }
            {
                Frag wf;
                wf.u = *reinterpret_cast<const uint4*>(s_wg + (32 * T + col) * PITCH + 2 * KC * 16);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, xe.v, acc, 0, 0, 0);
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float t[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    t[e] = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(nrl * acc[4 * g + e])) * pick(o4[T][g], e);
                gf[2 * T + (g >> 1)].w[2 * (g & 1)] = pack2(t[0], t[1]);
                gf[2 * T + (g >> 1)].w[2 * (g & 1) + 1] = pack2(t[2], t[3]);
            }
        }
        // output projection: features x tokens again, the lane holds four consecutive channels of its token
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
            if (ct < n_ct) {
                f32x16 acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
                for (int kk = 0; kk < 2 * NGT; ++kk) {
                    Frag wf;
                    wf.u = *reinterpret_cast<const uint4*>(s_wo + (32 * ct + col) * po + kk * 32 + hf * 16);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, gf[kk].v, acc, 0, 0, 0);
                }
                {
                    Frag wf;                                     // + b_o: the bias against a one
                    wf.u = *reinterpret_cast<const uint4*>(s_wo + (32 * ct + col) * po + 2 * NGT * 32);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, one.v, acc, 0, 0, 0);
                }
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int c0 = 32 * ct + 8 * g + 4 * hf;
                    *reinterpret_cast<uint2*>(s_tile + col * pt + c0 * 2) =
                        make_uint2(pack2(acc[4 * g], acc[4 * g + 1]), pack2(acc[4 * g + 2], acc[4 * g + 3]));
                }
            }
        }
        // the tile is 32 c contiguous elements of out (residues i0 .. i0 + 31 of sequence s): 16 bytes per lane
        {
            const int i0 = rt * 32, ppr = p.c >> 3;                         // 16-byte pieces per token
            unsigned char* ob = reinterpret_cast<unsigned char*>(p.out + ((size_t)s * p.R + i0) * p.c);
            for (int id = lane; id < 32 * ppr; id += 64) {
                const int row = id / ppr, pc = id - row * ppr;
                const uint4 v = *reinterpret_cast<const uint4*>(s_tile + row * pt + pc * 16);
                if (i0 + row < p.R) *reinterpret_cast<uint4*>(ob + (size_t)id * 16) = v;
            }
        }
    }
}

// ====================================================================================
struct Ws {
    bf16_t *wq, *wkv, *wg, *wo, *gext, *kv;
    unsigned char* keepT;
    float *Cq, *Ckv, *Co, *qpart, *cntpart, *o;
    size_t total;
};

static int kc_for(int K) { return K <= 32 ? 2 : (K <= 64 ? 4 : 8); }

static Ws carve(const ff_global_desc& d, void* base) {
    const int Hd = d.heads * d.head_dim, Kp = 16 * kc_for(d.c), groups = kv_groups(d.n_seq);
    char* b = (char*)base;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* p = b + off;
        off += align256(bytes);
        return p;
    };
    Ws w;
    w.wq = (bf16_t*)take((size_t)Hd * Kp * 2);
    w.wkv = (bf16_t*)take((size_t)32 * Kp * 2);
    w.wg = (bf16_t*)take((size_t)Hd * Kp * 2);
    w.wo = (bf16_t*)take((size_t)d.c * Hd * 2);
    w.Cq = (float*)take((size_t)Hd * 4);
    w.Ckv = (float*)take(32 * 4);
    w.gext = (bf16_t*)take((size_t)Hd * 8 * 2);
    w.Co = (float*)take((size_t)d.c * 4);
    w.kv = (bf16_t*)take((size_t)d.n_res * d.n_seq * 2 * d.head_dim * 2);
    w.keepT = (unsigned char*)take((size_t)d.n_res * d.n_seq);
    w.qpart = (float*)take((size_t)d.n_res * groups * Hd * 4);
    w.cntpart = (float*)take((size_t)d.n_res * groups * 4);
    w.o = (float*)take((size_t)d.n_res * Hd * 4);
    w.total = off;
    return w;
}

}  // namespace gca

bool global_supported(const ff_global_desc& d) {
    const int Hd = d.heads * d.head_dim;
    return d.dtype == FF_BF16 && d.c % 32 == 0 && d.c >= 32 && d.c <= 128 && (d.head_dim == 8 || d.head_dim == 16) &&
           (Hd == 32 || Hd == 64 || Hd == 128);
}

size_t global_workspace(const ff_global_desc& d) { return gca::carve(d, nullptr).total; }

ff_status global_run(const ff_global_desc& d, const ff_global_weights& w, const void* m, const float* mask, void* out,
                     void* ws, hipStream_t st) {
    using namespace gca;
    const int Hd = d.heads * d.head_dim, kc = kc_for(d.c), groups = kv_groups(d.n_seq);
    const Ws s = carve(d, ws);
    {
        KvArgs a{};
        PrepArgs& pa = a.prep;
        pa.w_q = (const bf16_t*)w.w_q; pa.w_k = (const bf16_t*)w.w_k; pa.w_v = (const bf16_t*)w.w_v; pa.w_g = (const bf16_t*)w.w_g;
        pa.b_g = (const bf16_t*)w.b_g; pa.w_o = (const bf16_t*)w.w_o; pa.b_o = (const bf16_t*)w.b_o;
        pa.ln_g = (const bf16_t*)w.ln_g; pa.ln_b = (const bf16_t*)w.ln_b;
        pa.wq = s.wq; pa.wkv = s.wkv; pa.wg = s.wg; pa.wo = s.wo; pa.Cq = s.Cq; pa.Ckv = s.Ckv; pa.gext = s.gext; pa.Co = s.Co;
        pa.c = d.c; pa.Hd = Hd; pa.d = d.head_dim; pa.Kp = 16 * kc;
        a.m = (const bf16_t*)m; a.mask = mask; a.S = d.n_seq; a.R = d.n_res; a.c = d.c; a.Hd = Hd; a.d = d.head_dim;
        a.groups = groups; a.eps = d.ln_eps; a.kv = s.kv; a.keepT = s.keepT; a.qpart = s.qpart;
        a.w_q = pa.w_q; a.w_k = pa.w_k; a.w_v = pa.w_v; a.ln_g = pa.ln_g; a.ln_b = pa.ln_b;
        a.cntpart = s.cntpart;
        a.kv_blocks = ((d.n_res + 31) / 32) * groups;
        // behind the key / value blocks: one wavefront per row of W_q' (for C_q), W_g' and W_o
        const dim3 grid(a.kv_blocks + (2 * Hd + d.c + 3) / 4);
        // weights, the wavefronts' batches of k | v [32 residues][4 sequences] and incoming tiles; afterwards the same bytes hold the
        // four wavefronts' partial sums [32 residues][Hd + 1]
        const size_t smem_loop = (size_t)(Hd + 32) * (kc * 32 + 16) + (size_t)4 * 32 * (16 * d.head_dim + 16) +
                                 (size_t)4 * 32 * (2 * d.c + 16) + 4 * 128 + (size_t)32 * 2 * kc * 4 + 128;
        const size_t smem_red = (size_t)4 * 32 * (Hd + 1) * 4;
        const size_t smem = smem_loop > smem_red ? smem_loop : smem_red;
        hipError_t attr = hipSuccess;
        Timed t(KK_GCA_KV, st);
#define FF_GCA_KV_Q(KCV, DV, QV)                                                                                 \
    do {                                                                                                         \
        static const hipError_t once = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gca_kv<KCV, DV, QV>), \
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024); \
        attr = once;                                                                                             \
        if (once == hipSuccess) hipLaunchKernelGGL((k_gca_kv<KCV, DV, QV>), grid, dim3(256), smem, st, a);       \
    } while (0)
#define FF_GCA_KV_D(KCV, DV)                                                                  \
    do {                                                                                      \
        if (Hd == 32) FF_GCA_KV_Q(KCV, DV, 1);                                                \
        else if (Hd == 64) FF_GCA_KV_Q(KCV, DV, 2);                                           \
        else FF_GCA_KV_Q(KCV, DV, 4);                                                         \
    } while (0)
#define FF_GCA_KV(KCV)                                                                        \
    do {                                                                                      \
        if (d.head_dim == 8) FF_GCA_KV_D(KCV, 8);                                             \
        else FF_GCA_KV_D(KCV, 16);                                                            \
    } while (0)
        if (kc == 2) FF_GCA_KV(2);
        else if (kc == 4) FF_GCA_KV(4);
        else FF_GCA_KV(8);
#undef FF_GCA_KV
#undef FF_GCA_KV_D
#undef FF_GCA_KV_Q
        if (attr != hipSuccess) return fail(FF_EHIP, "k_gca_kv: dynamic LDS limit: %s", hipGetErrorString(attr));
    }
    {
        SmArgs a{};
        a.kv = s.kv; a.keepT = mask ? s.keepT : nullptr; a.qpart = s.qpart; a.cntpart = s.cntpart; a.Cq = s.Cq; a.o = s.o;
        a.S = d.n_seq; a.R = d.n_res; a.Hd = Hd; a.H = d.heads; a.nchunk = groups;
        a.qscale = kLog2e / sqrtf((float)d.head_dim);
        Timed t(KK_GCA_SOFTMAX, st);
#define FF_GCA_SM(HV, DV)                                                                                          \
    do {                                                                                                           \
        constexpr int NT = 256;                                                                                    \
        hipLaunchKernelGGL((k_gca_softmax<HV, DV, NT>), dim3(d.n_res), dim3(NT), 0, st, a);                        \
    } while (0)
        if (d.head_dim == 8) {
            if (d.heads == 4) FF_GCA_SM(4, 8);
            else if (d.heads == 8) FF_GCA_SM(8, 8);
            else FF_GCA_SM(16, 8);
        } else {
            if (d.heads == 2) FF_GCA_SM(2, 16);
            else if (d.heads == 4) FF_GCA_SM(4, 16);
            else FF_GCA_SM(8, 16);
        }
#undef FF_GCA_SM
    }
    {
        OutArgs a{};
        a.m = (const bf16_t*)m; a.out = (bf16_t*)out; a.o = s.o; a.S = d.n_seq; a.R = d.n_res; a.c = d.c; a.Hd = Hd;
        a.eps = d.ln_eps; a.wg = s.wg; a.wo = s.wo; a.gext = s.gext; a.Co = s.Co;
        const int tasks = d.n_seq * ((d.n_res + 31) / 32);
        // as many blocks as are resident together (registers and LDS of the instance decide; four per compute unit
        // at most), at least one wavefront per residue tile
        int blocks = 0;
        const size_t smem = (size_t)Hd * (kc * 32 + 16) + (size_t)d.c * (Hd * 2 + 16) +
                            (size_t)4 * 32 * (d.c * 2 + 16);       // weights (with their extra step), one output tile per wavefront
        hipError_t attr = hipSuccess;
        Timed t(KK_GCA_OUT, st);
#define FF_GCA_OUT(KCV, NGTV)                                                                                    \
    do {                                                                                                         \
        static const hipError_t once = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gca_out<KCV, NGTV>), \
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 112 * 1024); \
        attr = once;                                                                                             \
        int per_cu = 0;                                                                                          \
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_gca_out<KCV, NGTV>, 256, smem) != hipSuccess || per_cu < 1) \
            per_cu = 1;                                                                                          \
        if (per_cu > 4) per_cu = 4;                                                                              \
        blocks = (tasks + 3) / 4;                                                                                \
        if (blocks > per_cu * compute_units()) blocks = per_cu * compute_units();                                \
        if (blocks * 4 < (d.n_res + 31) / 32) blocks = ((d.n_res + 31) / 32 + 3) / 4;                            \
        if (once == hipSuccess) hipLaunchKernelGGL((k_gca_out<KCV, NGTV>), dim3(blocks), dim3(256), smem, st, a); \
    } while (0)
#define FF_GCA_OUT_K(KCV)                                                                                        \
    do {                                                                                                         \
        if (Hd == 32) FF_GCA_OUT(KCV, 1);                                                                        \
        else if (Hd == 64) FF_GCA_OUT(KCV, 2);                                                                   \
        else FF_GCA_OUT(KCV, 4);                                                                                 \
    } while (0)
        if (kc == 2) FF_GCA_OUT_K(2);
        else if (kc == 4) FF_GCA_OUT_K(4);
        else FF_GCA_OUT_K(8);
#undef FF_GCA_OUT_K
#undef FF_GCA_OUT
        if (attr != hipSuccess) return fail(FF_EHIP, "k_gca_out: dynamic LDS limit: %s", hipGetErrorString(attr));
    }
    return check_launch("global column attention");
}

}  // namespace ff
