// bfloat16 matrix-core kernel family for gfx950 (wave64, v_mfma_f32_32x32x16_bf16).
//
// Pipeline per call (FastFold Sections 2.1, 2.3, 5.2):
//   k_prep      once per call: folds the LayerNorm gain into the merged q|k|v|gate(|bias)
//               weight matrix (Section 5.2 "merge GEMM"), with per-feature sums so that the
//               LayerNorm can be finished in the GEMM epilogue
//   k_gemm<PROJ> merged projection straight from the raw input: with W' = W*gamma,
//               LN(x) W^T = rstd * (x W'^T - mean * rowsum(W') + std * W beta), so the matrix cores
//               read x as it lies in HBM; the mean and offset terms are one extra contraction
//               step (operands split into bf16 hi + lo pairs) and the epilogue is a multiplication
//               by rstd: q scaled, gate = sigmoid(. + b_g), q,k,gate head-major, v transposed,
//               pair-bias columns as float32 [H][Lq][Lp]
//   k_attn      flash-style attention: S^T = K Q^T on the matrix cores with the bias tile as
//               accumulator input; the key mask and the running reference maximum ride in
//               two spare slots of the contraction, so the matrix core already returns
//               s - m (+ -inf for masked keys) and the vector unit only exponentiates
//               (the paper's fused scale + mask + bias softmax, Section 5.2, without ever
//               materialising the score tensor of Section 3.2); O^T = V^T P^T; gate product
//   k_gemm<OUT> output projection + b_o, scattered to the caller's layout
//   k_proj_attn sequences of 129..256 positions at head dimension 32: k_gemm<PROJ> and k_attn in one
//               kernel (a block = two batch rows x one head), q, k, v and gate never leave the chip
//
// Matrix-core operand layouts (wave64, 32x32x16, bf16 in, f32 out):
//   A (32 x 16): lane l holds row l%32, columns 8*(l/32) .. +7
//   B (16 x 32): lane l holds column l%32, rows 8*(l/32) .. +7
//   C/D (32 x 32): lane l holds column l%32, register v holds row 8*(v/4) + 4*(l/32) + v%4
// Computing S^T (keys x queries) puts one query in one lane, so softmax statistics are
// lane-local except for one exchange between the two half-waves, and the exponentiated tile
// already has the B-operand layout of the second contraction once the key order inside a
// 32-key tile is permuted; the same permutation is applied when K rows and V^T columns are
// fetched, so nothing moves between the two contractions.
//
// Workspace layout of this family (Lp = Lq = L rounded up to 64, token p = rl*Lp + l):
//   bias [H][Lq][Lp] float32 (times log2 e); for k_proj_attn the same elements in 32 x 32 tiles (bias_index)
//   q, k, g, o [rows][H][Lp][D] bf16;  vt [rows][H][Lp/32][D][32] bf16
//   prepared weights [(4*Hd + 32)][c] (+ [32][c_z] in row mode) bf16, their sums and offsets
// Pad tokens (l in [L, Lp)) hold finite values everywhere; they are masked as keys.
#include "ff_common.h"

#include <type_traits>

namespace ff {

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
__device__ __forceinline__ float lo_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_f32(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_round(float f) { return lo_f32(pack2(f, 0.f)); }

__device__ __forceinline__ uint4 ldg16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ uint2 ldg8(const void* p) { return *reinterpret_cast<const uint2*>(p); }
// The same loads and a store with the address split into a wave-uniform base (scalar registers)
// and a 32-bit byte offset per lane: one instruction, no address arithmetic in the vector unit.
__device__ __forceinline__ uint4 ldg16(const void* base, uint32_t lane_bytes) {
    return *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(base) + lane_bytes);
}
__device__ __forceinline__ uint2 ldg8(const void* base, uint32_t lane_bytes) {
    return *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(base) + lane_bytes);
}
__device__ __forceinline__ void stg16(void* base, uint32_t lane_bytes, uint4 v) {
    *reinterpret_cast<uint4*>(reinterpret_cast<char*>(base) + lane_bytes) = v;
}

// sum of the two bf16 halves of w, added to acc (v_dot2c_f32_bf16)
__device__ __forceinline__ float add_pair(uint32_t w, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, 0x3f803f80u), acc,
                                           false);
}

// sum of the squares of the two bf16 halves of w, added to acc (v_dot2c_f32_bf16: exact products)
__device__ __forceinline__ float add_pair_sq(uint32_t w, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, w), acc, false);
}

// value of the other half-wave's lane (l ^ 32)
__device__ __forceinline__ float other_half(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    // r[0] = {lower half of v, lower half of v}, r[1] = {upper half, upper half}
    return (threadIdx.x & 32) ? __uint_as_float(r[0]) : __uint_as_float(r[1]);
}

// LayerNorm statistics of a token whose K channels lie in the KC fragments of the two lanes
// (col, hf = 0 | 1), channels beyond K being zero: mean and variance + eps, float32, in one pass
// over the registers.  sum x and sum x^2 are accumulated from exact bf16 products (two channels
// per instruction), var = sum x^2 / K - mean^2: the cancellation costs a relative error of
// about 2^-22 (1 + mean^2 / var) of the variance, 2e-5 for a mean of twelve standard
// deviations.  (The two-pass form, sum (x - mean)^2, took 450 vector instructions per lane for
// K = 256, a quarter of this wavefront's work before its first matrix instruction.)
// Every kernel takes the statistics from here, so that they agree bit for bit.
template <int KC>
__device__ __forceinline__ void token_stats(const Frag (&xa)[KC], int K, float eps, float& mu, float& var) {
    float sum = 0.f, sq = 0.f;
#pragma unroll
    for (int s = 0; s < KC; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sum = add_pair(xa[s].w[i], sum);
            sq = add_pair_sq(xa[s].w[i], sq);
        }
    sum += other_half(sum);
    sq += other_half(sq);
    const float inv_k = 1.f / (float)K;
    mu = sum * inv_k;
    var = fmaxf(sq * inv_k - mu * mu, 0.f) + eps;
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
    bf16_t *wp, *zwp;      // prepared weights: main [(4Hd+32)][c], row-mode bias [32][c_z]
    uint4* aug;            // [(4Hd+32) + 32] per row of wp / zwp: its sum and output offset as bf16 pairs (see k_prep)
};

static MfmaWs split_ws(const Problem& p, int chunk, const Workspace& ws) {
    const size_t Lp = round_up(p.L, 64);
    const size_t n = (size_t)chunk * Lp * p.Hd;   // elements per tensor
    MfmaWs m;
    m.q = (bf16_t*)ws.qkvg;
    m.k = m.q + n;
    m.g = m.k + n;
    m.vt = m.g + n;
    m.o = (bf16_t*)ws.o;
    char* pr = (char*)ws.prep;
    const size_t rows_main = 4 * (size_t)p.Hd + 32;
    m.wp = (bf16_t*)pr;
    pr += align256(rows_main * p.c * 2);
    m.zwp = (bf16_t*)pr;
    pr += align256((size_t)32 * (p.c_z > 0 ? p.c_z : 1) * 2);
    m.aug = (uint4*)pr;
    return m;
}

bool mfma_supported(const Problem& p) {
    if (p.dtype != FF_BF16) return false;
    if (p.c % 32 != 0 || p.c > 256) return false;
    if (p.Hd % 32 != 0 || p.Hd > 256) return false;
    if (p.d != 8 && p.d != 16 && p.d != 32) return false;
    if (p.L > 16384) return false;
    if (p.H > 32) return false;
    if (p.mode == FF_MSA_ROW && (p.c_z % 16 != 0 || p.c_z > 256)) return false;
    return true;
}

size_t mfma_workspace(const Problem& p, int chunk, Workspace* ws, void* base) {
    const size_t Lp = round_up(p.L, 64), Lq = round_up(p.L, 64);
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
    ws->prep = b + off;
    const size_t rows_main = 4 * (size_t)p.Hd + 32;
    off += align256(rows_main * p.c * 2) + align256((size_t)32 * (p.c_z > 0 ? p.c_z : 1) * 2) +
           align256((rows_main + 32) * 16);
    ws->total = off;
    ws->chunk = chunk;
    return off;
}

// ====================================================================================
// Weight preparation: one wavefront per output row n of the merged matrix.
//   wp[n][k] = bf16(scale * W[n][k] * gamma[k]);  sn[n] = sum_k wp[n][k];
//   cn[n] = scale * sum_k W[n][k] * beta[k] (+ extra[n])
// sn and cn leave as one extra 8-slot piece of the contraction per row, split into bf16 pairs
// (hi + lo): [sn_hi, sn_lo, sn_hi, cn_hi, cn_lo, cn_hi, 0, 0].  Against the token's piece
// [m_hi, m_hi, m_lo, r_hi, r_hi, r_lo, 0, 0] (m = -mean, r = standard deviation) the matrix core
// adds -mean*sn + r*cn to x W'^T, so that the GEMM epilogue is one multiplication by 1/r.
struct PrepSeg {
    const bf16_t* w;              // [rows][K]
    const bf16_t* extra;          // [rows] added to cn, or NULL
    const bf16_t *gamma, *beta;   // [K]
    bf16_t* wp;                   // output rows of this segment [rows_pad][K]
    uint4* aug;                   // [rows_pad]
    int rows, rows_pad, K;        // rows_pad - rows zero rows follow
    float scale;
};
struct PrepArgs {
    PrepSeg seg[6];
    int nseg;
};

// One row of a folded matrix by one wavefront: store(k, bf16(scale * w[k] * gamma[k])) for k < K and
// the row's extra piece as the return value (valid in every lane).  Every kernel that folds a row
// goes through here, so that the same weights give the same bits wherever they are prepared (the
// pair bias of the triangle modes is prepared by k_prep when it rides along with the projections
// and by k_prep_bias when the rows are chunked, and both must give the same output bits).
template <typename Store>
__device__ __forceinline__ uint4 fold_row(const bf16_t* wrow, const bf16_t* gamma, const bf16_t* beta, int K, float scale,
                                          bool real, float extra, int lane, Store&& store) {
    float sum = 0.f, cst = 0.f;
    // K <= 256: at most four elements per lane.  The loads carry no condition (an element beyond K
    // reads element K - 1 and is dropped below, a pad row reads the row the caller passes for it): a
    // conditional load is a branch and a wait of its own, twelve memory round trips one after the other
    // instead of one.
    bf16_t wv[4], gv[4], bv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int k = lane + 64 * i;
        const int kc = k < K ? k : K - 1;
        wv[i] = wrow[kc];
        gv[i] = gamma[kc];
        bv[i] = beta[kc];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bool in = real && lane + 64 * i < K;
        if (!in) wv[i] = gv[i] = bv[i] = (bf16_t)0;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int k = lane + 64 * i;
        if (k < K) {
            const float w = bf16_to_f32(wv[i]) * scale;
            const float r = bf16_round(w * bf16_to_f32(gv[i]));
            cst += w * bf16_to_f32(bv[i]);
            store(k, f32_to_bf16(r));
            sum += r;
        }
    }
    sum = wave_sum(sum);
    cst = wave_sum(cst);
    const float cn = cst + extra;
    const float sn_hi = bf16_round(sum), sn_lo = bf16_round(sum - sn_hi);
    const float cn_hi = bf16_round(cn), cn_lo = bf16_round(cn - cn_hi);
    return make_uint4(pack2(sn_hi, sn_lo), pack2(sn_hi, cn_hi), pack2(cn_lo, cn_hi), 0u);
}

// row n of the concatenated segments, by one wavefront
__device__ __forceinline__ void prep_row(const PrepArgs& a, int n_in, int lane) {
    const int n = __builtin_amdgcn_readfirstlane(n_in);      // (a wavefront's row: the segment is then read with scalar loads)
    int base = 0, sg = -1, local = 0;
    for (int i = 0; i < a.nseg; ++i) {
        if (sg < 0 && n < base + a.seg[i].rows_pad) {
            sg = i;
            local = n - base;
        }
        base += a.seg[i].rows_pad;
    }
    if (sg < 0) return;
    PrepSeg sgm = a.seg[0];
#pragma unroll
    for (int i = 1; i < 6; ++i)
        if (i == sg) sgm = a.seg[i];
    const bool real = local < sgm.rows;
    const int K = sgm.K;
    // (no condition on the load, see fold_row: without an offset vector the row reads gamma[0] and drops it)
    const bool has_extra = real && sgm.extra != nullptr;
    const float extra_raw = bf16_to_f32(*(has_extra ? sgm.extra + local : sgm.gamma));
    const float extra = has_extra ? extra_raw : 0.f;
    bf16_t* wp = sgm.wp + (size_t)local * K;
    // (a pad row has no weights, its segment possibly no matrix at all: it reads gamma, K valid elements, instead)
    const uint4 piece = fold_row(real ? sgm.w + (size_t)local * K : sgm.gamma, sgm.gamma, sgm.beta, K, sgm.scale, real, extra, lane,
                                 [&](int k, bf16_t v) { wp[k] = v; });
    if (lane == 0) sgm.aug[local] = piece;
}

__global__ __launch_bounds__(256) void k_prep(PrepArgs a) {
    prep_row(a, blockIdx.x * 4 + (threadIdx.x >> 6), threadIdx.x & 63);
}

// ====================================================================================
// The pair bias b[h][i][j] = log2(e) * sum_c LN(z[i][j])_c W_b[h][c] as a pass of its own (row mode:
// over the pair representation with its own LayerNorm; chunked triangle modes: over all of x before
// the first chunk) and the weight preparation in ONE launch (they do not depend on each other).  Blocks below bias_blocks take
// 256 pairs each (one 32-pair tile per wavefront, the folded 32 x K weight tile built by the block
// itself in LDS, same algebra as k_gemm's pair-bias tile); the blocks above them run prep_row.
// Element (h, q, k) of the pair bias.  Plain: [H][Lq][Lp].  Tiled (for k_proj_attn): 32 x 32 tiles in
// the register order of an S^T accumulator, [H][Lq/32][Lp/32][4][64 lanes][4]: lane = (q % 32) + 32 hf
// holds the keys 16c + 8hf + 4i + e of the tile in element e of group 2c + i, so that a wavefront
// fetches a tile with four loads of 1 KiB each.
__device__ __forceinline__ size_t bias_index(bool tiled, int h, int q, int k, int Lq, int Lp) {
    if (!tiled) return ((size_t)h * Lq + q) * Lp + k;
    const int kk = k & 31;
    const int grp = 2 * (kk >> 4) + ((kk >> 2) & 1), hf = (kk >> 3) & 1;
    const size_t tile = ((size_t)h * (Lq >> 5) + (q >> 5)) * (Lp >> 5) + (k >> 5);
    return ((tile * 4 + grp) * 64 + (q & 31) + 32 * hf) * 4 + (kk & 3);
}

struct PrepBiasArgs {
    PrepArgs prep;
    int tiled;                   // layout of the output (bias_index)
    int bias_blocks;
    const bf16_t* z;             // pair (i, j) at z + (i*sr + j*sl)*K
    int64_t sr, sl;
    const bf16_t *w_b, *gamma, *beta;   // [H][K], [K], [K]
    float* bias;                 // [H][Lq][Lp]
    int L, Lp, Lq, K, H;
    float eps;
};

template <int KC>
__global__ __launch_bounds__(512) void k_prep_bias(PrepBiasArgs a) {
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if ((int)blockIdx.x >= a.bias_blocks) {
        prep_row(a.prep, ((int)blockIdx.x - a.bias_blocks) * 8 + wave, lane);
        return;
    }
    constexpr int PITCH = KC * 32 + 16;                 // bytes per weight row in LDS (padded: conflict-free reads)
    __shared__ __attribute__((aligned(16))) unsigned char s_w[32 * PITCH];
    __shared__ uint4 s_aug[32];
    const int K = a.K;

    // ---- pairs of this wavefront: raw operand fragments (issued first)
    const int tiles_m = a.L * (a.Lp >> 5);
    int tg = blockIdx.x * 8 + wave;
    if (tg > tiles_m - 1) tg = tiles_m - 1;             // (repeats the last tile: same values stored twice)
    const int pr = tg * 32 + col;
    const int qi = pr / a.Lp, kj = pr - qi * a.Lp;
    const bool valid = kj < a.L;
    // Eight lanes fetch one 128-byte line of a pair (64 channels); the lines pass through 4 KiB of LDS
    // per wavefront and come back in the operand layout (lane = pair, pieces 2s' + hf of line m =
    // contraction steps 4m + s').  A load with lane = pair touches 64 cache lines for 1 KiB, and the
    // cache looks up one line per cycle: the fetch alone took 2.5 us of the block's 6.
    constexpr int NG = (KC + 3) / 4;
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[8][4096];
    unsigned char* s_st = s_stage[wave];
    uint4 raw[NG][4];
    {
        const int q0 = (tg * 32) / a.Lp, k0 = tg * 32 - q0 * a.Lp;       // (uniform: a tile lies inside one query row)
        const int pieces = K >> 3;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int kk = k0 + 8 * i + (lane >> 3);
            const bf16_t* zq = a.z + ((int64_t)q0 * a.sr + (int64_t)(kk < a.L ? kk : 0) * a.sl) * K + (lane & 7) * 8;
#pragma unroll
            for (int m = 0; m < NG; ++m) {
                raw[m][i] = make_uint4(0, 0, 0, 0);
                if (kk < a.L && 8 * m + (lane & 7) < pieces) raw[m][i] = ldg16(zq + 64 * m);
            }
        }
    }

    // ---- the folded weight tile: zeros, then one wavefront per head row (fold_row)
    for (int i = tid; i < 32 * PITCH / 16; i += 512) reinterpret_cast<uint4*>(s_w)[i] = make_uint4(0, 0, 0, 0);
    if (tid < 32) s_aug[tid] = make_uint4(0, 0, 0, 0);
    __syncthreads();
    for (int row = wave; row < a.H; row += 8) {
        bf16_t* dst = reinterpret_cast<bf16_t*>(&s_w[row * PITCH]);
        const uint4 piece = fold_row(a.w_b + (size_t)row * K, a.gamma, a.beta, K, kLog2e, true, 0.f, lane,
                                     [&](int k, bf16_t v) { dst[k] = v; });
        if (lane == 0) s_aug[row] = piece;
    }

    // ---- the pairs as operands (the staging area is the wavefront's own, its LDS operations complete in order)
    Frag xa[KC];
#pragma unroll
    for (int m = 0; m < NG; ++m) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int tl = 8 * i + (lane >> 3);
            *reinterpret_cast<uint4*>(s_st + tl * 128 + (((lane & 7) ^ (tl & 7)) * 16)) = raw[m][i];
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int sp = 0; sp < 4; ++sp)
            if (4 * m + sp < KC)
                xa[4 * m + sp].u = *reinterpret_cast<const uint4*>(s_st + col * 128 + (((2 * sp + hf) ^ (col & 7)) * 16));
        __builtin_amdgcn_wave_barrier();
    }

    // ---- LayerNorm statistics of the wavefront's pairs
    float mu, var;
    token_stats<KC>(xa, K, a.eps, mu, var);
    const float rstd = valid ? rsqrtf(var) : 0.f;
    const float m = valid ? -mu : 0.f, r = var * rstd;
    const float m_hi = bf16_round(m), m_lo = bf16_round(m - m_hi);
    const float r_hi = bf16_round(r), r_lo = bf16_round(r - r_hi);
    Frag xaug;
    xaug.u = make_uint4(0, 0, 0, 0);
    if (hf == 0) xaug.u = make_uint4(pack2(m_hi, m_hi), pack2(m_lo, r_hi), pack2(r_hi, r_lo), 0u);

    __syncthreads();
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
    for (int s = 0; s < KC; ++s) {
        Frag wf;
        wf.u = *reinterpret_cast<const uint4*>(&s_w[col * PITCH + (2 * s + hf) * 16]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, xa[s].v, acc, 0, 0, 0);
    }
    {
        Frag wa;
        wa.u = s_aug[col];
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa.v, xaug.v, acc, 0, 0, 0);
    }
    // lane = pair (qi, kj), register v = head 8*(v/4) + 4*hf + v%4
    float* bp = a.bias + bias_index(a.tiled != 0, 0, qi, kj, a.Lq, a.Lp);
    const size_t plane = (size_t)a.Lq * a.Lp;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int h = 8 * (v >> 2) + 4 * hf + (v & 3);
        if (h < a.H) bp[(size_t)h * plane] = acc[v] * rstd;
    }
}

// Rows q in [L, Lq) of the bias tensor [H][Lq][Lp] belong to pad queries: no kernel computes them, but
// the attention kernel stages whole 64-query tiles.  Zeros there keep its lanes for pad queries (never
// stored) on the common path whatever the caller's workspace held before.
__global__ __launch_bounds__(256) void k_zero_bias_pad(float* bias, int L, int Lq, int Lp, int H, int tiled) {
    const int per_head = (Lq - L) * Lp;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= per_head * H) return;
    const int h = i / per_head, r = i - h * per_head;
    const int q = L + r / Lp, k = r - (q - L) * Lp;
    bias[bias_index(tiled != 0, h, q, k, Lq, Lp)] = 0.f;
}

// ====================================================================================
// GEMM with the whole contraction length (<= 256) resident: a wavefront owns TT 32-token
// tiles as register-resident operand fragments and sweeps over 32-feature tiles of the
// weight matrix.  The block streams those tiles through LDS with loads that write LDS
// directly (global_load_lds_dwordx4: lane i of a wavefront deposits its 16 bytes at the
// wave-uniform LDS base + 16 i), NS tiles per step, double buffered: the tiles of step i+1
// are in flight while the matrix cores work on step i.
//
// LDS image of a tile: 32 rows of P = 2 KC 16-byte pieces, piece p of row r at slot
// r P + (p ^ g(r)); g spreads 16 consecutive rows over the 16 slots of a 256-byte LDS line, so
// the operand reads (lane = row, all lanes the same piece) are conflict free without padding.
struct GemmArgs {
    const bf16_t* src;     // PROJ: x or z (strided tokens); OUT: o [rows][H][Lp][D]
    int64_t sr, sl;        // token strides of src (PROJ) / out (OUT)
    int r0, rows, L, Lp, Lq;
    int K;                 // contraction length
    float eps;
    const bf16_t* w;       // PROJ: prepared weights [tiles*32][K]; OUT: w_o [N][K]
    const uint4* aug;      // PROJ: per-feature extra piece of the contraction (sum and offset, see k_prep)
    const bf16_t* bvec;    // OUT: b_o [N]
    int Hd, H, D;
    int dsh;               // log2(D), D in {8, 16, 32}
    float invD;            // 1 / D
    int nt_main;           // PROJ: 32-feature tiles of q|k|v|gate; tile nt_main is the pair-bias tile
    bf16_t *q, *k, *g, *vt;  // PROJ outputs
    float* bias;             // PROJ pair-bias output [H][Lq][Lp]
    bf16_t* out;             // OUT output, token (r,l) at (r*sr + l*sl)*N
    const bf16_t* res;       // OUT with RES: added to the output, laid out like out (may be out itself)
    int N;                   // OUT: features
    int ft_first, ft_count;  // range of feature tiles of this launch
    int tiles_per_split;     // tiles per blockIdx.y
};

typedef void __attribute__((address_space(3)))* lptr_t;
constexpr int kWaitVmcnt0 = 0x0F70;      // s_waitcnt vmcnt(0), the other counters untouched

// Wait until at most n (rounded down to 8, 4, 2 or 0) vector-memory operations of this wavefront
// are outstanding.  They complete in order, so with n = number of stores issued after a load this
// waits for the load but not for those stores.
__device__ __forceinline__ void wait_vmem_but_last(int n) {
    if (n >= 8) __builtin_amdgcn_s_waitcnt(0x0F78);
    else if (n >= 4) __builtin_amdgcn_s_waitcnt(0x0F74);
    else if (n >= 2) __builtin_amdgcn_s_waitcnt(0x0F72);
    else __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
}

// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base wave-uniform).
// Written as assembly on purpose: the compiler would make every later LDS read wait for a load it
// knows to write LDS, also those of the other half of the ring.  The kernel waits for these loads
// itself (s_waitcnt vmcnt(0) before the barrier that publishes the tile).
__device__ __forceinline__ void load16_to_lds(const void* gsrc, unsigned lds_base) {
    const unsigned base = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gsrc), "s"(base) : "memory", "m0");
}

constexpr int kGemmWaves = 8;      // wavefronts per block: two per SIMD

// dynamic LDS of k_gemm: weight ring, LayerNorm statistics, per-feature sums and offsets
static size_t gemm_smem_bytes(int kc, int tt, int ns, int tiles_per_split) {
    return (size_t)2 * ns * 32 * 2 * kc * 16 + (size_t)kGemmWaves * tt * 64 * 4 + (size_t)tiles_per_split * 32 * (4 + 16);
}

// tile kinds of k_gemm (q and k share their epilogue)
enum { TK_Q = 0, TK_K = 1, TK_V = 2, TK_GATE = 3, TK_BIAS = 4, TK_OUT = 5 };

template <int KC, bool PROJ, int TT, int NS, bool RES>
__global__ __launch_bounds__(kGemmWaves * 64, 2) void k_gemm(GemmArgs a) {
    static_assert(!(PROJ && RES), "the residual belongs to the output projection");
    constexpr int NW = kGemmWaves;
    constexpr int P = 2 * KC;                           // 16-byte pieces per weight row
    constexpr int STAGE = 32 * P * 16;                  // bytes of one 32-feature tile in LDS
    constexpr int RSH = P >= 16 ? 0 : (P == 8 ? 1 : 2);
    constexpr int GM = (P >= 16 ? 16 : P) - 1;          // g(r) = (r >> RSH) & GM
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* s_w = smem;                                              // [2][NS][STAGE]
    float* s_stat = reinterpret_cast<float*>(smem + 2 * NS * STAGE);        // [wave][tt][2][32]: 1/std of the wave's tokens in [1]
    float* s_cn = s_stat + NW * TT * 64;                                     // OUT: [tiles_per_split][32] output bias
    uint4* s_aug = reinterpret_cast<uint4*>(s_cn + a.tiles_per_split * 32);  // PROJ: [tiles_per_split][32] extra piece per feature

    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = a.K;
    const int tiles_m = a.rows * (a.Lp >> 5);
    const int ft_begin = a.ft_first + blockIdx.y * a.tiles_per_split;
    int ft_end = ft_begin + a.tiles_per_split;
    if (ft_end > a.ft_first + a.ft_count) ft_end = a.ft_first + a.ft_count;
    if (ft_begin >= ft_end) return;     // (whole block)

    // ---- token operand fragments, raw (issued first: they come from HBM)
    Frag xa[TT][KC];
    bool tok_valid[TT], tile_off[TT];     // tile_off (wave-uniform): a repeated tile that must not be stored
    int tok_rl[TT], tok_l[TT];            // batch row (wave-uniform) and position of this lane's token
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        // (token tiles beyond the last one repeat it: the same values are stored twice)
        int tg = (blockIdx.x * NW + wave) * TT + tt;
        const bool repeated = tg > tiles_m - 1;
        if (repeated) tg = tiles_m - 1;
        const int p = tg * 32 + col;
        const int rl = p / a.Lp, l = p - rl * a.Lp;
        tok_rl[tt] = __builtin_amdgcn_readfirstlane(rl);       // a tile lies inside one batch row
        tok_l[tt] = l;
        // (with a residual that may be the output itself a tile must be added and stored once only)
        tile_off[tt] = RES && repeated;
        tok_valid[tt] = l < a.L && !tile_off[tt];
        const bf16_t* sp = a.src + ((int64_t)(a.r0 + rl) * a.sr + (int64_t)l * a.sl) * K;
#pragma unroll
        for (int s = 0; s < KC; ++s) {
            xa[tt][s].u = make_uint4(0, 0, 0, 0);
            const int f = 16 * s + 8 * hf;
            if constexpr (PROJ) {
                if (tok_valid[tt] && f < K) xa[tt][s].u = ldg16(sp + f);
            } else {
                // gated context, head-major [row][head][l][d]
                const int hh = (int)(((float)f + 0.5f) * a.invD);
                if (tok_valid[tt] && f < K)
                    xa[tt][s].u = ldg16(a.src + ((size_t)(rl * a.H + hh) * a.Lp + l) * a.D + (f - hh * a.D));
            }
        }
    }

    // ---- weight tiles: each wavefront moves KC/NW chunks of 64 pieces (1 KiB) of a tile.
    // Pieces beyond K re-read the last valid piece (the token operand is zero there).
    constexpr int IPW = KC >= NW ? KC / NW : 1;
    int goff[IPW];
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
        int chunk = j * NW + wave;
        if (KC < NW && chunk >= KC) chunk = 0;
        const int ps = chunk * 64 + lane, row = ps / P, pp = ps % P;
        int kk = (pp ^ ((row >> RSH) & GM)) * 8;
        if (kk > K - 8) kk = K - 8;
        goff[j] = row * K + kk;
    }
    const unsigned s_w_lds = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lptr_t)s_w);
    auto issue_tile = [&](int ft, int stage) {
        const bf16_t* wt = a.w + (size_t)ft * 32 * K;
#pragma unroll
        for (int j = 0; j < IPW; ++j) {
            const int chunk = j * NW + wave;
            if (KC >= NW || chunk < KC) load16_to_lds(wt + goff[j], s_w_lds + stage * STAGE + chunk * 1024);
        }
    };
    // steps 0 and 1 fill the two halves of the ring
#pragma unroll
    for (int n = 0; n < 2 * NS; ++n)
        if (ft_begin + n < ft_end) issue_tile(ft_begin + n, n);
    // per-feature sums / offsets of this block's tiles
    for (int i = tid; i < (ft_end - ft_begin) * 32; i += NW * 64) {
        if constexpr (PROJ) {
            s_aug[i] = a.aug[ft_begin * 32 + i];
        } else {
            s_cn[i] = bf16_to_f32(a.bvec[ft_begin * 32 + i]);
        }
    }
    // operand read: piece 2s + hf of row col sits at byte rd0 ^ (32 s) of its tile
    const unsigned rd0 = (unsigned)col * (P * 16) + 16u * (unsigned)((((col >> RSH) & GM)) ^ hf);

    // ---- epilogue addressing: every tensor of this family has Lp*Hd elements per batch row
    const int LpD = a.Lp * a.D;
    size_t row_base[TT];      // PROJ: element offset of the batch row in q, k, gate, v^T; OUT: of the token in out
    int l0v[TT];
    unsigned t_lane[TT];      // q, k, gate, out: this lane's part of the element offset (the same for every tile)
    bool any_valid[TT];       // some token of the tile is a real one
    // v^T: lane = feature col of a 32-feature tile that starts at a multiple of 32 inside v
    const unsigned v_lane = (unsigned)(col >> a.dsh) * LpD + (unsigned)(col & (a.D - 1)) * 32 + 8 * hf;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        if constexpr (PROJ) row_base[tt] = (size_t)tok_rl[tt] * a.H * LpD;
        else {
            // (pad tokens take the address of the last real one: they load the residual, never store)
            const int lc = tok_l[tt] < a.L ? tok_l[tt] : a.L - 1;
            row_base[tt] = (size_t)(((int64_t)(a.r0 + tok_rl[tt]) * a.sr + (int64_t)lc * a.sl) * a.N);
        }
        if constexpr (PROJ) t_lane[tt] = (unsigned)tok_l[tt] * a.D + (a.D >= 16 ? 8 * hf : hf * LpD);
        else t_lane[tt] = 8 * hf;
        const int l0 = __builtin_amdgcn_readfirstlane(tok_l[tt] - col);
        l0v[tt] = l0 * a.D;                                                   // (l0 / 32) * D * 32
        any_valid[tt] = l0 < a.L && !tile_off[tt];
    }
    float rstd[TT];           // 1 / standard deviation of this lane's token
    Frag xaug[TT];            // its extra piece of the contraction: (-mean, standard deviation) as bf16 pairs (see k_prep)
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        rstd[tt] = 0.f;
        xaug[tt].u = make_uint4(0, 0, 0, 0);
    }

    // ---- residual (RES): the matrix core adds it.  Two more contraction steps multiply a
    // selection matrix (feature f of the tile picks slot f, then f - 16) with the residual
    // values of 16 features per token: 1.0 * bf16 into the float32 accumulator is exact, the
    // operand is the token's row as it lies in memory (16 bytes per lane, the very bytes the
    // lane stores later, so the output may replace the residual in place), and the sum is
    // rounded to bf16 once.  ra feeds the first tile of a pipeline step, rb the second; each is
    // reloaded for the next step as soon as its matrix instructions have been issued.
    Frag sel[2];
    Frag ra[TT][2], rb[TT][2];
    auto load_res = [&](Frag (&r)[TT][2], int ft) {
        if (ft > ft_end - 1) ft = ft_end - 1;            // (past the end: a harmless repeat)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const bf16_t* rp = a.res + row_base[tt] + (size_t)ft * 32 + 8 * hf;
            r[tt][0].u = ldg16(rp);
            r[tt][1].u = ldg16(rp + 16);
        }
    };
    if constexpr (RES) {
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int k = col - 16 * m - 8 * hf;             // slot of this lane's feature inside its piece
#pragma unroll
            for (int i = 0; i < 4; ++i)
                sel[m].w[i] = (k >> 1) == i ? ((k & 1) ? 0x3f800000u : 0x00003f80u) : 0u;
        }
        load_res(ra, ft_begin);
        load_res(rb, ft_begin + 1);
    }

    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
    __syncthreads();

    // Software pipeline inside every wavefront: the matrix-core instructions of tile i alternate,
    // one contraction step at a time, with the vector instructions of the epilogue of tile i-1
    // (a wavefront issues a vector instruction only every eight cycles or so and a 32x32x16
    // matrix instruction lasts 32: the epilogue fits into the shadow of the matrix core).
    // Two accumulator sets alternate between the roles "being computed" and "being stored".
    constexpr int VPC = 16 / KC > 0 ? 16 / KC : 1;      // epilogue values per contraction step
    constexpr int AHEAD = KC < 4 ? KC : 4;              // operand reads in flight (LDS latency is about two steps)
    const int LpD2 = LpD;
    int n_stores = 0;                     // stores and residual loads issued in this step (a lower bound)
    f32x16 acc[2][TT];

    // matrix part of tile ftn (weights at st) into an[], epilogue of tile ftp (kind KP) from ap[]
    auto tile_step = [&](auto vt_c, auto kp_c, auto next_c, f32x16 (&an)[TT], f32x16 (&ap)[TT], Frag (&rn)[TT][2],
                         const unsigned char* st, int ftn, int ftp) {
        constexpr bool VT = decltype(vt_c)::value;
        constexpr int KP = decltype(kp_c)::value;
        constexpr bool NEXT = decltype(next_c)::value;
        // ---- epilogue state of tile ftp
        const int nbp = ftp * 32;
        const int so = (ftp - ft_begin) * 32;
        // OUT: bias of four features, V: 1/std of four tokens; the group after the one in use is
        // already on its way from LDS (c4n, rs4n), so that no step waits for it
        float4 c4 = make_float4(0.f, 0.f, 0.f, 0.f), c4n = c4;
        float4 rs4[TT], rs4n[TT];
        auto fetch_group = [&](int g) {
            if constexpr (KP == TK_OUT) {
                c4n = *reinterpret_cast<const float4*>(s_cn + so + 8 * g + 4 * hf);
            } else if constexpr (KP == TK_V) {
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
                    rs4n[tt] = *reinterpret_cast<const float4*>(s_stat + (wave * TT + tt) * 64 + 32 + 8 * g + 4 * hf);
            }
        };
        if constexpr (KP == TK_OUT || KP == TK_V) fetch_group(0);
        uint32_t pk[TT][8];
        float pend[TT];
        size_t qk_off[TT];
        int hlim = 0;
        if constexpr (KP == TK_BIAS) {
            hlim = a.H - 4 * hf;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                qk_off[tt] = (size_t)(a.r0 + tok_rl[tt]) * a.Lp + tok_l[tt] + (size_t)(4 * hf) * a.Lq * a.Lp;
        }
        // value v of the lane: one multiplication by 1/std (the matrix core has already added the
        // LayerNorm mean and offset terms), the sigmoid for the gate, bf16
        auto epi_value = [&](int v) {
            const int g = v >> 2, e = v & 3;
            if constexpr (KP == TK_OUT || KP == TK_V) {
                if (e == 0) {
                    c4 = c4n;
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) rs4[tt] = rs4n[tt];
                    if (g < 3) fetch_group(g + 1);
                }
            }
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                float t;
                if constexpr (KP == TK_OUT) {
                    t = ap[tt][v] + (e == 0 ? c4.x : (e == 1 ? c4.y : (e == 2 ? c4.z : c4.w)));
                } else if constexpr (KP == TK_V) {
                    // lane = feature, value = token 8g + 4hf + e
                    t = ap[tt][v] * (e == 0 ? rs4[tt].x : (e == 1 ? rs4[tt].y : (e == 2 ? rs4[tt].z : rs4[tt].w)));
                } else {
                    t = ap[tt][v] * rstd[tt];
                }
                if constexpr (KP == TK_GATE) t = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-t * kLog2e));
                if constexpr (KP == TK_BIAS) {
                    // pair bias: feature = head, token (rl, l) = pair (q, k)
                    const int hu = 8 * g + e;                    // head of the lower half-wave
                    if (hu < hlim) a.bias[qk_off[tt] + (size_t)hu * a.Lq * a.Lp] = t;
                } else {
                    // (the empty statements pin the arithmetic to this contraction step: the
                    // compiler would otherwise sink it below the matrix-core instructions)
                    if (v & 1) {
                        pk[tt][v >> 1] = pack2(pend[tt], t);
                        asm volatile("" : "+v"(pk[tt][v >> 1]));
                    } else {
                        pend[tt] = t;
                        asm volatile("" : "+v"(pend[tt]));
                    }
                }
            }
        };
        // ---- the pipeline: KC steps over the weight tile, then the extra piece (PROJ)
        Frag wf[KC];
        Frag waug;
        if constexpr (NEXT) {
#pragma unroll
            for (int s = 0; s < AHEAD; ++s) wf[s].u = *reinterpret_cast<const uint4*>(st + (rd0 ^ (32u * s)));
            if constexpr (PROJ) waug.u = s_aug[(ftn - ft_begin) * 32 + col];
        }
#pragma unroll
        for (int s = 0; s < KC; ++s) {
            if constexpr (NEXT) {
                if (s + AHEAD < KC) wf[s + AHEAD].u = *reinterpret_cast<const uint4*>(st + (rd0 ^ (32u * (s + AHEAD))));
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    f32x16 c = an[tt];
                    if (s == 0) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) c[v] = 0.f;
                    }
                    if constexpr (VT) an[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[tt][s].v, wf[s].v, c, 0, 0, 0);
                    else an[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[s].v, xa[tt][s].v, c, 0, 0, 0);
                }
            }
            if constexpr (KP != -1) {
#pragma unroll
                for (int vv = 0; vv < VPC; ++vv) epi_value(s * VPC + vv);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (NEXT && PROJ) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                if constexpr (VT) an[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xaug[tt].v, waug.v, an[tt], 0, 0, 0);
                else an[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(waug.v, xaug[tt].v, an[tt], 0, 0, 0);
            }
        }
        if constexpr (NEXT && RES) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                an[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sel[0].v, rn[tt][0].v, an[tt], 0, 0, 0);
                an[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sel[1].v, rn[tt][1].v, an[tt], 0, 0, 0);
            }
        }
        // ---- stores of tile ftp
        if constexpr (KP == TK_V) {
            const size_t head_off = (size_t)((nbp - 2 * a.Hd) >> a.dsh) * LpD2;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                merge_halves(pk[tt][0], pk[tt][2]);
                merge_halves(pk[tt][1], pk[tt][3]);
                merge_halves(pk[tt][4], pk[tt][6]);
                merge_halves(pk[tt][5], pk[tt][7]);
                // v^T tiled by 32 keys: [row][head][l / 32][e][l % 32]
                bf16_t* tile = a.vt + (row_base[tt] + head_off + (size_t)l0v[tt]);
                *reinterpret_cast<uint4*>(tile + v_lane) = make_uint4(pk[tt][0], pk[tt][1], pk[tt][2], pk[tt][3]);
                *reinterpret_cast<uint4*>(tile + v_lane + 16) = make_uint4(pk[tt][4], pk[tt][5], pk[tt][6], pk[tt][7]);
            }
            n_stores += 2 * TT;
        } else if constexpr (KP == TK_Q || KP == TK_GATE || KP == TK_OUT) {
            // features f .. f+7 and f+16 .. f+23 (f = first feature of the tile + 8 hf): uniform part of their place
            size_t u0 = (size_t)nbp, u1 = (size_t)nbp + 16;               // out: [token][N]
            bf16_t* base = a.out;
            if constexpr (PROJ) {                                          // q, k, gate: [row][head][l][d]
                const int kind = (nbp >= a.Hd) + (nbp >= 2 * a.Hd) + (nbp >= 3 * a.Hd);
                const int f = nbp - kind * a.Hd;
                u0 = (size_t)(f >> a.dsh) * LpD2 + (f & (a.D - 1));
                u1 = (size_t)((f + 16) >> a.dsh) * LpD2 + ((f + 16) & (a.D - 1));
                base = kind == 0 ? a.q : (kind == 1 ? a.k : a.g);
            }
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                merge_halves(pk[tt][0], pk[tt][2]);
                merge_halves(pk[tt][1], pk[tt][3]);
                merge_halves(pk[tt][4], pk[tt][6]);
                merge_halves(pk[tt][5], pk[tt][7]);
                bf16_t* rowp = base + row_base[tt];
                if (PROJ || tok_valid[tt]) {
                    *reinterpret_cast<uint4*>(rowp + u0 + t_lane[tt]) = make_uint4(pk[tt][0], pk[tt][1], pk[tt][2], pk[tt][3]);
                    *reinterpret_cast<uint4*>(rowp + u1 + t_lane[tt]) = make_uint4(pk[tt][4], pk[tt][5], pk[tt][6], pk[tt][7]);
                }
                if (PROJ || any_valid[tt]) n_stores += 2;     // (wave-uniform: the instructions were issued)
            }
        }
    };
    // kind of tile ft: q and k share their epilogue
    auto kind_of = [&](int ft) -> int {
        if constexpr (!PROJ) return TK_OUT;
        if (ft >= a.nt_main) return TK_BIAS;
        const int k = (ft * 32 >= a.Hd) + (ft * 32 >= 2 * a.Hd) + (ft * 32 >= 3 * a.Hd);
        return k == TK_K ? TK_Q : k;
    };
    using std::integral_constant;
    auto run_step = [&](int kn, int kp, f32x16 (&an)[TT], f32x16 (&ap)[TT], Frag (&rn)[TT][2], const unsigned char* st,
                        int ftn, int ftp) {
#define FF_STEP(KPV)                                                                                                         \
    do {                                                                                                                     \
        if (kn < 0) tile_step(integral_constant<bool, false>{}, integral_constant<int, KPV>{},                               \
                              integral_constant<bool, false>{}, an, ap, rn, st, ftn, ftp);                                        \
        else if (kn == TK_V) tile_step(integral_constant<bool, true>{}, integral_constant<int, KPV>{},                       \
                                       integral_constant<bool, true>{}, an, ap, rn, st, ftn, ftp);                                \
        else tile_step(integral_constant<bool, false>{}, integral_constant<int, KPV>{}, integral_constant<bool, true>{}, an, \
                       ap, rn, st, ftn, ftp);                                                                                     \
    } while (0)
        if constexpr (PROJ) {
            switch (kp) {
                case TK_Q: FF_STEP(TK_Q); break;
                case TK_V: FF_STEP(TK_V); break;
                case TK_GATE: FF_STEP(TK_GATE); break;
                case TK_BIAS: FF_STEP(TK_BIAS); break;
                default: FF_STEP(-1); break;
            }
        } else {
            if (kp == TK_OUT) FF_STEP(TK_OUT);
            else FF_STEP(-1);
        }
#undef FF_STEP
    };

    if constexpr (PROJ) {
        // LayerNorm statistics of the raw rows (token_stats)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            float mu, var;
            token_stats<KC>(xa[tt], K, a.eps, mu, var);
            rstd[tt] = tok_valid[tt] ? rsqrtf(var) : 0.f;
            const float m = tok_valid[tt] ? -mu : 0.f, r = var * rstd[tt];
            const float m_hi = bf16_round(m), m_lo = bf16_round(m - m_hi);
            const float r_hi = bf16_round(r), r_lo = bf16_round(r - r_hi);
            if (hf == 0) {
                xaug[tt].u = make_uint4(pack2(m_hi, m_hi), pack2(m_lo, r_hi), pack2(r_hi, r_lo), 0u);
                s_stat[((wave * TT + tt) * 2 + 1) * 32 + col] = rstd[tt];
            }
        }
    }

    const int n_it = (ft_end - ft_begin + NS - 1) / NS;
    int kp = -1, ftp = ft_begin;
    bool last_in_1 = false;
    for (int it = 0; it < n_it; ++it) {
        const int ftb = ft_begin + it * NS;
        const bool two = ftb + 1 < ft_end;
        const unsigned char* st = s_w + ((it & 1) * NS) * STAGE;
        run_step(kind_of(ftb), kp, acc[0], acc[1], ra, st, ftb, ftp);
        kp = kind_of(ftb);
        ftp = ftb;
        last_in_1 = false;
        if constexpr (RES) {
            load_res(ra, ftb + NS);
            n_stores += 2 * TT;
        }
        if (two) {
            run_step(kind_of(ftb + 1), kp, acc[1], acc[0], rb, st + STAGE, ftb + 1, ftp);
            kp = kind_of(ftb + 1);
            ftp = ftb + 1;
            last_in_1 = true;
            if constexpr (RES) {
                load_res(rb, ftb + 1 + NS);
                n_stores += 2 * TT;
            }
        }
        if (it + 1 >= n_it) break;
        // Order of this wavefront's memory operations: ... L(i+1), S, L(i+2), S, ... (L = tile loads
        // of a step, S = the stores issued during one step).  The next step needs L(it+1):
        // everything but the stores issued after it, those of this step, must have completed.
        // After the barrier all wavefronts have their share of L(it+1) in LDS and have finished
        // reading this step's half of the ring, which the loads of step it+2 then overwrite.
        wait_vmem_but_last(__builtin_amdgcn_readfirstlane(n_stores));
        __syncthreads();
#pragma unroll
        for (int n = 0; n < NS; ++n) {
            const int ft = ft_begin + (it + 2) * NS + n;
            if (ft < ft_end) issue_tile(ft, (it & 1) * NS + n);
        }
        n_stores = 0;
    }
    // epilogue of the last tile
    if (last_in_1) run_step(-1, kp, acc[0], acc[1], ra, s_w, ftp, ftp);
    else run_step(-1, kp, acc[1], acc[0], ra, s_w, ftp, ftp);
}

// ====================================================================================
// Attention.  Block = RB wavefronts = RB batch rows, same head, same 64 queries: the bias
// tile [64 queries x 64 keys] is staged once per block in LDS and used by all its rows;
// K rows and V^T columns go straight from global memory into operand registers, one tile
// ahead of their use.
//
// The q.k contraction has two extra slots.  Slot A multiplies 1 (key side) with -m_ref
// (query side): the matrix core returns s - m_ref, m_ref being a per-query reference close
// to the running maximum that is raised only when a tile exceeds it by more than kRaise
// (then the accumulators are rescaled).  Slot B multiplies the mask term of the key (0 or
// -inf) with 1.  The softmax denominator is summed by the vector unit from the rounded weights,
// two at a time.
struct AttnArgs {
    const bf16_t *q, *k, *g, *vt;
    bf16_t* o;
    const float* bias;     // [H][Lq][Lp] or NULL
    const float* mask;     // caller's mask or NULL
    int64_t sr, sl;
    int r0, rows, L, Lp, Lq, H, Hd;
    float inv_nq, inv_nqh;   // 1 / (Lp / 64), 1 / (Lp / 64 * H): quotients of item indices below 2^22 without an integer division
};

// keys per bias tile in LDS (one barrier per tile): 64, or 128 for long sequences (GK template parameter)
constexpr int kBiasPad = 4;      // floats added to an LDS bias row: conflict-free 16-byte reads
constexpr float kRaise = 10.f;   // log2 units
constexpr float kOver = 1048576.f;   // 2^20: partial denominator (16 keys) that triggers a raise of the reference

// (bias-free 4-row blocks for head dims below 32 are held to 168 registers, three wavefronts per
// SIMD: d = 8 fits as it is, d = 16 spills fifteen registers and is still 9 % faster; at d = 32 the
// same bound costs more in spills than the third wavefront brings)
template <int D, bool HAS_BIAS, int RB, int GK, bool PERSIST>
__global__ __launch_bounds__(RB * 64, (RB == 4 && !HAS_BIAS && D < 32) ? 3 : 2) void k_attn(AttnArgs a) {
    constexpr int PCX = D / 8;              // index of the 8-slot piece holding the two extra slots
    constexpr int KS = PCX / 2 + 1;         // 16-wide contraction steps
    constexpr int SX = PCX / 2, HX = PCX % 2;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int TPG = GK / 32, kBiasPitch = GK + kBiasPad;
    float* s_bias = reinterpret_cast<float*>(smem);                                  // [2][64][kBiasPitch]

    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // (scalar: so is everything that places the wavefront's item)
    // Work-groups are handed to the 8 XCDs round-robin and each XCD has its own L2.  The blocks
    // that share K and V (same rows and head, different queries) get consecutive slots of ONE
    // XCD, so K and V are fetched into one L2 once instead of once per query block.
    // The grid is persistent: at most one block per set of RB wave slots of a compute unit, each
    // taking the items (RB batch rows x one head x 64 queries) slot, slot + stride, ... of its XCD.
    // The operands of an item's first tiles are fetched while the block still works on the last
    // tile and the epilogue of the item before, so that only the first item of a block waits for
    // memory before its first matrix instruction.
    const int nq = a.Lp >> 6;
    const int n_items = nq * a.H * ((a.rows + RB - 1) / RB);
    const int per_xcd = (n_items + 7) >> 3;
    const int slot_stride = gridDim.x >> 3;
    int slot = blockIdx.x >> 3;
    auto item_at = [&](int sl) __attribute__((always_inline)) -> int {                  // item of slot sl of this XCD, -1 if there is none
        const int lg = (blockIdx.x & 7) * per_xcd + sl;
        return (sl < per_xcd && lg < n_items) ? lg : -1;
    };
    int logical = item_at(slot);
    if (logical < 0) return;                              // (whole block)
    int rl, h, q0;                                        // of the item whose operands are fetched next
    bool row_ok;
    auto place = [&](int lg) __attribute__((always_inline)) {
        // lg = (block of RB rows * H + head) * nq + query tile; float quotients, corrected by one
        // where the rounding went the wrong way (exact for lg < 2^22, which the host checks)
        const int nqh = nq * a.H;
        int rb = (int)(((float)lg + 0.5f) * a.inv_nqh);
        rb -= rb * nqh > lg;
        rb += (rb + 1) * nqh <= lg;
        const int rem = lg - rb * nqh;
        int hh = (int)(((float)rem + 0.5f) * a.inv_nq);
        hh -= hh * nq > rem;
        hh += (hh + 1) * nq <= rem;
        // (the float quotients pass through vector registers: back to scalar ones, so that every
        // address built from them has a scalar base)
        const int rl_raw = __builtin_amdgcn_readfirstlane(rb) * RB + wave;
        row_ok = rl_raw < a.rows;
        rl = row_ok ? rl_raw : a.rows - 1;
        h = __builtin_amdgcn_readfirstlane(hh);
        q0 = (rem - h * nq) * 64;
    };
    place(logical);
    const bool xlane = hf == HX;            // this lane carries the extra slots in step SX
    // Addresses: every tensor of this kernel has Lp*D elements per (batch row, head); item_off is
    // that block's element offset (scalar), the per-lane parts are 32-bit byte offsets that never change.
    size_t item_off = 0;
    // permuted key of S^T row m = col: rows 8g + 4b + e hold key 16*(g/2) + 8b + 4*(g%2) + e
    const int kperm = 16 * (col >> 4) + 8 * ((col >> 2) & 1) + 4 * ((col >> 3) & 1) + (col & 3);
    const uint32_t qg_lane = (uint32_t)(col * D + 8 * hf) * 2;                       // q, o: query col, elements 8hf..
    const uint32_t k_lane = (uint32_t)(kperm * D + 8 * hf) * 2;                      // k: key kperm of a tile
    const uint32_t v_lane = (uint32_t)((col < D ? col : 0) * 32 + 8 * hf) * 2;       // v^T: element col, keys 8hf..
    const uint32_t gate_lane = (uint32_t)(col * D + 4 * hf) * 2;                     // gate: query col, elements 4hf..

    // ---- Q operand fragments: B operand, lane = query, 8 consecutive e
    Frag qf[2][KS];
    auto fetch_q = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const bf16_t* qp = a.q + item_off + (size_t)(q0 + 32 * j) * D;      // (uniform; query q0 + 32j + col < Lp)
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                qf[j][s].u = make_uint4(0, 0, 0, 0);
                if (2 * s + hf < PCX) qf[j][s].u = ldg16(qp + 16 * s, qg_lane);
            }
        }
    };

    // ---- bias tile pipeline: [64 queries][GK keys]; GK/4 threads per row, RPP rows per pass
    constexpr int TPR = GK / 4, RPP = RB * 64 / TPR, BP = 64 / RPP;
    static_assert(BP == 2 || BP == 4, "bias tile passes");
    const int b_row = tid / TPR, b_c4 = tid % TPR;
    const float* bias_t = nullptr;            // (scalar) row q0 of the item's head
    const uint32_t b_lane = (uint32_t)(b_row * a.Lp) * 4;
    float* s_bias_t = s_bias + (size_t)b_row * kBiasPitch + 4 * b_c4;
    // (named registers: an array captured by a lambda would be spilled to scratch)
    float4 bq0, bq1, bq2, bq3;
    auto load_bias = [&](int g) __attribute__((always_inline)) {
        int colk = GK * g + 4 * b_c4;              // (a last group that is only half there repeats valid keys)
        if (colk > a.Lp - 4) colk = a.Lp - 4;
        const uint32_t off = b_lane + (uint32_t)colk * 4;
        auto ld = [&](const float* base) __attribute__((always_inline)) {
            return *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(base) + off);
        };
        bq0 = ld(bias_t);
        bq1 = ld(bias_t + (size_t)RPP * a.Lp);
        if constexpr (BP > 2) {
            bq2 = ld(bias_t + (size_t)(2 * RPP) * a.Lp);
            bq3 = ld(bias_t + (size_t)(3 * RPP) * a.Lp);
        }
    };
    auto store_bias = [&](int buf) __attribute__((always_inline)) {
        float* sp = s_bias_t + (size_t)buf * 64 * kBiasPitch;
        *reinterpret_cast<float4*>(sp) = bq0;
        *reinterpret_cast<float4*>(sp + RPP * kBiasPitch) = bq1;
        if constexpr (BP > 2) {
            *reinterpret_cast<float4*>(sp + 2 * RPP * kBiasPitch) = bq2;
            *reinterpret_cast<float4*>(sp + 3 * RPP * kBiasPitch) = bq3;
        }
    };

    // k is [row][head][l][d], v^T is [row][head][l / 32][e][l % 32]: a 32-key tile of either is one
    // contiguous block of 64*D bytes
    const float* mp;
    const bool has_mask = a.mask != nullptr;
    const int msl = (int)a.sl;                     // (1 or n_b)
    constexpr int kstep = 32 * D;
    auto set_pointers = [&]() __attribute__((always_inline)) {             // operands of the item (rl, h, q0)
        item_off = (size_t)(rl * a.H + h) * a.Lp * D;
        mp = has_mask ? a.mask + (int64_t)(a.r0 + rl) * a.sr : nullptr;
        if constexpr (HAS_BIAS) bias_t = a.bias + ((size_t)h * a.Lq + q0) * a.Lp;
    };
    set_pointers();
    fetch_q();
    if constexpr (HAS_BIAS) load_bias(0);      // (stored to LDS after the first K and V loads have been issued)

    // Software pipeline over 32-key tiles i:
    //   K(i+2), mask(i+2), V(i+1) are in flight (global -> registers) while
    //   S^T(i+1) = K(i+1) Q^T runs on the matrix cores while
    //   the vector unit takes the exponentials of tile i, followed by O^T += V^T(i) P^T(i).
    // K and V use two register sets each (even / odd tiles); nothing looks at a loaded value
    // before its use.  The bias tile in LDS covers 64 keys (an even and an odd tile).
    Frag kb0[KS], kb1[KS], vb0[2], vb1[2];
    float mv0 = 1.f, mv1 = 1.f;
    auto fetch_k = [&](Frag (&kb)[KS], float& mv, int kt) __attribute__((always_inline)) {
        // (the empty statement hides the lane offset from the loop optimiser, which would otherwise
        // add it to the tile's base once and carry a 64-bit pointer per lane through the loop)
        // and the tile index from being folded into an immediate offset that does not fit the instruction)
        uint32_t lane_off = k_lane;
        asm volatile("" : "+v"(lane_off));
        int kts = kt;
        asm volatile("" : "+s"(kts));
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            kb[s].u = make_uint4(0, 0, 0, 0);
            if (2 * s + hf < PCX) kb[s].u = ldg16(a.k + item_off + (size_t)kts * kstep + 16 * s, lane_off);
        }
        // mask value of the lane's key (whoever uses mv pins it first, or the compiler compares it
        // with zero right here and waits for every load just issued).  Keys beyond L - 1 read the
        // entry of key L - 1; scalar base of the tile + 32-bit lane offset.
        mv = 1.f;
        if (has_mask) {
            int k0 = 32 * kts;
            if (k0 > ((a.L - 1) & ~31)) k0 = (a.L - 1) & ~31;
            const int lk = kperm < a.L - 1 - k0 ? kperm : a.L - 1 - k0;          // >= 0
            mv = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(mp + (int64_t)k0 * msl) +
                                                 (uint32_t)(lk * msl) * 4u);
        }
    };
    auto fetch_v = [&](Frag (&vb)[2], int kt) __attribute__((always_inline)) {
        uint32_t lane_off = v_lane;
        asm volatile("" : "+v"(lane_off));
        int kts = kt;
        asm volatile("" : "+s"(kts));
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            vb[c].u = make_uint4(0, 0, 0, 0);
            if (col < D) vb[c].u = ldg16(a.vt + item_off + (size_t)kts * kstep + 16 * c, lane_off);
        }
    };

    f32x16 o_acc[2];
    float m_ref[2], l_run[2];
    bool first = true;
    int gbase = 0;          // bias groups staged so far (all items): group g of the item uses LDS buffer (gbase + g) & 1

    // S^T of tile kt into sa in two parts: the bias tile as accumulator input (LDS reads, issued
    // early: the loads of the next K and V tiles hide their latency), then the contraction, which
    // returns whether any key of the tile is valid
    auto qk_bias = [&](int kt, f32x16 (&sa)[2]) __attribute__((always_inline)) {
        const float* sb = s_bias + (size_t)((kt / TPG + gbase) & 1) * 64 * kBiasPitch;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            if constexpr (HAS_BIAS) {
                const float* br = sb + (size_t)(32 * j + col) * kBiasPitch + 32 * (kt % TPG) + 8 * hf;
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const float4 x4 = *reinterpret_cast<const float4*>(br + 16 * c + 4 * i);
                        sa[j][8 * c + 4 * i] = x4.x; sa[j][8 * c + 4 * i + 1] = x4.y;
                        sa[j][8 * c + 4 * i + 2] = x4.z; sa[j][8 * c + 4 * i + 3] = x4.w;
                    }
            }
        }
    };
    auto qk_mma = [&](Frag (&kb)[KS], float mv, int kt, f32x16 (&sa)[2]) __attribute__((always_inline)) -> bool {
        asm volatile("" : "+v"(mv));
        const bool key_valid = (!has_mask || mv != 0.f) && 32 * kt + kperm < a.L;
        if (!__any(key_valid)) return false;
        if (xlane) kb[SX].w[0] = key_valid ? 0x00003f80u : 0xff803f80u;   // (1.0, mask term)
        if constexpr (!HAS_BIAS) {          // (zero accumulator input: a constant operand of the first step)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) sa[j][v] = 0.f;
        }
        // the two query tiles alternate, so that no matrix-core instruction waits for the one before it
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                sa[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb[s].v, qf[j][s].v, sa[j], 0, 0, 0);
        return true;
    };
    // Exponentials of tile sa and O^T update.
    // FUSE = false: sn is the next tile, already issued with the old reference if sn_live.
    // FUSE = true: the next tile's contraction S^T(ktn) = K Q^T (operands kbn, mask value mvn) is
    // issued from in here, one matrix instruction after every other group of exponentials, so that
    // the wavefront never queues behind its own matrix instructions (issued back to back, each waits
    // for the matrix core to finish the one before, and the vector instructions behind them wait
    // too).  Query tile 1 of the next tile is contracted while query tile 0 of this one is
    // exponentiated and vice versa: when the reference of a query tile has to be raised, the next
    // tile of that query tile is either complete (then it is corrected, as before) or not begun
    // (then it sees the new reference in the Q operand).  Returns whether the next tile holds a
    // valid key (FUSE) or sn_live.
    auto soft_pv = [&](f32x16 (&sa)[2], Frag (&vb)[2], f32x16 (&sn)[2], bool sn_live, auto fuse_c, Frag (&kbn)[KS],
                       float mvn, int ktn) __attribute__((always_inline)) -> bool {
        constexpr bool FUSE = decltype(fuse_c)::value;
        bool next_live = sn_live;
        if constexpr (FUSE) {
            asm volatile("" : "+v"(mvn));
            const bool key_valid = (!has_mask || mvn != 0.f) && 32 * ktn + kperm < a.L;
            next_live = __any(key_valid);           // (a tile without valid keys is still contracted: all -inf, never used)
            if (xlane) kbn[SX].w[0] = key_valid ? 0x00003f80u : 0xff803f80u;   // (1.0, mask term)
            if constexpr (!HAS_BIAS) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) sn[j][v] = 0.f;
            }
        }
        // sa holds s - m_ref (masked keys: -inf).  Only the first tile takes the maximum; later tiles
        // are exponentiated as they are and a partial denominator beyond kOver (some s - m_ref above
        // about 16) sends the query tile through raise_ref afterwards: rare, and the common tile
        // saves the sixteen max operations per query.  (For head dims below 32 a row of ones in V^T
        // could let the matrix core sum the denominator, but an overflow would then already be
        // accumulated, so every tile would need its maximum: 3 % slower at d = 8 in a same-box comparison.)
        auto tile_max = [&](int j) __attribute__((always_inline)) -> float {
            float mx = sa[j][0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sa[j][v]);
            return fmaxf(mx, other_half(mx));
        };
        auto raise_ref = [&](int j, float tmax, bool always, bool correct_next) __attribute__((always_inline)) {
            const bool raise = always || tmax > kRaise;
            const float new_ref = raise ? bf16_round(m_ref[j] + tmax) : m_ref[j];
            const float delta = new_ref - m_ref[j];
            m_ref[j] = new_ref;
            const float sc = first ? 1.f : __builtin_amdgcn_exp2f(-delta);   // first: nothing accumulated yet
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                o_acc[j][v] *= sc;
                sa[j][v] -= delta;
            }
            if (correct_next) {
#pragma unroll
                for (int v = 0; v < 16; ++v) sn[j][v] -= delta;
            }
            l_run[j] *= sc;
            if (xlane) qf[j][SX].w[0] = pack2(-new_ref, 1.f);
        };
        if (first) {
            const float t0 = tile_max(0), t1 = tile_max(1);
            if (first || __any(t0 > kRaise || t1 > kRaise)) {
                raise_ref(0, t0, first, !FUSE && sn_live);      // (FUSE: the next tile has not begun)
                raise_ref(1, t1, first, !FUSE && sn_live);
                first = false;
            }
        }
        // matrix instruction m of the next tile's query tile jn (FUSE)
        auto next_mma = [&](int jn, int m) __attribute__((always_inline)) {
            sn[jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kbn[m].v, qf[jn][m].v, sn[jn], 0, 0, 0);
        };
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            Frag pf[2];
            float lt = 0.f;
            // eight groups of two exponentials, a pack and a partial denominator; with `weave` a
            // matrix instruction of the other query tile follows every other group, and the fences
            // keep the compiler from gathering them again
            auto exponentiate = [&](auto weave_c) __attribute__((always_inline)) {
                constexpr bool WEAVE = decltype(weave_c)::value;
                lt = 0.f;
                if constexpr (!WEAVE) {
#pragma unroll
                    for (int c = 0; c < 2; ++c)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float p0 = __builtin_amdgcn_exp2f(sa[j][8 * c + 2 * i]);
                            const float p1 = __builtin_amdgcn_exp2f(sa[j][8 * c + 2 * i + 1]);
                            pf[c].w[i] = pack2(p0, p1);
                            // denominator from the rounded weights, two per instruction
                            lt = add_pair(pf[c].w[i], lt);
                        }
                } else {
                    // (between two fences: the exponentials of group g + 1, then pack and partial
                    // denominator of group g, whose exponentials have had a group's time to finish)
                    float e0 = __builtin_amdgcn_exp2f(sa[j][0]), e1 = __builtin_amdgcn_exp2f(sa[j][1]);
#pragma unroll
                    for (int g = 0; g < 8; ++g) {
                        float n0 = 0.f, n1 = 0.f;
                        if (g < 7) {
                            n0 = __builtin_amdgcn_exp2f(sa[j][2 * g + 2]);
                            n1 = __builtin_amdgcn_exp2f(sa[j][2 * g + 3]);
                            asm volatile("" : "+v"(n0), "+v"(n1));
                        }
                        uint32_t& w = pf[g >> 2].w[g & 3];
                        w = pack2(e0, e1);
                        lt = add_pair(w, lt);
                        asm volatile("" : "+v"(w));
                        if ((g & 1) && (g >> 1) < KS) next_mma(1 - j, g >> 1);
                        __builtin_amdgcn_sched_barrier(0);
                        e0 = n0;
                        e1 = n1;
                    }
                }
            };
            exponentiate(std::integral_constant<bool, FUSE>{});
            if (__any(!(lt <= kOver))) {
                // (FUSE: the next tile of query tile 1 was issued during query tile 0, that of
                // query tile 0 is issued during query tile 1)
                raise_ref(j, tile_max(j), false, FUSE ? j == 1 : sn_live);
                exponentiate(std::integral_constant<bool, false>{});
            }
            l_run[j] += lt;
#pragma unroll
            for (int c = 0; c < 2; ++c)
                o_acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb[c].v, pf[c].v, o_acc[j], 0, 0, 0);
        }
        return next_live;
    };

    const int nt = a.Lp >> 5;               // even
    fetch_k(kb0, mv0, 0);
    fetch_k(kb1, mv1, 1);
    fetch_v(vb0, 0);
    f32x16 s0[2], s1[2];
    uint2 gate[2][4];       // gate values of the item's queries, fetched during its last tile
  for (;;) {
    // ---- an item begins: its Q, K(0), K(1), V(0) and first bias group are on their way or here
    const int e_rl = rl, e_h = h, e_q0 = q0;        // the epilogue's copy: (rl, h, q0) move on to the next item before it
    const bool e_row_ok = row_ok;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        m_ref[j] = 0.f;
        l_run[j] = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[j][v] = 0.f;
        if (xlane) qf[j][SX].w[0] = 0x3f800000u;        // (-m_ref = 0, 1.0)
    }
    first = true;
    if constexpr (HAS_BIAS) {
        // (group 0 goes to the buffer that the last group of the item before does not use; every
        // wavefront finished with the group before that one when it passed the last barrier)
        store_bias(gbase & 1);
        if (TPG == 2 && nt > 2) load_bias(1);
    }
    __syncthreads();                        // bias group 0 is in LDS
    qk_bias(0, s0);
    bool live0 = qk_mma(kb0, mv0, 0, s0), live1 = false;
    // (long sequences, PERSIST = false: one item per block.  There the start of an item is a few per
    // cent of its time, and blocks handed out as compute units fall free even out the differences
    // between compute units that a fixed share of 24 long items per block adds up: 3 % at 1024 keys)
    const int next = PERSIST ? item_at(slot + slot_stride) : -1;
    // The bias of key group g (TPG tiles) sits in LDS buffer (gbase + g) & 1.  It is loaded to registers one
    // and a half iterations before tile g*TPG is first touched, stored and published (the only
    // barrier of the group) at the end of the even half of the iteration before.
    // (the last pair of tiles has a body of its own: the loop proper then holds no load that
    // depends on a condition, which keeps the compiler's wait counts exact)
    // Head dims below 32: the next tile's contraction is issued from inside the exponentials (soft_pv,
    // FUSE).  Measured at 1024 keys, d = 8: 702 -> 671 us.  At d = 32, with three times the matrix
    // instructions per tile, the same weave is 2 % slower than the contraction issued ahead in one go.
    constexpr bool WEAVE_QK = D < 32;
    auto tile_pair = [&](int i, auto last_c) __attribute__((always_inline)) {
        constexpr bool LAST = decltype(last_c)::value;
        // ---- even tile i: K(i+2) -> set 0, V(i+1) -> set 1, S^T(i+1) -> s1, exponentials of s0
        qk_bias(i + 1, s1);
        if constexpr (!LAST) fetch_k(kb0, mv0, i + 2);
        fetch_v(vb1, i + 1);
        using std::integral_constant;
        if constexpr (LAST) {
            // no tile i+2.  The gate values of the epilogue set out, then the operands of the next
            // item's first tiles as their registers fall free: K set 0 here, K set 1, V set 0, the
            // bias registers and Q (its last matrix instruction has been issued; if the last
            // exponentials still raise the reference, what they write into the Q operand is
            // overwritten when the next item begins) half a pair later.  A block's last item
            // fetches its own first tiles again instead: loads that do not depend on a condition
            // keep the compiler's wait counts exact, so that the epilogue waits for the gate
            // values only.
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16_t* gp = a.g + item_off + (size_t)(q0 + 32 * j) * D;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    gate[j][g] = make_uint2(0, 0);
                    if (8 * g + 4 * hf < D) gate[j][g] = ldg8(gp + 8 * g, gate_lane);
                }
            }
            if constexpr (PERSIST) {
                place(next >= 0 ? next : logical);
                set_pointers();
                fetch_k(kb0, mv0, 0);
            }
        }
        if constexpr (WEAVE_QK) {
            if (live0) live1 = soft_pv(s0, vb0, s1, false, integral_constant<bool, true>{}, kb1, mv1, i + 1);
            else live1 = qk_mma(kb1, mv1, i + 1, s1);
        } else {
            live1 = qk_mma(kb1, mv1, i + 1, s1);
            if (live0) soft_pv(s0, vb0, s1, live1, integral_constant<bool, false>{}, kb1, mv1, 0);
        }
        if constexpr (HAS_BIAS && !LAST) {
            if ((i + 2) % TPG == 0) {
                store_bias(((i + 2) / TPG + gbase) & 1);
                __syncthreads();
            }
        }
        // ---- odd tile i+1: K(i+3) -> set 1, V(i+2) -> set 0, S^T(i+2) -> s0, exponentials of s1
        live0 = false;
        if constexpr (!LAST) {
            qk_bias(i + 2, s0);
            fetch_k(kb1, mv1, i + 3);
            fetch_v(vb0, i + 2);
            if constexpr (HAS_BIAS) {
                if ((i + 4) % TPG == 0 && i + 4 < nt) load_bias((i + 4) / TPG);
            }
            if constexpr (WEAVE_QK) {
                if (live1) live0 = soft_pv(s1, vb1, s0, false, integral_constant<bool, true>{}, kb0, mv0, i + 2);
                else live0 = qk_mma(kb0, mv0, i + 2, s0);
            } else {
                live0 = qk_mma(kb0, mv0, i + 2, s0);
                if (live1) soft_pv(s1, vb1, s0, live0, integral_constant<bool, false>{}, kb0, mv0, 0);
            }
        } else {
            if constexpr (PERSIST) {
                fetch_k(kb1, mv1, 1);
                fetch_v(vb0, 0);
                if constexpr (HAS_BIAS) load_bias(0);
                fetch_q();
            }
            if (live1) soft_pv(s1, vb1, s0, false, integral_constant<bool, false>{}, kb0, mv0, 0);
        }
    };
    for (int i = 0; i + 2 < nt; i += 2) tile_pair(i, std::integral_constant<bool, false>{});
    tile_pair(nt - 2, std::integral_constant<bool, true>{});

    // ---- epilogue: normalise, gate, store.  o_acc[j]: lane = query, register v = e = 8*(v/4) + 4*hf + v%4
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const float l_tot = l_run[j] + other_half(l_run[j]);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        const int qi = e_q0 + 32 * j + col;                       // < Lp
        // gate and context are head-major [row][head][l][d]: the wave's 32 queries are one
        // contiguous block of 64*D bytes
        bf16_t* op = a.o + (size_t)(e_rl * a.H + e_h) * a.Lp * D + (size_t)(e_q0 + 32 * j) * D;   // (uniform)
        uint32_t pk[8];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint2 gr = gate[j][g];              // elements 8g + 4hf .. + 3 (zero beyond D)
            pk[2 * g] = pack2(o_acc[j][4 * g] * inv * lo_f32(gr.x), o_acc[j][4 * g + 1] * inv * hi_f32(gr.x));
            pk[2 * g + 1] = pack2(o_acc[j][4 * g + 2] * inv * lo_f32(gr.y), o_acc[j][4 * g + 3] * inv * hi_f32(gr.y));
        }
        merge_halves(pk[0], pk[2]);      // lower half-wave: e 0..7, upper: e 8..15
        merge_halves(pk[1], pk[3]);
        merge_halves(pk[4], pk[6]);      // lower: e 16..23, upper: e 24..31
        merge_halves(pk[5], pk[7]);
        if (e_row_ok && qi < a.L) {
            if (8 * hf < D) stg16(op, qg_lane, make_uint4(pk[0], pk[1], pk[2], pk[3]));
            if (16 + 8 * hf < D) stg16(op + 16, qg_lane, make_uint4(pk[4], pk[5], pk[6], pk[7]));
        }
    }
    if (next < 0) break;
    logical = next;
    slot += slot_stride;
    gbase += (nt + TPG - 1) / TPG;
  }
}

// ====================================================================================
// Projection and attention in one kernel, for sequences of at most 256 positions with head
// dimension 32 (the row-wise and triangle attentions of the training crop, Section 5.2's merged
// projections feeding its fused softmax): a block takes two batch rows and one head, projects
// that head's q, k, v and gate for all tokens of the two rows straight from the raw input (the
// LayerNorm folded into the weights as in k_gemm) and attends at once.  q and the gate never
// leave the registers, k and v^T live in LDS, so that of the five tensors k_gemm<PROJ> hands to
// k_attn through HBM only the gated context is ever written.
//
// Wavefront w owns tokens 32w .. 32w+31 of both rows: as projection tokens first, as queries
// afterwards.  A projection tile leaves the matrix core with the lane = token, register =
// feature 8*(v/4) + 4*hf + v%4 layout; packed in register order it is a valid B operand of
// S^T = K Q^T as long as the key side uses the same order of the contraction, which is how the k
// tile is written to LDS (one 16-byte piece per step and half-wave).  The gate has the layout
// of O^T already.  v is computed with the operands swapped (lane = feature), which is the
// layout of a row of v^T.  The bias tile of a key tile is loaded once and used as accumulator
// input for both rows.
//
// LDS: the head's four folded 32 x K weight tiles (row pitch 2K + 16 bytes), their extra pieces,
// k [2][256][80 bytes] (four pieces of the contraction and the piece with 1 and the mask term),
// v^T [2][32][528 bytes], 1/std of the tokens, one flag per (row, key tile) that tells whether
// the tile holds a valid key, and 2 KiB per wavefront through which the raw tokens, fetched as
// whole 128-byte lines, are turned into matrix-core operands.  With 256 channels that is 159 KiB
// of the compute unit's 160: one block of eight wavefronts per compute unit.
//
// Measured on the training crop of the row-wise attention (128 x 256 tokens, 8 heads): 50 us
// against 34 + 31 us for k_gemm<PROJ> and k_attn.  No unit is saturated (LDS busy 22 %, matrix
// pipe 25 %, vector unit 39 % of the kernel): in the projections every matrix instruction waits
// for a fresh weight operand from LDS, the attention is paced by the exponentials, and two
// wavefronts per SIMD with one dependent chain each leave a third of the issue slots empty.  Of
// the two wavefronts of a SIMD the older one is served first and finishes each phase about a
// quarter earlier; the block waits for the younger one at both barriers.
struct FusedArgs {
    const bf16_t* x;       // raw input, token (r, l) at (r*sr + l*sl)*K
    int64_t sr, sl;        // token strides of x and of the mask
    int r0, rows, L, Lp, Lq;
    float eps;
    const bf16_t* wp;      // prepared weights [(4*Hd + 32)][K]
    const uint4* aug;      // their extra pieces
    int H, Hd;
    const float* bias;     // tiled (bias_index) or NULL
    const float* mask;     // caller's mask or NULL
    bf16_t* o;             // gated context [rows][H][Lp][32]
};

constexpr int kFuKPitch = 80;       // bytes of a key row in LDS
constexpr int kFuVPitch = 528;      // bytes of a v^T row in LDS: 256 keys and a pad
constexpr int kFuWaves = 8;

static size_t fused_smem_bytes(int kc) {
    return (size_t)4 * 32 * (32 * kc + 16) + 128 * 16 + 2 * 256 * kFuKPitch + 2 * 32 * kFuVPitch + kFuWaves * 2 * 32 * 4 + 64 +
           kFuWaves * 2048;
}

template <int KC, bool HAS_BIAS>
__global__ __launch_bounds__(kFuWaves * 64) void k_proj_attn(FusedArgs a) {
    constexpr int K = 16 * KC, WP = 32 * KC + 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* s_w = smem;                                                  // [4][32][WP]
    uint4* s_aug = reinterpret_cast<uint4*>(s_w + 4 * 32 * WP);                 // [4][32]
    unsigned char* s_k = reinterpret_cast<unsigned char*>(s_aug + 128);         // [2][256][kFuKPitch]
    unsigned char* s_vt = s_k + 2 * 256 * kFuKPitch;                            // [2][32][kFuVPitch]
    float* s_stat = reinterpret_cast<float*>(s_vt + 2 * 32 * kFuVPitch);        // [wave][2][32]
    int* s_live = reinterpret_cast<int*>(s_stat + kFuWaves * 2 * 32);           // [2][8]
    unsigned char* s_st = reinterpret_cast<unsigned char*>(s_live + 16) + (threadIdx.x >> 6) * 2048;   // [wave][16][128]

    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nt = a.Lp >> 5;                               // 32-token tiles of a row: even, at most 8
    const bool active = wave < nt;                          // (wave-uniform)
    // Work-groups go to the 8 XCDs round-robin and each XCD has its own L2: the heads of a row
    // pair run on one XCD at about the same time, so the rows of x come from HBM once.  Item
    // jj*H + h of an XCD is row pair xcd + 8 jj, head h; a block takes the items slot, slot +
    // slots, ...: with the slots a multiple of H its head never changes and the weights are
    // loaded once.
    const int n_rp = (a.rows + 1) >> 1;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
    const int n_local = xcd < n_rp ? ((n_rp - xcd + 7) >> 3) * a.H : 0;
    int h_loaded = -1;
    const int l_tok = 32 * wave + col;
    const bool tok_in = active && l_tok < a.L;
    const bool has_mask = a.mask != nullptr;

    for (int it = slot; it < n_local; it += slots) {
        const int jj = it / a.H, h = it - jj * a.H;
        const int rp = xcd + 8 * jj;
        // ---- raw tokens (row 0 issued first; row 1 follows line by line as the registers fall free),
        // the mask entries.  Eight lanes fetch one 128-byte line of a token (a load with lane =
        // token, the operand layout, touches 64 lines for 1 KiB and the cache looks up one line per
        // cycle: 5 us per item instead of 1.2); raw[m][hh][i] holds line m of the tokens 16hh + 8i +
        // lane/8 of the wavefront's tile, piece lane%8.  Issued before the barrier: the loads are on
        // their way while the block waits for its last wavefront.
        constexpr int NG = KC / 4;              // 128-byte lines per token
        uint4 raw[NG][2][2];
        float mval[2];
        bool row_ok[2];
        int rlv[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int rl = 2 * rp + j;
            row_ok[j] = rl < a.rows;
            rlv[j] = row_ok[j] ? rl : a.rows - 1;
            mval[j] = 1.f;
            if (has_mask && tok_in) mval[j] = a.mask[(int64_t)(a.r0 + rlv[j]) * a.sr + (int64_t)l_tok * a.sl];
        }
        auto fetch_line = [&](int j, int m) __attribute__((always_inline)) {
            const int64_t row_tok = (int64_t)(a.r0 + rlv[j]) * a.sr;
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int l = 32 * wave + 16 * hh + 8 * i + (lane >> 3);
                    const bool in = active && l < a.L;
                    raw[m][hh][i] = make_uint4(0, 0, 0, 0);
                    if (in) raw[m][hh][i] = ldg16(a.x + (row_tok + (int64_t)l * a.sl) * K + (lane & 7) * 8 + 64 * m);
                }
        };
#pragma unroll
        for (int m = 0; m < NG; ++m) fetch_line(0, m);

        if (it != slot) __syncthreads();            // every wavefront has left the item before: k and v^T may be overwritten

        // ---- the head's weight tiles
        if (h != h_loaded) {
            // (128 rows of 2 KC pieces, KC / 2 pieces per thread, up to four loads in flight)
            constexpr int WB = KC / 2 < 4 ? KC / 2 : 4;          // loads in flight per thread
#pragma unroll
            for (int n0 = 0; n0 < KC / 2; n0 += WB) {
                uint4 wv[WB];
#pragma unroll
                for (int n = 0; n < WB; ++n) {
                    const int p = tid + (n0 + n) * kFuWaves * 64;
                    const int row = p / (2 * KC), pp = p - row * (2 * KC);
                    wv[n] = ldg16(a.wp + ((size_t)((row >> 5) * a.Hd + h * 32 + (row & 31)) * K + pp * 8));
                }
#pragma unroll
                for (int n = 0; n < WB; ++n) {
                    const int p = tid + (n0 + n) * kFuWaves * 64;
                    const int row = p / (2 * KC), pp = p - row * (2 * KC);
                    *reinterpret_cast<uint4*>(s_w + row * WP + pp * 16) = wv[n];
                }
            }
            if (tid < 128) s_aug[tid] = a.aug[(tid >> 5) * a.Hd + h * 32 + (tid & 31)];
            h_loaded = h;
            __syncthreads();
        }

        // ---- projections: q and gate stay in registers, k and v^T go to LDS
        Frag qf[2][3];          // (set and used by wavefronts with tokens only)
        uint32_t gpk[2][8];
        if (active) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                // The lines pass through the wavefront's staging area (16 tokens x 128 bytes, the eight
                // pieces of a token rotated by its index: conflict-free) and come back in the operand
                // layout, lane = token, pieces 2s' + hf of line m = contraction steps 4m + s'.  The
                // area is private to the wavefront, whose LDS operations complete in order.
                f32x16 aq, ak, av, ag;
#pragma unroll
                for (int v = 0; v < 16; ++v) aq[v] = ak[v] = av[v] = ag[v] = 0.f;
                const unsigned char* wrow = s_w + col * WP + hf * 16;
                float sum = 0.f, sq = 0.f;
#pragma unroll
                for (int m = 0; m < NG; ++m) {
                    Frag xg[4];
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                        for (int i = 0; i < 2; ++i) {
                            const int tl = 8 * i + (lane >> 3);
                            *reinterpret_cast<uint4*>(s_st + tl * 128 + (((lane & 7) ^ (tl & 7)) * 16)) = raw[m][hh][i];
                        }
                        __builtin_amdgcn_wave_barrier();
                        if ((col >> 4) == hh) {
                            const int tl = col & 15;
#pragma unroll
                            for (int sp = 0; sp < 4; ++sp)
                                xg[sp].u = *reinterpret_cast<const uint4*>(s_st + tl * 128 + (((2 * sp + hf) ^ (tl & 7)) * 16));
                        }
                        __builtin_amdgcn_wave_barrier();
                    }
                    if (j == 0) fetch_line(1, m);         // (the line's registers are free again)
                    // LayerNorm statistics as in token_stats, one line at a time
#pragma unroll
                    for (int sp = 0; sp < 4; ++sp)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            sum = add_pair(xg[sp].w[i], sum);
                            sq = add_pair_sq(xg[sp].w[i], sq);
                        }
#pragma unroll
                    for (int sp = 0; sp < 4; ++sp) {
                        const int st = 4 * m + sp;
                        Frag wq, wk, wv, wg;
                        wq.u = *reinterpret_cast<const uint4*>(wrow + 0 * 32 * WP + 32 * st);
                        wk.u = *reinterpret_cast<const uint4*>(wrow + 1 * 32 * WP + 32 * st);
                        wv.u = *reinterpret_cast<const uint4*>(wrow + 2 * 32 * WP + 32 * st);
                        wg.u = *reinterpret_cast<const uint4*>(wrow + 3 * 32 * WP + 32 * st);
                        aq = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wq.v, xg[sp].v, aq, 0, 0, 0);
                        ak = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wk.v, xg[sp].v, ak, 0, 0, 0);
                        av = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xg[sp].v, wv.v, av, 0, 0, 0);
                        ag = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wg.v, xg[sp].v, ag, 0, 0, 0);
                    }
                }
                sum += other_half(sum);
                sq += other_half(sq);
                const float mu = sum * (1.f / (float)K);
                const float var = fmaxf(sq * (1.f / (float)K) - mu * mu, 0.f) + a.eps;
                const float rstd = tok_in ? rsqrtf(var) : 0.f;
                const float mneg = tok_in ? -mu : 0.f, r = var * rstd;
                const float m_hi = bf16_round(mneg), m_lo = bf16_round(mneg - m_hi);
                const float r_hi = bf16_round(r), r_lo = bf16_round(r - r_hi);
                Frag xaug;
                xaug.u = make_uint4(0, 0, 0, 0);
                if (hf == 0) {
                    xaug.u = make_uint4(pack2(m_hi, m_hi), pack2(m_lo, r_hi), pack2(r_hi, r_lo), 0u);
                    s_stat[(wave * 2 + j) * 32 + col] = rstd;
                }
                const bool key_valid = tok_in && mval[j] != 0.f;
                const bool any_valid = __any(key_valid);
                if (lane == 0) s_live[j * 8 + wave] = any_valid ? 1 : 0;
                {
                    Frag wq, wk, wv, wg;
                    wq.u = s_aug[col];
                    wk.u = s_aug[32 + col];
                    wv.u = s_aug[64 + col];
                    wg.u = s_aug[96 + col];
                    aq = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wq.v, xaug.v, aq, 0, 0, 0);
                    ak = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wk.v, xaug.v, ak, 0, 0, 0);
                    av = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xaug.v, wv.v, av, 0, 0, 0);
                    ag = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wg.v, xaug.v, ag, 0, 0, 0);
                }
                // q: B operand of S^T, step s = registers 8s .. 8s+7; step 2 carries (-m_ref, 1)
                // k: the same pieces into the token's LDS row, then (1, mask term)
                unsigned char* krow = s_k + (j * 256 + l_tok) * kFuKPitch;
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    uint32_t kw[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        qf[j][s].w[i] = pack2(aq[8 * s + 2 * i] * rstd, aq[8 * s + 2 * i + 1] * rstd);
                        kw[i] = pack2(ak[8 * s + 2 * i] * rstd, ak[8 * s + 2 * i + 1] * rstd);
                    }
                    *reinterpret_cast<uint4*>(krow + (2 * s + hf) * 16) = make_uint4(kw[0], kw[1], kw[2], kw[3]);
                }
                qf[j][2].u = make_uint4(hf == 0 ? 0x3f800000u : 0u, 0u, 0u, 0u);            // (-m_ref = 0, 1.0)
                if (hf == 0) {
                    *reinterpret_cast<uint4*>(krow + 64) = make_uint4(key_valid ? 0x00003f80u : 0xff803f80u, 0u, 0u, 0u);   // (1.0, mask term)
                }
                // gate: the layout of O^T
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float g0 = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-(ag[2 * i] * rstd) * kLog2e));
                    const float g1 = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-(ag[2 * i + 1] * rstd) * kLog2e));
                    gpk[j][i] = pack2(g0, g1);
                }
                // v: lane = feature col, register v = token 8*(v/4) + 4*hf + v%4 of the wavefront's tile
                // (1/std of those tokens comes back from LDS: written above by this wavefront, whose LDS
                // operations complete in order)
                __builtin_amdgcn_wave_barrier();
                unsigned char* vrow = s_vt + (j * 32 + col) * kFuVPitch + (32 * wave + 4 * hf) * 2;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 rs = *reinterpret_cast<const float4*>(s_stat + (wave * 2 + j) * 32 + 8 * g + 4 * hf);
                    *reinterpret_cast<uint2*>(vrow + 16 * g) =
                        make_uint2(pack2(av[4 * g] * rs.x, av[4 * g + 1] * rs.y), pack2(av[4 * g + 2] * rs.z, av[4 * g + 3] * rs.w));
                }
            }
        }
        __syncthreads();

        // ---- attention of the wavefront's 32 queries of both rows over the nt key tiles
        if (active) {
            // (the lane's indices anew, opaque to the optimiser: the addresses of this phase would
            // otherwise be computed before the projections and held in registers through them)
            int lane_a = lane;
            asm volatile("" : "+v"(lane_a));
            const int col_a = lane_a & 31, hf_a = lane_a >> 5;
            // permuted key of S^T row m = col (see k_attn): the lane's registers 8c .. 8c+7 then hold
            // the keys 16c + 8hf .. + 7 of the tile
            const int kperm_a = 16 * (col_a >> 4) + 8 * ((col_a >> 2) & 1) + 4 * ((col_a >> 3) & 1) + (col_a & 3);
            int lv[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                int bits = 0;
                for (int t = 0; t < nt; ++t) bits |= s_live[j * 8 + t] << t;
                lv[j] = __builtin_amdgcn_readfirstlane(bits);
            }
            f32x16 o_acc[2];
            float m_ref[2], l_run[2];
            bool first[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                m_ref[j] = 0.f;
                l_run[j] = 0.f;
                first[j] = true;
#pragma unroll
                for (int v = 0; v < 16; ++v) o_acc[j][v] = 0.f;
            }
            // (tiled bias, see bias_index: the tiles of the wavefront's 32 queries follow each other)
            const float* bh = HAS_BIAS ? a.bias + ((size_t)h * (a.Lq >> 5) + wave) * nt * 1024 : nullptr;
            const uint32_t b_lane = (uint32_t)lane_a * 16;
            auto load_bias = [&](int kt, f32x16& bt) __attribute__((always_inline)) {
                if constexpr (HAS_BIAS) {
                    const char* bp = reinterpret_cast<const char*>(bh + 1024 * kt) + b_lane;
#pragma unroll
                    for (int c = 0; c < 2; ++c)
#pragma unroll
                        for (int i = 0; i < 2; ++i) {
                            const float4 x4 = *reinterpret_cast<const float4*>(bp + (2 * c + i) * 1024);
                            bt[8 * c + 4 * i] = x4.x; bt[8 * c + 4 * i + 1] = x4.y;
                            bt[8 * c + 4 * i + 2] = x4.z; bt[8 * c + 4 * i + 3] = x4.w;
                        }
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) bt[v] = 0.f;
                }
            };
            auto tile = [&](int kt, const f32x16& bt) __attribute__((always_inline)) {
                f32x16 sa[2];
                Frag vf[2][2];
                bool live[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    live[j] = (lv[j] >> kt) & 1;
                    if (live[j]) {
                        const unsigned char* krow = s_k + (j * 256 + 32 * kt + kperm_a) * kFuKPitch;
                        Frag kf[3];
                        kf[0].u = *reinterpret_cast<const uint4*>(krow + hf_a * 16);
                        kf[1].u = *reinterpret_cast<const uint4*>(krow + 32 + hf_a * 16);
                        kf[2].u = make_uint4(0, 0, 0, 0);
                        if (hf_a == 0) kf[2].u = *reinterpret_cast<const uint4*>(krow + 64);
                        const unsigned char* vrow = s_vt + (j * 32 + col_a) * kFuVPitch + (32 * kt + 8 * hf_a) * 2;
                        vf[j][0].u = *reinterpret_cast<const uint4*>(vrow);
                        vf[j][1].u = *reinterpret_cast<const uint4*>(vrow + 32);
                        sa[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0].v, qf[j][0].v, bt, 0, 0, 0);
                        sa[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[1].v, qf[j][1].v, sa[j], 0, 0, 0);
                        sa[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[2].v, qf[j][2].v, sa[j], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (!live[j]) continue;
                    // sa holds s - m_ref (masked keys: -inf).  The first live tile sets the reference to
                    // its maximum; later tiles are exponentiated as they are, and a partial denominator
                    // beyond kOver sends the tile through raise_ref (see k_attn)
                    auto tile_max = [&]() __attribute__((always_inline)) -> float {
                        float mx = sa[j][0];
#pragma unroll
                        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sa[j][v]);
                        return fmaxf(mx, other_half(mx));
                    };
                    auto raise_ref = [&](float tmax, bool always) __attribute__((always_inline)) {
                        const bool raise = always || tmax > kRaise;
                        const float new_ref = raise ? bf16_round(m_ref[j] + tmax) : m_ref[j];
                        const float delta = new_ref - m_ref[j];
                        m_ref[j] = new_ref;
                        const float sc = first[j] ? 1.f : __builtin_amdgcn_exp2f(-delta);
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            o_acc[j][v] *= sc;
                            sa[j][v] -= delta;
                        }
                        l_run[j] *= sc;
                        if (hf_a == 0) qf[j][2].w[0] = pack2(-new_ref, 1.f);
                    };
                    if (first[j]) {
                        raise_ref(tile_max(), true);
                        first[j] = false;
                    }
                    Frag pf[2];
                    float lt;
                    auto exponentiate = [&]() __attribute__((always_inline)) {
                        lt = 0.f;
#pragma unroll
                        for (int c = 0; c < 2; ++c)
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const float p0 = __builtin_amdgcn_exp2f(sa[j][8 * c + 2 * i]);
                                const float p1 = __builtin_amdgcn_exp2f(sa[j][8 * c + 2 * i + 1]);
                                pf[c].w[i] = pack2(p0, p1);
                                lt = add_pair(pf[c].w[i], lt);
                            }
                    };
                    exponentiate();
                    if (__any(!(lt <= kOver))) {
                        raise_ref(tile_max(), false);
                        exponentiate();
                    }
                    l_run[j] += lt;
#pragma unroll
                    for (int c = 0; c < 2; ++c)
                        o_acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[j][c].v, pf[c].v, o_acc[j], 0, 0, 0);
                }
            };
            f32x16 bA, bB;
            load_bias(0, bA);
            for (int kt = 0; kt < nt; kt += 2) {
                load_bias(kt + 1, bB);
                tile(kt, bA);
                load_bias(kt + 2 < nt ? kt + 2 : nt - 1, bA);        // (past the end: a harmless repeat)
                tile(kt + 1, bB);
            }

            // ---- normalise, gate, store: o_acc[j]: lane = query, register v = e = 8*(v/4) + 4*hf + v%4
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float l_tot = l_run[j] + other_half(l_run[j]);
                const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
                uint32_t pk[8];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    pk[i] = pack2(o_acc[j][2 * i] * inv * lo_f32(gpk[j][i]), o_acc[j][2 * i + 1] * inv * hi_f32(gpk[j][i]));
                merge_halves(pk[0], pk[2]);      // lower half-wave: e 0..7, upper: e 8..15
                merge_halves(pk[1], pk[3]);
                merge_halves(pk[4], pk[6]);      // lower: e 16..23, upper: e 24..31
                merge_halves(pk[5], pk[7]);
                bf16_t* op = a.o + ((size_t)(rlv[j] * a.H + h) * a.Lp + 32 * wave) * 32;        // (uniform)
                const uint32_t o_lane = (uint32_t)(col * 32 + 8 * hf) * 2;
                if (row_ok[j] && l_tok < a.L) {
                    stg16(op, o_lane, make_uint4(pk[0], pk[1], pk[2], pk[3]));
                    stg16(op + 16, o_lane, make_uint4(pk[4], pk[5], pk[6], pk[7]));
                }
            }
        }
    }
}

// ====================================================================================
// host side
// token tiles per wavefront: two halve the LDS traffic per MFMA, one keeps the register count at
// two wavefronts per SIMD when the contraction is long
// (and one when two would leave compute units without a block)
static int gemm_tt(bool proj, int K, int tiles_m) {
    return (K > (proj ? 64 : 128) || tiles_m < 2 * kGemmWaves * 256) ? 1 : 2;
}
constexpr int kGemmNS = 2;      // weight tiles per pipeline step

static int gemm_blocks_m(bool proj, int tiles_m, int K) {
    const int per_block = kGemmWaves * gemm_tt(proj, K, tiles_m);
    return (tiles_m + per_block - 1) / per_block;
}

// More than 64 KiB of dynamic LDS has to be asked for once per kernel.  The request is the
// initialiser of a function-local static: the language runs it exactly once, also when several
// threads make their first call together, and every caller sees its result.
template <typename Kernel>
static hipError_t allow_large_lds(Kernel kernel) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               96 * 1024);
}

template <int KC, bool PROJ, int TT, bool RES>
static ff_status launch_gemm_inst(const GemmArgs& a, dim3 grid, hipStream_t st) {
    const size_t smem = gemm_smem_bytes(KC, TT, kGemmNS, a.tiles_per_split);
    static const hipError_t attr = allow_large_lds(&k_gemm<KC, PROJ, TT, kGemmNS, RES>);
    if (attr != hipSuccess) return fail(FF_EHIP, "k_gemm: dynamic LDS limit: %s", hipGetErrorString(attr));
    hipLaunchKernelGGL((k_gemm<KC, PROJ, TT, kGemmNS, RES>), grid, dim3(kGemmWaves * 64), smem, st, a);
    return FF_OK;
}

template <bool PROJ, bool RES>
static ff_status launch_gemm(const GemmArgs& a, int K, dim3 grid, hipStream_t st) {
    const int kc = K / 16;
    if (gemm_tt(PROJ, K, a.rows * (a.Lp >> 5)) == 1) {
        if (kc <= 2) return launch_gemm_inst<2, PROJ, 1, RES>(a, grid, st);
        if (kc <= 4) return launch_gemm_inst<4, PROJ, 1, RES>(a, grid, st);
        if (kc <= 8) return launch_gemm_inst<8, PROJ, 1, RES>(a, grid, st);
        return launch_gemm_inst<16, PROJ, 1, RES>(a, grid, st);
    }
    if (kc <= 2) return launch_gemm_inst<2, PROJ, 2, RES>(a, grid, st);
    if (kc <= 4) return launch_gemm_inst<4, PROJ, 2, RES>(a, grid, st);
    if constexpr (!PROJ) return launch_gemm_inst<8, PROJ, 2, RES>(a, grid, st);
    return fail(FF_EUNSUPPORTED, "k_gemm: no instantiation for K = %d with two token tiles", K);
}

// blocks along the feature axis: at least one block (eight wavefronts) per compute unit
static int pick_split(int blocks_m, int tiles_n) {
    int split = 1;
    while (blocks_m * split < 256 && split < tiles_n) ++split;
    while (tiles_n % split != 0) ++split;      // equal shares
    return split;
}

// Batch rows per attention block (one wavefront each).  With a bias, 8 rows halve the bias traffic
// of 4.  Without one nothing is shared inside a block, and for head dims below 32 the kernel needs
// at most 168 registers: blocks of 4 wavefronts then fit three to a compute unit (three
// wavefronts per SIMD) where a block of 8 leaves a third of the register file empty.
static int attn_rows_per_block(const Problem& p, int rows) {
    if (rows < 8) return 4;
    return (!p.has_bias && p.d < 32) ? 4 : 8;
}

// work items of one attention launch over `rows` batch rows
static int64_t attn_items(const Problem& p, int rows) {
    const int rb = attn_rows_per_block(p, rows);
    return (int64_t)(round_up(p.L, 64) / 64) * p.H * ((rows + rb - 1) / rb);
}

bool mfma_chunk_ok(const Problem& p, int chunk) {
    // the attention kernel splits item indices with float reciprocals, exact below 2^22
    return attn_items(p, chunk) < (1 << 22);
}

static int query_compute_units() {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
        return v;
    return 256;
}
// (queried once; a function-local static is initialised exactly once, also under concurrent first calls)
int compute_units() {
    static const int n = query_compute_units();
    return n;
}

// blocks of this attention instantiation that one compute unit holds at once
template <int D, bool HAS_BIAS, int RB, int GK, bool PERSIST>
static int attn_blocks_per_cu(size_t smem) {
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, reinterpret_cast<const void*>(&k_attn<D, HAS_BIAS, RB, GK, PERSIST>),
                                                     RB * 64, smem) != hipSuccess || nb < 1)
        nb = 1;
    return nb;
}

template <int D, bool HAS_BIAS, int RB, int GK, bool PERSIST>
static ff_status launch_attn(int n_items, size_t smem, hipStream_t st, const AttnArgs& a) {
    // (the LDS of an instantiation is fixed by its template parameters: at most 66 KiB, asked for once)
    static const hipError_t attr =
        GK > 64 ? allow_large_lds(&k_attn<D, HAS_BIAS, RB, GK, PERSIST>) : hipSuccess;
    if (attr != hipSuccess) return fail(FF_EHIP, "k_attn: dynamic LDS limit: %s", hipGetErrorString(attr));
    int n_blocks = n_items;
    if constexpr (PERSIST) {
        // persistent blocks: as many as the chip holds at once (registers and LDS of this
        // instantiation decide how many fit a compute unit), each working through its share of the items
        static const int per_cu = attn_blocks_per_cu<D, HAS_BIAS, RB, GK, PERSIST>(smem);
        const int resident = compute_units() * per_cu;
        if (n_blocks > resident) n_blocks = resident;
    }
    hipLaunchKernelGGL((k_attn<D, HAS_BIAS, RB, GK, PERSIST>), dim3(((n_blocks + 7) / 8) * 8), dim3(RB * 64), smem, st, a);
    return FF_OK;
}

static bool fused_proj_attn(const Problem& p);

static GemmArgs proj_args(const Problem& p, const MfmaWs& m, const Workspace& ws) {
    const int Lp = round_up(p.L, 64), Lq = round_up(p.L, 64);
    GemmArgs g{};
    g.sr = p.sr; g.sl = p.sl; g.L = p.L; g.Lp = Lp; g.Lq = Lq; g.K = p.c; g.eps = p.eps;
    g.w = m.wp; g.aug = m.aug; g.Hd = p.Hd; g.H = p.H; g.D = p.d; g.invD = 1.f / (float)p.d; g.dsh = p.d == 8 ? 3 : (p.d == 16 ? 4 : 5);
    g.nt_main = 4 * p.Hd / 32;
    g.q = m.q; g.k = m.k; g.g = m.g; g.vt = m.vt; g.bias = ws.bias;
    return g;
}

ff_status mfma_prepare(const Problem& p, const ff_attn_weights& w, const void* x, const void* z, const Workspace& ws,
                       hipStream_t st) {
    const MfmaWs m = split_ws(p, ws.chunk, ws);
    const int Lp = round_up(p.L, 64), Lq = round_up(p.L, 64);
    const float qscale = kLog2e / sqrtf((float)p.d);
    const bool tri = p.mode == FF_TRI_START || p.mode == FF_TRI_END;
    {
        const bf16_t *gm = (const bf16_t*)w.ln_g, *bt = (const bf16_t*)w.ln_b;
        const int Hd = p.Hd, c = p.c;
        PrepArgs a{};
        auto seg = [&](int i, const void* wsrc, const void* extra, int rows, int rows_pad, int row0, float scale) {
            a.seg[i] = {(const bf16_t*)wsrc, (const bf16_t*)extra, gm, bt, m.wp + (size_t)row0 * c, m.aug + row0,
                        rows, rows_pad, c, scale};
        };
        seg(0, w.w_q, nullptr, Hd, Hd, 0, qscale);
        seg(1, w.w_k, nullptr, Hd, Hd, Hd, 1.f);
        seg(2, w.w_v, nullptr, Hd, Hd, 2 * Hd, 1.f);
        seg(3, w.w_g, w.b_g, Hd, Hd, 3 * Hd, 1.f);
        seg(4, tri ? w.w_b : nullptr, nullptr, tri ? p.H : 0, 32, 4 * Hd, kLog2e);
        a.nseg = 5;
        const int rows = 4 * Hd + 32;
        const bool chunked_tri = tri && (ws.chunk < p.R || (p.has_bias && fused_proj_attn(p)));
        if (p.mode == FF_MSA_ROW || chunked_tri) {
            // the pair-bias pass shares the launch: row mode projects z (own LayerNorm); chunked
            // triangle attention needs the bias of all rows before the first chunk
            PrepBiasArgs b{};
            b.prep = a;
            b.tiled = fused_proj_attn(p) ? 1 : 0;
            b.bias_blocks = (p.L * (Lp / 32) + 7) / 8;
            b.w_b = (const bf16_t*)w.w_b;
            if (chunked_tri) {
                b.z = (const bf16_t*)x; b.sr = p.sr; b.sl = p.sl; b.K = p.c;
                b.gamma = gm; b.beta = bt;
            } else {
                b.z = (const bf16_t*)z; b.sr = p.L; b.sl = 1; b.K = p.c_z;
                b.gamma = (const bf16_t*)w.lnz_g; b.beta = (const bf16_t*)w.lnz_b;
            }
            b.bias = ws.bias; b.L = p.L; b.Lp = Lp; b.Lq = Lq; b.H = p.H; b.eps = p.eps;
            const dim3 grid(b.bias_blocks + (rows + 7) / 8);
            const int kc = (b.K + 15) / 16;
            Timed t(KK_BIAS, st);
            if (kc <= 2) hipLaunchKernelGGL(k_prep_bias<2>, grid, dim3(512), 0, st, b);
            else if (kc <= 4) hipLaunchKernelGGL(k_prep_bias<4>, grid, dim3(512), 0, st, b);
            else if (kc <= 8) hipLaunchKernelGGL(k_prep_bias<8>, grid, dim3(512), 0, st, b);
            else hipLaunchKernelGGL(k_prep_bias<16>, grid, dim3(512), 0, st, b);
        } else {
            Timed t(KK_PREP, st);
            hipLaunchKernelGGL(k_prep, dim3((rows + 3) / 4), dim3(256), 0, st, a);
        }
    }
    if (p.has_bias && Lq > p.L) {
        const int n = (Lq - p.L) * Lp * p.H;
        Timed t(KK_PREP, st);
        hipLaunchKernelGGL(k_zero_bias_pad, dim3((n + 255) / 256), dim3(256), 0, st, ws.bias, p.L, Lq, Lp, p.H,
                           fused_proj_attn(p) ? 1 : 0);
    }
    return check_launch("prepare (mfma)");
}

// Shapes that k_proj_attn takes: head dimension 32, between 129 and 256 positions (fewer would leave
// most of its eight wavefronts without tokens), 64, 128 or 256 channels.  The pair bias then comes
// from k_prep_bias in every mode (the triangle modes too: it cannot ride along with projections
// that never leave the attention kernel), in the tiled layout of bias_index.
static bool fused_proj_attn(const Problem& p) {
    if (p.d != 32 || p.L <= 128 || p.L > 256) return false;
    return p.c == 64 || p.c == 128 || p.c == 256;
}

template <int KC, bool HAS_BIAS>
static ff_status launch_fused(const FusedArgs& a, hipStream_t st) {
    static const hipError_t attr = allow_large_lds(&k_proj_attn<KC, HAS_BIAS>);
    if (attr != hipSuccess) return fail(FF_EHIP, "k_proj_attn: dynamic LDS limit: %s", hipGetErrorString(attr));
    // one block per compute unit (LDS); per XCD at most as many blocks as it has items
    const int n_rp = (a.rows + 1) / 2;
    int slots = compute_units() / 8;
    const int items_xcd = ((n_rp + 7) / 8) * a.H;
    if (slots > items_xcd) slots = items_xcd;
    if (slots < 1) slots = 1;
    hipLaunchKernelGGL((k_proj_attn<KC, HAS_BIAS>), dim3(8 * slots), dim3(kFuWaves * 64), fused_smem_bytes(KC), st, a);
    return FF_OK;
}

ff_status mfma_chunk(const Problem& p, const ff_attn_weights& w, const void* x, const float* mask, const void* res,
                     void* out, const Workspace& ws, int r0, int rows, hipStream_t st) {
    const int Lp = round_up(p.L, 64), Lq = round_up(p.L, 64);
    const MfmaWs m = split_ws(p, ws.chunk, ws);
    const bool tri = p.mode == FF_TRI_START || p.mode == FF_TRI_END;
    const int tiles_m = rows * (Lp / 32);
    const int blocks_m = gemm_blocks_m(true, tiles_m, p.c);
    const bool fused = fused_proj_attn(p);
    if (fused) {
        FusedArgs f{};
        f.x = (const bf16_t*)x; f.sr = p.sr; f.sl = p.sl; f.r0 = r0; f.rows = rows; f.L = p.L; f.Lp = Lp; f.Lq = Lq;
        f.eps = p.eps; f.wp = m.wp; f.aug = m.aug; f.H = p.H; f.Hd = p.Hd; f.bias = ws.bias; f.mask = mask; f.o = m.o;
        Timed t(KK_PROJ_ATTN, st);
        ff_status ls = FF_OK;
#define FF_FUSED(KCV)                                              \
    do {                                                           \
        if (p.has_bias) ls = launch_fused<KCV, true>(f, st);       \
        else ls = launch_fused<KCV, false>(f, st);                 \
    } while (0)
        if (p.c == 64) FF_FUSED(4);
        else if (p.c == 128) FF_FUSED(8);
        else FF_FUSED(16);
#undef FF_FUSED
        if (ls != FF_OK) return ls;
    } else {
        GemmArgs g = proj_args(p, m, ws);
        g.src = (const bf16_t*)x; g.r0 = r0; g.rows = rows;
        // one chunk covering every row: the pair-bias tile rides along with the projections
        const bool fused_bias = tri && ws.chunk >= p.R;
        const int split = pick_split(blocks_m, g.nt_main);
        g.ft_first = 0; g.ft_count = g.nt_main + (fused_bias ? 1 : 0);
        g.tiles_per_split = (g.ft_count + split - 1) / split;
        Timed t(KK_PROJ, st);
        const ff_status ls = launch_gemm<true, false>(g, p.c, dim3(blocks_m, split), st);
        if (ls != FF_OK) return ls;
    }

    AttnArgs a{};
    a.q = m.q; a.k = m.k; a.g = m.g; a.vt = m.vt; a.o = m.o; a.bias = ws.bias; a.mask = mask;
    a.sr = p.sr; a.sl = p.sl; a.r0 = r0; a.rows = rows; a.L = p.L; a.Lp = Lp; a.Lq = Lq; a.H = p.H; a.Hd = p.Hd;
    a.inv_nq = 1.f / (float)(Lp / 64); a.inv_nqh = 1.f / (float)((Lp / 64) * p.H);
    if (!fused) {
        Timed t(KK_ATTN, st);
        ff_status ls = FF_OK;
        const int rb = attn_rows_per_block(p, rows);
        const int n_items = (int)attn_items(p, rows);          // < 2^22: mfma_chunk_ok
        // keys per bias tile: 128 halve the barriers of long sequences, 64 keep the first tile of short ones small
        const int gk = (p.has_bias && rb == 8 && Lp >= 512) ? 128 : 64;
        // short sequences: persistent blocks, one per rb wave slots of a compute unit (the kernel
        // keeps two wavefronts per SIMD), each working through its share of the items
        const bool persist = Lp < 512;
        const size_t bias_bytes = (size_t)2 * 64 * (gk + kBiasPad) * 4;   // two float tiles
#define FF_ATTN3(DD, HB, RBV, GKV, SM)                                       \
    do {                                                                     \
        if (persist) ls = launch_attn<DD, HB, RBV, GKV, true>(n_items, SM, st, a);   \
        else ls = launch_attn<DD, HB, RBV, GKV, false>(n_items, SM, st, a);          \
    } while (0)
#define FF_ATTN2(DD, RBV)                                                   \
    do {                                                                    \
        if (p.has_bias && gk == 128) ls = launch_attn<DD, true, 8, 128, false>(n_items, bias_bytes, st, a); \
        else if (p.has_bias) FF_ATTN3(DD, true, RBV, 64, bias_bytes);                        \
        else FF_ATTN3(DD, false, RBV, 64, 0);                                                \
    } while (0)
#define FF_ATTN(DD)                  \
    do {                             \
        if (rb == 8) FF_ATTN2(DD, 8); \
        else FF_ATTN2(DD, 4);        \
    } while (0)
        if (p.d == 8) FF_ATTN(8);
        else if (p.d == 16) FF_ATTN(16);
        else FF_ATTN(32);
#undef FF_ATTN
#undef FF_ATTN2
#undef FF_ATTN3
        if (ls != FF_OK) return ls;
    }

    GemmArgs o{};
    o.src = m.o; o.sr = p.sr; o.sl = p.sl; o.r0 = r0; o.rows = rows; o.L = p.L; o.Lp = Lp; o.Lq = Lq;
    o.K = p.Hd; o.w = (const bf16_t*)w.w_o; o.bvec = (const bf16_t*)w.b_o;
    o.Hd = p.Hd; o.H = p.H; o.D = p.d; o.invD = 1.f / (float)p.d; o.dsh = p.d == 8 ? 3 : (p.d == 16 ? 4 : 5); o.out = (bf16_t*)out; o.N = p.c;
    {
        const int tiles_n = o.N / 32;
        const int blocks_o = gemm_blocks_m(false, tiles_m, p.Hd);
        const int split = pick_split(blocks_o, tiles_n);
        o.ft_first = 0; o.ft_count = tiles_n;
        o.tiles_per_split = tiles_n / split;
        Timed t(KK_OUT, st);
        o.res = (const bf16_t*)res;
        const ff_status ls = res ? launch_gemm<false, true>(o, p.Hd, dim3(blocks_o, split), st)
                                 : launch_gemm<false, false>(o, p.Hd, dim3(blocks_o, split), st);
        if (ls != FF_OK) return ls;
    }
    return check_launch("attention chunk (mfma)");
}

}  // namespace ff
