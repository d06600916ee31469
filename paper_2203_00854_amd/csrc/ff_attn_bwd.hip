// Backward pass of the fused attention core (FastFold Section 6.3 benchmarks the fused softmax forward and
// backward; Table 6 reports forward and backward per Evoformer layer), bf16 operands, float32 statistics and
// accumulators, gfx950 matrix cores.  Per batch row r and head h, with scale = 1 / sqrt(d):
//   S[i,j] = scale q[i].k[j] + bias[h,i,j] + M(mask[r,j]);  P = softmax_j S;  ctx[i] = sum_j P[i,j] v[j];  o = g * ctx
//   dg = do * ctx;  dctx = do * g;  dv[j] = sum_i P[i,j] dctx[i];  dP[i,j] = dctx[i].v[j];
//   dS[i,j] = P[i,j] (dP[i,j] - delta[i]),  delta[i] = dctx[i].ctx[i];
//   dq[i] = scale sum_j dS[i,j] k[j];  dk[j] = scale sum_i dS[i,j] q[i];  dbias[h,i,j] = sum_r dS[r,h,i,j]
//
// The score matrix is never stored (Section 3.2): as in the forward pass it is recomputed tile by tile.
// One wavefront per 32-query (or 32-key) tile, four consecutive tiles of one (row, head) per block; the tiles of the
// other side, which all four contract with, are copied into LDS once per block, a tile ahead of the arithmetic:
//   k_bwd_transpose  position-contiguous copies [d][L] of q, k and v for the operands whose contraction runs over
//                positions (k_bwd_stats adds the one of dctx); the row of ones that stands in for no mask; and the
//                bias times sqrt(d), tile by tile in the order of the accumulator registers, once with lane = query
//                and once with lane = key, so that a bias tile is four 16-byte loads per lane in every kernel
//   k_bwd_stats  forward recomputation with an online softmax: the logsumexp of every query (base 2), ctx,
//                dg, dctx and delta
//   k_bwd_dq     per query tile, over the key tiles: S^T = K Q^T and dP^T = V dctx^T (lane = query, so that
//                logsumexp and delta are lane-local), dS^T, dq^T += K^T dS^T
//   k_bwd_dkv    per key tile, over the query tiles: S = Q K^T and dP = dctx V^T (lane = key), P and dS,
//                dv^T += dctx^T P, dk^T += Q^T dS
//   k_bwd_dbias  per (head, patch of 4 x 4 tiles, chunk of batch rows), a wavefront per tile: dS summed in registers over the rows of the
//                chunk, the chunks' partial sums added in a fixed order by a small second kernel (deterministic,
//                no atomics)
// Operands whose contraction runs over the head dim are 16-byte row reads; operands whose contraction runs
// over keys or queries ("transposed" fragments: lane = channel) are two 8-byte reads of the position-contiguous
// copies, taken in exactly the order in which the accumulator of the previous contraction leaves its values, so
// nothing moves between two contractions.  What is added to q.k and what is subtracted from dP enter through the
// matrix core: the bias tile and -delta as the accumulators' starting values, the -inf of masked keys as one more
// contraction step (key side 0 or -inf, query side 1).  A thread's share of the staging copies (which pieces,
// from where, to where) is worked out once per block (StagePlan), not per tile.
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
    const float* mrow;                       // mask entry of (r, j): mrow[r * mstride + j] (without a mask: a row of ones, stride 0)
    int mstride;
    float* ones;                             // workspace [Lp]: that row of ones (written by k_bwd_transpose)
    bf16_t *dq, *dk, *dv, *dg;               // [R][H][L][D]
    float* dbias;                            // [H][L][L] or NULL
    float* dbias_part;                       // workspace [row_chunks][H][L][L] (partial sums over the rows of a chunk)
    int row_chunks, rows_per_chunk;
    bf16_t* dctx;                            // workspace [R][H][L][D]
    bf16_t *qT, *kT, *vT, *dctxT;            // workspace [R][H][D][Lp]: position-contiguous copies for the transposed operands
    float *lse, *delta;                      // workspace [R*H][Lp]
    float *biasA, *biasK;                    // workspace [H][Lp/32][Lp/32][4][64][4]: the bias, times sqrt(D), tile by tile in the
                                             // order of the accumulator registers (biasA: lane = query, biasK: lane = key)
    int R, H, L, Lp;
    float qscale2;                           // log2(e) / sqrt(D)
    float scale;                             // 1 / sqrt(D)
    float sqrt_d;                            // sqrt(D)
};

// Row fragments of the 32 positions n0 .. n0+31 of x [L][D] (x already offset to its (row, head)): lane (n, hf)
// holds channels 16 s + 8 hf .. + 7 of position n0 + col; zeros beyond L or D.
template <int D, bool FULL = false>       // FULL: the caller knows n0 + 31 < L
__device__ __forceinline__ void load_rows(Frag (&f)[(D + 15) / 16], const bf16_t* x, int n0, int L, int col, int hf) {
    constexpr int KS = (D + 15) / 16;
    const int n = n0 + col;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        f[s].u = make_uint4(0, 0, 0, 0);
        if ((FULL || n < L) && 16 * s + 8 * hf < D) f[s].u = *reinterpret_cast<const uint4*>(x + (size_t)n * D + 16 * s + 8 * hf);
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
    // blockIdx.y: with a bias 0 = the bias tiles (first, so that their chains of dependent loads run beside the
    // copies), then q, k, v; without a bias q, k, v
    const int which = a.bias ? (int)blockIdx.y - 1 : (int)blockIdx.y;
    if (blockIdx.x == 0 && which == 0)
        for (int n = threadIdx.x; n < a.Lp; n += 256) a.ones[n] = 1.f;
    const int task = blockIdx.x * 4 + wave;
    if (which < 0) {
        // The bias tile (it, jt) of head h, times sqrt(D), as the accumulator of the logits holds it: float4 g of
        // lane (col, hf) = entries 8 g + 4 hf .. + 3 along the register axis.  biasA: lane = query i0 + col, registers
        // along the keys; biasK: lane = key j0 + col, registers along the queries.  Zeros outside [0, L)^2.
        if (task >= a.H * nt * nt) return;
        const int h = task / (nt * nt), rem = task - h * nt * nt, it = rem / nt, jt = rem - it * nt;
        const float* bh = a.bias + (size_t)h * a.L * a.L;
        float* ta = a.biasA + (size_t)task * 1024 + lane * 4;
        float* tk = a.biasK + (size_t)task * 1024 + lane * 4;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float va[4], vk[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int x = 8 * g + 4 * hf + e;
                const int ia = it * 32 + col, ja = jt * 32 + x, ik = it * 32 + x, jk = jt * 32 + col;
                va[e] = (ia < a.L && ja < a.L) ? bh[(size_t)ia * a.L + ja] * a.sqrt_d : 0.f;
                vk[e] = (ik < a.L && jk < a.L) ? bh[(size_t)ik * a.L + jk] * a.sqrt_d : 0.f;
            }
            *reinterpret_cast<float4*>(ta + 256 * g) = make_float4(va[0], va[1], va[2], va[3]);
            *reinterpret_cast<float4*>(tk + 256 * g) = make_float4(vk[0], vk[1], vk[2], vk[3]);
        }
        return;
    }
    if (task >= a.R * a.H * nt) return;
    const int rh = task / nt, n0 = (task - rh * nt) * 32, n = n0 + col;
    const bf16_t* src = which == 0 ? a.q : (which == 1 ? a.k : a.v);
    bf16_t* dst = which == 0 ? a.qT : (which == 1 ? a.kT : a.vT);
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

// The logits enter the matrix core's accumulator already holding what is added to q.k: S = (q.k + B) * scale with
// B[i][j] = bias[h][i][j] * sqrt(d) for a key that may be attended to and -inf for one that is masked or beyond L
// (exp2 of the base-2 logit then gives weight 0 without any select).  The bias part comes from the copies that
// k_bwd_transpose leaves in the order of the accumulator registers (four 16-byte loads per lane and tile, a
// contiguous KiB per instruction; bias_tile_fetch can run tiles ahead).  The -inf part is one more matrix
// instruction: a contraction step whose key side holds 0 or -inf in its first slot and whose query side a one.
__device__ __forceinline__ void bias_tile_fetch(float4 (&rows)[4], const float* tiles, int h, int nt, int it, int jt, int lane) {
    const float* p = tiles + (((size_t)h * nt + it) * nt + jt) * 1024 + lane * 4;
#pragma unroll
    for (int g = 0; g < 4; ++g) rows[g] = *reinterpret_cast<const float4*>(p + 256 * g);
}
__device__ __forceinline__ void rows_to_acc(f32x16& b, const float4 (&rows)[4]) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        b[4 * g] = rows[g].x; b[4 * g + 1] = rows[g].y; b[4 * g + 2] = rows[g].z; b[4 * g + 3] = rows[g].w;
    }
}
// operand fragments of that step: ok = the lane's key may be attended to
__device__ __forceinline__ Frag key_side(bool ok, int hf) {
    Frag f;
    f.u = make_uint4((hf == 0 && !ok) ? 0xff80u : 0u, 0u, 0u, 0u);        // bfloat16 -inf
    return f;
}
__device__ __forceinline__ Frag one_side(int hf) {
    Frag f;
    f.u = make_uint4(hf == 0 ? 0x3f80u : 0u, 0u, 0u, 0u);                 // bfloat16 1
    return f;
}

// ====================================================================================
// Staging of a 32-position tile of one (row, head) for the four wavefronts of a block, which all contract with it:
// the row-major tile of two tensors (x, y: [32][D]), their position-contiguous tiles (xT, yT: [D][32]) and two
// float vectors of the 32 positions.  The block copies 16-byte pieces global -> registers -> LDS, one tile ahead
// of the tile being worked on (two LDS stages, one barrier per tile); a wavefront reads its operand fragments
// from LDS just before the matrix instructions that use them.
constexpr int kStPitch = 80;                          // bytes per staged row: 32 bf16 + 16 bytes, 16-byte aligned
constexpr int kStRowsX = 0, kStRowsY = 32 * kStPitch, kStColsX = 64 * kStPitch, kStColsY = 96 * kStPitch;
constexpr int kStVecA = 128 * kStPitch, kStVecB = kStVecA + 128, kStSpare = kStVecB + 128, kStBytes = kStSpare + 16;

struct TileSrc {
    const bf16_t *x, *y;         // [L][D] of the (row, head), or NULL (tile not needed: zeros)
    const bf16_t *xT, *yT;       // [D][Lp] of the (row, head), or NULL
    const float *va, *vb;        // [Lp] of the (row, head), or NULL
    int L, Lp;
};

// A thread moves up to three 16-byte pieces of every tile.  Which pieces, where they come from and where they go in the
// stage does not depend on the tile, so it is worked out once (StagePlan::init): per piece the address for tile
// position 0, the bytes per position and the offset in the stage.  A piece nobody needs (its tensor is NULL, or the
// thread has no third piece) asks for the start of x again and lands in a spare slot of the stage: every load and
// every store of the loop is unconditional.
template <int D, bool FULL>
struct StagePlan {
    const unsigned char *b0, *b1, *b2;     // piece address at tile position 0
    int s0, s1, s2;                        // bytes per position
    int d0, d1, d2;                        // offset in the stage
    int n0_, n1_, n2_;                     // !FULL: position of a row piece within the tile (zeros beyond L), else a large negative number

    static __device__ __forceinline__ void piece(const TileSrc& t, int id, const unsigned char*& base, int& stride, int& dst, int& row) {
        constexpr int PR = D / 8, NR = 32 * PR, NC = 4 * D, N = 2 * NR + 2 * NC + 16;
        base = reinterpret_cast<const unsigned char*>(t.x); stride = 0; dst = kStSpare; row = -(1 << 30);
        if (id >= N) return;
        if (id < 2 * NR) {
            const bool second = id >= NR;
            const int k = second ? id - NR : id, n = k / PR, pc = k - n * PR;
            const bf16_t* src = second ? t.y : t.x;
            if (!src) return;
            base = reinterpret_cast<const unsigned char*>(src + (size_t)n * D + 8 * pc); stride = 2 * D;
            dst = (second ? kStRowsY : kStRowsX) + n * kStPitch + pc * 16; row = n;
            return;
        }
        id -= 2 * NR;
        if (id < 2 * NC) {
            const bool second = id >= NC;
            const int k = second ? id - NC : id, e = k >> 2, pc = k & 3;
            const bf16_t* src = second ? t.yT : t.xT;
            if (!src) return;
            base = reinterpret_cast<const unsigned char*>(src + (size_t)e * t.Lp + 8 * pc); stride = 2;
            dst = (second ? kStColsY : kStColsX) + e * kStPitch + pc * 16;
            return;
        }
        id -= 2 * NC;
        const bool second = id >= 8;
        const int pc = second ? id - 8 : id;
        const float* src = second ? t.vb : t.va;
        if (!src) return;
        base = reinterpret_cast<const unsigned char*>(src + 4 * pc); stride = 4;
        dst = (second ? kStVecB : kStVecA) + pc * 16;
    }
    __device__ __forceinline__ void init(const TileSrc& t, int tid) {
        piece(t, tid, b0, s0, d0, n0_);
        piece(t, tid + 256, b1, s1, d1, n1_);
        piece(t, tid + 512, b2, s2, d2, n2_);
    }
    // the pieces of the tile at position n: requested from memory ...
    __device__ __forceinline__ void fetch(int n, uint4& r0, uint4& r1, uint4& r2) const {
        r0 = *reinterpret_cast<const uint4*>(b0 + (size_t)n * s0);
        r1 = *reinterpret_cast<const uint4*>(b1 + (size_t)n * s1);
        r2 = *reinterpret_cast<const uint4*>(b2 + (size_t)n * s2);
    }
    // ... and put into the stage (L: rows at positions n + row >= L are zeros)
    __device__ __forceinline__ void store(unsigned char* stage, int n, int L, uint4 r0, uint4 r1, uint4 r2) const {
        const uint4 z = make_uint4(0, 0, 0, 0);
        if (!FULL) {
            if (n + n0_ >= L) r0 = z;
            if (n + n1_ >= L) r1 = z;
            if (n + n2_ >= L) r2 = z;
        }
        *reinterpret_cast<uint4*>(stage + d0) = r0;
        *reinterpret_cast<uint4*>(stage + d1) = r1;
        *reinterpret_cast<uint4*>(stage + d2) = r2;
    }
};
// operand fragments out of a stage: rows of the lane's position (as load_rows), channels of the lane (as load_cols)
template <int D>
__device__ __forceinline__ void staged_rows(Frag (&f)[(D + 15) / 16], const unsigned char* rows, int col, int hf) {
#pragma unroll
    for (int s = 0; s < (D + 15) / 16; ++s) {
        f[s].u = make_uint4(0, 0, 0, 0);
        if (16 * s + 8 * hf < D) f[s].u = *reinterpret_cast<const uint4*>(rows + col * kStPitch + (16 * s + 8 * hf) * 2);
    }
}
template <int D>
__device__ __forceinline__ void staged_cols(Frag (&f)[2], const unsigned char* cols, int col, int hf) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        f[s].u = make_uint4(0, 0, 0, 0);
        if (col < D) {
            const unsigned char* p = cols + col * kStPitch + (16 * s + 4 * hf) * 2;
            const uint2 lo = *reinterpret_cast<const uint2*>(p), hi = *reinterpret_cast<const uint2*>(p + 16);
            f[s].u = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
    }
}

// Tile loop of the two kernels whose wavefronts keep a query tile and walk over the key tiles.  Memory is two
// tiles ahead of the arithmetic: while tile t is worked on, tile t + 1 waits in registers (it was requested during
// tile t - 1 and goes into the free LDS stage at the end of tile t) and tile t + 2 is being requested; one tile
// ahead the block stalled on every tile for most of a memory latency.  Two named register sets (even tiles, odd
// tiles), hence a loop body written for a literal parity P and used twice: tile tt + P, stage P, sets [P].
//   rs[P]: staged pieces of the thread; brow[P]: the lane's bias rows; mk[P]: the lane's key-mask entry.
// tiles between a request to memory and its use (1 or 2)
constexpr int kAhead = 1;
#define FF_BWD_Q_PROLOGUE                                                                                        \
    uint4 rs[2][3];                                                                                              \
    float4 brow[2][4];                                                                                           \
    float mk[2] = {1.f, 1.f};                                                                                    \
    const int i0a = active ? i0 : 0;                                                                             \
    const float* mrow = a.mrow + (size_t)r * a.mstride;                                                          \
    {                                                                                                            \
        const int n1 = 32 < a.L ? 32 : 0;         /* (a single tile: fetched twice, the second copy unused) */   \
        plan.fetch(0, rs[0][0], rs[0][1], rs[0][2]);                                         \
        if (kAhead == 2) plan.fetch(n1, rs[1][0], rs[1][1], rs[1][2]);                       \
        if (BIAS) {                                                                                              \
            bias_tile_fetch(brow[0], a.biasA, h, nt, i0a >> 5, 0, lane);                                         \
            if (kAhead == 2) bias_tile_fetch(brow[1], a.biasA, h, nt, i0a >> 5, n1 >> 5, lane);                  \
        }                                                                                                        \
        if (FULL || col < a.L) mk[0] = mrow[col];                                                                \
        if (kAhead == 2 && (FULL || n1 + col < a.L)) mk[1] = mrow[n1 + col];                                     \
    }                                                                                                            \
    plan.store(s_stage, 0, a.L, rs[0][0], rs[0][1], rs[0][2]);                                    \
    __syncthreads();
// (bt and kx: what the accumulator of the logits starts from, see bias_tile_fetch.  Every load of the loop is issued on
// every path - the last two tiles ask for themselves again - because a load under a condition makes the compiler
// wait, at every later wait, also for the loads just issued.)
#define FF_BWD_Q_HEAD(P)                                                                                         \
    const int j0 = 32 * (tt + (P));                                                                              \
    const unsigned char* stage = s_stage + (P) * kStBytes;                                                       \
    constexpr int PF = kAhead == 2 ? (P) : 1 - (P);       /* the register set that receives what is requested now */ \
    const int jn = j0 + 32 * kAhead < a.L ? j0 + 32 * kAhead : j0;                                               \
    plan.fetch(jn, rs[PF][0], rs[PF][1], rs[PF][2]);                                         \
    const Frag kx = key_side((FULL || j0 + col < a.L) && mk[P] != 0.f, hf);                                      \
    f32x16 bt;                                                                                                   \
    if (BIAS) rows_to_acc(bt, brow[P]);                                                                          \
    else bt = zero16();                                                                                          \
    if (BIAS) bias_tile_fetch(brow[PF], a.biasA, h, nt, i0a >> 5, jn >> 5, lane);                                \
    if (FULL || jn + col < a.L) mk[PF] = mrow[jn + col];
#define FF_BWD_Q_TAIL(P)                                                                                         \
    if (j0 + 32 < a.L)                                                                                           \
        plan.store(s_stage + (1 - (P)) * kStBytes, j0 + 32, a.L, rs[1 - (P)][0], rs[1 - (P)][1], rs[1 - (P)][2]); \
    __syncthreads();

// ====================================================================================
// Block = four consecutive query tiles of one (row, head); the key-side tiles (k rows, v position-contiguous) are
// staged once per block and key tile; the bias rows and the key-mask entries of the next tile are requested
// while this one is worked on.
template <int D, bool FULL, bool BIAS>
__global__ __launch_bounds__(256) void k_bwd_stats(Args a) {
    constexpr int KS = (D + 15) / 16;
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[2 * kStBytes];
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nt = a.Lp >> 5, bpr = (nt + 3) >> 2;
    const int rh = blockIdx.x / bpr, it = (blockIdx.x - rh * bpr) * 4 + wave;
    const int r = rh / a.H, h = rh - r * a.H, i0 = it * 32, i = i0 + col;
    const bool active = it < nt;
    const size_t base = (size_t)rh * a.L * D;
    TileSrc src;
    src.x = a.k + base; src.y = nullptr; src.xT = nullptr; src.yT = a.vT + (size_t)rh * D * a.Lp;
    src.va = nullptr; src.vb = nullptr; src.L = a.L; src.Lp = a.Lp;
    Frag qf[KS];
    load_rows<D, FULL>(qf, a.q + base, active ? i0 : 0, a.L, col, hf);
    StagePlan<D, FULL> plan;
    plan.init(src, tid);
    FF_BWD_Q_PROLOGUE
    const Frag one = one_side(hf);

    // (the reference starts finite: exp2(-inf - m) is 0 for a masked key, not NaN, also before the first valid one)
    constexpr float kSlack = 8.f;
    float m = -1e30f, l = 0.f;
    f32x16 ctx = zero16();          // ctx^T: lane = query, register v = channel 8(v/4) + 4hf + v%4
#define FF_BWD_STATS_TILE(P)                                                                                     \
    {                                                                                                            \
        FF_BWD_Q_HEAD(P)                                                                                         \
        if (active) {                                                                                            \
            Frag kf[KS], vt[2], pf[2];                                                                           \
            staged_rows<D>(kf, stage + kStRowsX, col, hf);                                                       \
            staged_cols<D>(vt, stage + kStColsY, col, hf);                                                       \
            f32x16 s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kx.v, one.v, bt, 0, 0, 0);                        \
            _Pragma("unroll") for (int t = 0; t < KS; ++t)                                                       \
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t].v, qf[t].v, s, 0, 0, 0);                       \
            float tmax = s[0];                                                                                   \
            _Pragma("unroll") for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, s[v]);                             \
            tmax *= a.qscale2;                                      /* (qscale2 > 0) */                          \
            /* m is the query's reference for the exponentials (the same in its two lanes), not its exact       \
               maximum: it moves, and the sums are rescaled, only when a logit of the tile exceeds it by more    \
               than kSlack - after a query's first tiles almost never, and then the tile pays neither for the    \
               exchange between the halves nor for the rescaling; weights stay below 2^kSlack */                 \
            if (__builtin_amdgcn_ballot_w64(tmax > m + kSlack) != 0) {                                           \
                const float m_new = fmaxf(m, fmaxf(tmax, other_half(tmax)));                                     \
                const float alpha = __builtin_amdgcn_exp2f(m - m_new);                                           \
                _Pragma("unroll") for (int v = 0; v < 16; ++v) ctx[v] *= alpha;                                  \
                l *= alpha;                                                                                      \
                m = m_new;                                                                                       \
            }                                                                                                    \
            float lt = 0.f;                                                                                      \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) {                                                     \
                s[v] = __builtin_amdgcn_exp2f(s[v] * a.qscale2 - m);                                             \
                lt += s[v];                                                                                      \
            }                                                                                                    \
            l += lt;                                                                                             \
            pack_rows(pf, s);                                                                                    \
            _Pragma("unroll") for (int t = 0; t < 2; ++t)                                                        \
                ctx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt[t].v, pf[t].v, ctx, 0, 0, 0);                   \
        }                                                                                                        \
        FF_BWD_Q_TAIL(P)                                                                                         \
    }
    for (int tt = 0; 32 * tt < a.L; tt += 2) {
        FF_BWD_STATS_TILE(0)
        if (32 * (tt + 1) < a.L) FF_BWD_STATS_TILE(1)
    }
#undef FF_BWD_STATS_TILE
    if (!active) return;             // (no barrier after this point)
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
// Block = four consecutive query tiles of one (row, head); staged per key tile: k rows, v rows, k position-contiguous.
template <int D, bool FULL, bool BIAS>
__global__ __launch_bounds__(256, 3) void k_bwd_dq(Args a) {
    constexpr int KS = (D + 15) / 16;
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[2 * kStBytes];
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nt = a.Lp >> 5, bpr = (nt + 3) >> 2;
    const int rh = blockIdx.x / bpr, it = (blockIdx.x - rh * bpr) * 4 + wave;
    const int r = rh / a.H, h = rh - r * a.H, i0 = it * 32, i = i0 + col;
    const bool active = it < nt;
    const size_t base = (size_t)rh * a.L * D;
    TileSrc src;
    src.x = a.k + base; src.y = a.v + base; src.xT = a.kT + (size_t)rh * D * a.Lp; src.yT = nullptr;
    src.va = nullptr; src.vb = nullptr; src.L = a.L; src.Lp = a.Lp;
    Frag qf[KS], dcf[KS];
    load_rows<D, FULL>(qf, a.q + base, active ? i0 : 0, a.L, col, hf);
    load_rows<D, FULL>(dcf, a.dctx + base, active ? i0 : 0, a.L, col, hf);
    const float lse = a.lse[(size_t)rh * a.Lp + (active ? i : col)], delta = a.delta[(size_t)rh * a.Lp + (active ? i : col)];
    StagePlan<D, FULL> plan;
    plan.init(src, tid);
    FF_BWD_Q_PROLOGUE
    const Frag one = one_side(hf);

    f32x16 dq = zero16();           // dq^T: lane = query, register = channel
    f32x16 ndelta;
#pragma unroll
    for (int v = 0; v < 16; ++v) ndelta[v] = -delta;
#define FF_BWD_DQ_TILE(P)                                                                                        \
    {                                                                                                            \
        FF_BWD_Q_HEAD(P)                                                                                         \
        if (active) {                                                                                            \
            Frag kf[KS], vf[KS], kt[2], dsf[2];                                                                  \
            staged_rows<D>(kf, stage + kStRowsX, col, hf);                                                       \
            staged_rows<D>(vf, stage + kStRowsY, col, hf);                                                       \
            f32x16 s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kx.v, one.v, bt, 0, 0, 0);                        \
            f32x16 dp = ndelta;              /* dP - delta: the accumulator starts from -delta */                \
            _Pragma("unroll") for (int t = 0; t < KS; ++t) {                                                     \
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t].v, qf[t].v, s, 0, 0, 0);                       \
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t].v, dcf[t].v, dp, 0, 0, 0);                    \
            }                                                                                                    \
            staged_cols<D>(kt, stage + kStColsX, col, hf);                                                       \
            _Pragma("unroll") for (int v = 0; v < 16; ++v)                                                       \
                s[v] = __builtin_amdgcn_exp2f(s[v] * a.qscale2 - lse) * dp[v];                                   \
            pack_rows(dsf, s);                                                                                   \
            _Pragma("unroll") for (int t = 0; t < 2; ++t)                                                        \
                dq = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt[t].v, dsf[t].v, dq, 0, 0, 0);                    \
        }                                                                                                        \
        FF_BWD_Q_TAIL(P)                                                                                         \
    }
    for (int tt = 0; 32 * tt < a.L; tt += 2) {
        FF_BWD_DQ_TILE(0)
        if (32 * (tt + 1) < a.L) FF_BWD_DQ_TILE(1)
    }
#undef FF_BWD_DQ_TILE
    if (active && i < a.L) {
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
// Block = four consecutive key tiles of one (row, head); the query-side tiles (q, dctx, their position-contiguous
// copies, logsumexp, delta) are staged once per block and query tile.
// (three wavefronts per SIMD where the lengths are whole tiles: at d = 32 with a bias that costs four spilled
// registers, all outside the tile loop; in the variant with bounds checks one of them would land inside it, and a
// reload inside the loop is waited for together with every load in flight)
template <int D, bool FULL, bool BIAS>
__global__ __launch_bounds__(256, FULL ? 3 : 1) void k_bwd_dkv(Args a) {
    constexpr int KS = (D + 15) / 16;
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[2 * kStBytes];
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nt = a.Lp >> 5, bpr = (nt + 3) >> 2;               // key tiles, blocks per (row, head)
    const int rh = blockIdx.x / bpr, jt = (blockIdx.x - rh * bpr) * 4 + wave;
    const int r = rh / a.H, h = rh - r * a.H, j0 = jt * 32, j = j0 + col;
    const bool active = jt < nt;                                 // (a block's last wavefronts may have no key tile)
    const size_t base = (size_t)rh * a.L * D;
    TileSrc src;
    src.x = a.q + base; src.y = a.dctx + base;
    src.xT = a.qT + (size_t)rh * D * a.Lp; src.yT = a.dctxT + (size_t)rh * D * a.Lp;
    src.va = a.lse + (size_t)rh * a.Lp; src.vb = a.delta + (size_t)rh * a.Lp;
    src.L = a.L; src.Lp = a.Lp;

    Frag kf[KS], vf[KS];
    load_rows<D, FULL>(kf, a.k + base, active ? j0 : 0, a.L, col, hf);
    load_rows<D, FULL>(vf, a.v + base, active ? j0 : 0, a.L, col, hf);
    const bool key_ok = active && (FULL || j < a.L) && a.mrow[(size_t)r * a.mstride + ((FULL || j < a.L) ? j : 0)] != 0.f;
    // What the accumulator of the logits starts from (see bias_tile_fetch), here with lane = key and register v =
    // query i0 + 8(v/4) + 4hf + v%4: the bias tile times sqrt(d), and -inf in every register if the lane's key is
    // masked or beyond L.  Two sets of bias tiles (even and odd query tiles), requested ahead like the staged tiles.
    const Frag kx = key_side(key_ok, hf), one = one_side(hf);
    const int jta = active ? jt : 0;
    float4 brow[2][4];
    uint4 rs[2][3];
    StagePlan<D, FULL> plan;
    plan.init(src, tid);
    {
        const int n1 = 32 < a.L ? 32 : 0;
        plan.fetch(0, rs[0][0], rs[0][1], rs[0][2]);
        if (kAhead == 2) plan.fetch(n1, rs[1][0], rs[1][1], rs[1][2]);
        if (BIAS) {
            bias_tile_fetch(brow[0], a.biasK, h, nt, 0, jta, lane);
            if (kAhead == 2) bias_tile_fetch(brow[1], a.biasK, h, nt, n1 >> 5, jta, lane);
        }
    }
    plan.store(s_stage, 0, a.L, rs[0][0], rs[0][1], rs[0][2]);
    __syncthreads();

    f32x16 dk = zero16(), dv = zero16();     // dk^T, dv^T: lane = key, register = channel
#define FF_BWD_DKV_TILE(P)                                                                                       \
    {                                                                                                            \
        const int i0 = 32 * (tt + (P));                                                                          \
        const unsigned char* stage = s_stage + (P) * kStBytes;                                                   \
        constexpr int PF = kAhead == 2 ? (P) : 1 - (P);                                                          \
        const int in = i0 + 32 * kAhead < a.L ? i0 + 32 * kAhead : i0;    /* (the last tiles ask for themselves again) */ \
        plan.fetch(in, rs[PF][0], rs[PF][1], rs[PF][2]);                                     \
        f32x16 s;                                                                                                \
        if (BIAS) {                                                                                              \
            rows_to_acc(s, brow[P]);                                                                             \
            bias_tile_fetch(brow[PF], a.biasK, h, nt, in >> 5, jta, lane);                                       \
        } else {                                                                                                 \
            s = zero16();                                                                                        \
        }                                                                                                        \
        if (active) {                                                                                            \
            Frag qf[KS], dcf[KS], qt[2], dct[2], pf[2], dsf[2];                                                  \
            staged_rows<D>(qf, stage + kStRowsX, col, hf);                                                       \
            staged_rows<D>(dcf, stage + kStRowsY, col, hf);                                                      \
            f32x16 dp;        /* lane = key, register v = query i0 + 8(v/4) + 4hf + v%4; starts from -delta */   \
            _Pragma("unroll") for (int gq = 0; gq < 4; ++gq) {                                                   \
                const float4 d4 = *reinterpret_cast<const float4*>(stage + kStVecB + (8 * gq + 4 * hf) * 4);     \
                dp[4 * gq] = -d4.x; dp[4 * gq + 1] = -d4.y; dp[4 * gq + 2] = -d4.z; dp[4 * gq + 3] = -d4.w;      \
            }                                                                                                    \
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(one.v, kx.v, s, 0, 0, 0);      /* -inf for a masked key */ \
            _Pragma("unroll") for (int t = 0; t < KS; ++t) {                                                     \
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[t].v, kf[t].v, s, 0, 0, 0);                       \
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dcf[t].v, vf[t].v, dp, 0, 0, 0);                    \
            }                                                                                                    \
            staged_cols<D>(qt, stage + kStColsX, col, hf);                                                       \
            staged_cols<D>(dct, stage + kStColsY, col, hf);                                                      \
            _Pragma("unroll") for (int gq = 0; gq < 4; ++gq) {                                                   \
                const float4 l4 = *reinterpret_cast<const float4*>(stage + kStVecA + (8 * gq + 4 * hf) * 4);     \
                const float ls[4] = {l4.x, l4.y, l4.z, l4.w};                                                    \
                _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                                  \
                    const int v = 4 * gq + e;                                                                    \
                    /* (a query beyond L or without keys has logsumexp +inf, a masked key a logit of -inf:        \
                       weight 0 either way) */                                                                   \
                    const float p = __builtin_amdgcn_exp2f(s[v] * a.qscale2 - ls[e]);                            \
                    s[v] = p;                                                                                    \
                    dp[v] = p * dp[v];                                                                           \
                }                                                                                                \
            }                                                                                                    \
            pack_rows(pf, s);                                                                                    \
            pack_rows(dsf, dp);                                                                                  \
            _Pragma("unroll") for (int t = 0; t < 2; ++t) {                                                      \
                dv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dct[t].v, pf[t].v, dv, 0, 0, 0);                    \
                dk = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt[t].v, dsf[t].v, dk, 0, 0, 0);                    \
            }                                                                                                    \
        }                                                                                                        \
        if (i0 + 32 < a.L)                                                                                       \
            plan.store(s_stage + (1 - (P)) * kStBytes, i0 + 32, a.L, rs[1 - (P)][0], rs[1 - (P)][1], rs[1 - (P)][2]); \
        __syncthreads();                                                                                         \
    }
    for (int tt = 0; 32 * tt < a.L; tt += 2) {
        FF_BWD_DKV_TILE(0)
        if (32 * (tt + 1) < a.L) FF_BWD_DKV_TILE(1)
    }
#undef FF_BWD_DKV_TILE
    if (active && (FULL || j < a.L)) {
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
// dbias: block = 16 wavefronts = a patch of 4 x 4 tiles of one head and one chunk of batch rows; wavefront (wi, wj)
// sums dS of tile (it0 + wi, jt0 + wj) over the rows of the chunk in registers.  Per batch row the patch needs the
// q and dctx rows of four query tiles and the k and v rows of four key tiles (16 operand tiles, 2 KiB per result
// tile instead of the 8 KiB a wavefront on its own would fetch), logsumexp and delta of its 128 queries and the mask
// entries of its 128 keys.  The block copies them global -> registers -> LDS (two stages, one barrier per row); a
// thread's share is two 16-byte pieces and one float per row, so that a row is requested two iterations before it is
// needed at the price of nine registers.
constexpr int kDbOperand = 32 * kStPitch;                 // bytes of a staged operand tile [32][D]
constexpr int kDbVec = 16 * kDbOperand;                   // then logsumexp [128], delta [128], key mask [128] (floats)
constexpr int kDbStage = kDbVec + 3 * 128 * 4;

template <int D, bool FULL>
__global__ __launch_bounds__(1024) void k_bwd_dbias(Args a) {
    constexpr int KS = (D + 15) / 16, PR = D / 8, NP = 16 * 32 * PR;      // 16-byte row pieces per batch row
    extern __shared__ __attribute__((aligned(16))) unsigned char s_db[];
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wi = wave >> 2, wj = wave & 3;
    const int nt = a.Lp >> 5, np = (nt + 3) >> 2;
    const int chunk = blockIdx.x / (a.H * np * np), rem = blockIdx.x - chunk * a.H * np * np;
    const int h = rem / (np * np), pp = rem - h * np * np, it0 = 4 * (pp / np), jt0 = 4 * (pp - (pp / np) * np);
    const int it = it0 + wi, jt = jt0 + wj;
    const bool active = it < nt && jt < nt;
    const int r_begin = chunk * a.rows_per_chunk;
    const int r_end = r_begin + a.rows_per_chunk < a.R ? r_begin + a.rows_per_chunk : a.R;
    const int i0 = it * 32, j0 = jt * 32, i = i0 + col;
    if (r_begin >= r_end) return;                          // (whole block)

    // ---- the thread's pieces: address for batch row 0, offset in a stage; rows beyond L are staged as zeros
    const size_t row_stride = (size_t)a.H * a.L * D;       // elements from a batch row to the next
    // (piece tid + 1024, which exists at D = 32 only, is the same row and piece of the operand eight further on)
    constexpr bool TWO = NP > 1024;
    static_assert(NP == 2048 || NP <= 1024, "one or two pieces for every thread");
    const bf16_t *pb0, *pb1;
    int pd0;
    bool pz0, pz1;
    {
        auto plan = [&](int p, const bf16_t*& base, int& dst, bool& zero) {
            const bool has = p < NP;
            const int pq = has ? p : 0;
            const int o = pq / (32 * PR), n = (pq - o * 32 * PR) / PR, pc = pq - (pq / PR) * PR;
            const bf16_t* t = o < 4 ? a.q : (o < 8 ? a.dctx : (o < 12 ? a.k : a.v));
            const int pos = ((o & 3) + (o < 8 ? it0 : jt0)) * 32 + n;
            const bool ok = pos < a.L;
            base = t + ((size_t)h * a.L + (ok ? pos : 0)) * D + 8 * pc;
            dst = has ? o * kDbOperand + n * kStPitch + pc * 16 : -1;
            zero = !ok;
        };
        int unused;
        plan(tid, pb0, pd0, pz0);
        plan(TWO ? tid + 1024 : tid, pb1, unused, pz1);
    }
    // threads 0 .. 383: one float of logsumexp | delta | key mask per row
    const float* vb = a.lse;
    int vstride = 0;                                       // (floats from a batch row to the next: below 2^31)
    int vd = -1;
    bool vz = false;
    if (tid < 384) {
        const int kind = tid >> 7, x = tid & 127;
        if (kind < 2) {
            const int q = it0 * 32 + x;
            vb = (kind == 0 ? a.lse : a.delta) + (size_t)h * a.Lp + (q < a.Lp ? q : 0);
            vstride = a.H * a.Lp;
        } else {
            const int j = jt0 * 32 + x;
            vz = j >= a.L;
            vb = a.mrow + (vz ? 0 : j);
            vstride = a.mstride;
        }
        vd = kDbVec + kind * 512 + x * 4;
    }
#define FF_DB_FETCH(R, ROW)                                                                         \
    {                                                                                               \
        const int rr_ = (ROW) < r_end ? (ROW) : r_end - 1;      /* (past the end: the last row again) */ \
        R##a = *reinterpret_cast<const uint4*>(pb0 + (size_t)rr_ * row_stride);                     \
        if (TWO) R##b = *reinterpret_cast<const uint4*>(pb1 + (size_t)rr_ * row_stride);            \
        R##v = vb[rr_ * vstride];                                                                   \
    }
#define FF_DB_STORE(R, STAGE)                                                                       \
    {                                                                                               \
        /* (through opaque registers: pieces that go from a load straight to an LDS store end up in scratch memory otherwise) */ \
        uint32_t a0_ = R##a.x, a1_ = R##a.y, a2_ = R##a.z, a3_ = R##a.w, b0_ = R##b.x, b1_ = R##b.y, b2_ = R##b.z, b3_ = R##b.w; \
        asm volatile("" : "+v"(a0_), "+v"(a1_), "+v"(a2_), "+v"(a3_), "+v"(b0_), "+v"(b1_), "+v"(b2_), "+v"(b3_));      \
        if (pz0) a0_ = a1_ = a2_ = a3_ = 0u;                                                        \
        if (pz1) b0_ = b1_ = b2_ = b3_ = 0u;                                                        \
        if (pd0 >= 0) *reinterpret_cast<uint4*>((STAGE) + pd0) = make_uint4(a0_, a1_, a2_, a3_);    \
        if (TWO) *reinterpret_cast<uint4*>((STAGE) + pd0 + 8 * kDbOperand) = make_uint4(b0_, b1_, b2_, b3_); \
        if (vd >= 0) *reinterpret_cast<float*>((STAGE) + vd) = vz ? 0.f : R##v;                     \
    }
    // two register sets, by name (a copy from one set to another would have to wait for the load that fills it; a
    // third set spilled, and a spilled load result is waited for at once, which undoes the whole pipeline)
    uint4 rAa, rAb = make_uint4(0, 0, 0, 0), rBa, rBb = make_uint4(0, 0, 0, 0);
    float rAv, rBv;
    FF_DB_FETCH(rA, r_begin)
    FF_DB_FETCH(rB, r_begin + 1)

    f32x16 bt = zero16();           // bias tile times sqrt(d) (the same for every batch row; the key mask is not)
    if (active) {
        float4 rows[4];
        bias_tile_fetch(rows, a.biasA, h, nt, it, jt, lane);
        rows_to_acc(bt, rows);
    }
    const Frag one = one_side(hf);
    f32x16 acc = zero16();          // lane = query i, register v = key j0 + 8(v/4) + 4hf + v%4
    FF_DB_STORE(rA, s_db)
    __syncthreads();
    // Row r: the set FREE (its row is in the stage) asks for row r + 2, the stage is worked on, the set NEXT (row r + 1,
    // requested one row ago) goes into the other stage.
#define FF_DB_ROW(FREE, NEXT)                                                                                    \
    {                                                                                                            \
        const unsigned char* stage = s_db + ((r - r_begin) & 1) * kDbStage;                                      \
        FF_DB_FETCH(FREE, r + 2)                                                                                 \
        if (active) {                                                                                            \
            Frag qf[KS], dcf[KS], kf[KS], vf[KS];                                                                \
            staged_rows<D>(qf, stage + wi * kDbOperand, col, hf);                                                \
            staged_rows<D>(dcf, stage + (4 + wi) * kDbOperand, col, hf);                                         \
            staged_rows<D>(kf, stage + (8 + wj) * kDbOperand, col, hf);                                          \
            staged_rows<D>(vf, stage + (12 + wj) * kDbOperand, col, hf);                                         \
            const float lse = *reinterpret_cast<const float*>(stage + kDbVec + (wi * 32 + col) * 4);             \
            const float delta = *reinterpret_cast<const float*>(stage + kDbVec + 512 + (wi * 32 + col) * 4);     \
            const float mk = *reinterpret_cast<const float*>(stage + kDbVec + 1024 + (wj * 32 + col) * 4);       \
            const Frag kx = key_side(mk != 0.f, hf);                                                             \
            /* the accumulators start from the bias tile (and -inf for this row's masked keys) and -delta */      \
            f32x16 s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kx.v, one.v, bt, 0, 0, 0), dp;                    \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) dp[v] = -delta;                                       \
            _Pragma("unroll") for (int t = 0; t < KS; ++t) {                                                     \
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t].v, qf[t].v, s, 0, 0, 0);                       \
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t].v, dcf[t].v, dp, 0, 0, 0);                    \
            }                                                                                                    \
            _Pragma("unroll") for (int v = 0; v < 16; ++v)                                                       \
                acc[v] += __builtin_amdgcn_exp2f(s[v] * a.qscale2 - lse) * dp[v];                                \
        }                                                                                                        \
        if (r + 1 < r_end) FF_DB_STORE(NEXT, s_db + ((r + 1 - r_begin) & 1) * kDbStage)                          \
        __syncthreads();                                                                                         \
        ++r;                                                                                                     \
    }
    for (int r = r_begin; r < r_end;) {
        FF_DB_ROW(rA, rB)
        if (r >= r_end) break;
        FF_DB_ROW(rB, rA)
    }
#undef FF_DB_ROW
#undef FF_DB_FETCH
#undef FF_DB_STORE
    if (active && i < a.L) {
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

// Row chunks of the bias gradient: enough (head, patch of 4 x 4 tiles, chunk) blocks for one per compute unit, at
// least 8 rows each.
static int dbias_chunks(const ff_core_desc& d) {
    const int nt = (d.length + 31) / 32, np = (nt + 3) / 4;
    const long patches = (long)d.heads * np * np;
    int chunks = (int)((256 + patches - 1) / patches);
    if (chunks > d.rows / 8) chunks = d.rows / 8;
    return chunks < 1 ? 1 : chunks;
}

size_t core_backward_workspace(const ff_core_desc& d) {
    const size_t Lp = bwd::round_up(d.length, 32), rh = (size_t)d.rows * d.heads;
    const int chunks = dbias_chunks(d);
    return bwd::align256(Lp * 4) + 2 * bwd::align256(rh * Lp * 4) + bwd::align256(rh * d.length * d.head_dim * 2) +
           4 * bwd::align256(rh * d.head_dim * Lp * 2) + 2 * bwd::align256((size_t)d.heads * Lp * Lp * 4) +
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
    a.ones = (float*)p; p += align256((size_t)a.Lp * 4);
    a.mrow = mask ? mask : a.ones;
    a.mstride = mask ? d.length : 0;
    a.lse = (float*)p; p += align256(rh * a.Lp * 4);
    a.delta = (float*)p; p += align256(rh * a.Lp * 4);
    a.dctx = (bf16_t*)p; p += align256(rh * d.length * d.head_dim * 2);
    const size_t tbytes = align256(rh * d.head_dim * a.Lp * 2);
    a.qT = (bf16_t*)p; p += tbytes;
    a.kT = (bf16_t*)p; p += tbytes;
    a.vT = (bf16_t*)p; p += tbytes;
    a.dctxT = (bf16_t*)p; p += tbytes;
    const size_t bbytes = align256((size_t)d.heads * a.Lp * a.Lp * 4);
    a.biasA = (float*)p; p += bbytes;
    a.biasK = (float*)p; p += bbytes;
    a.row_chunks = bias ? dbias_chunks(d) : 1;
    a.rows_per_chunk = (d.rows + a.row_chunks - 1) / a.row_chunks;
    a.dbias_part = a.row_chunks > 1 ? (float*)p : nullptr;
    a.qscale2 = kLog2e / sqrtf((float)d.head_dim);
    a.scale = 1.f / sqrtf((float)d.head_dim);
    a.sqrt_d = sqrtf((float)d.head_dim);
    const int nt = a.Lp / 32;
    const dim3 g1((unsigned)((rh * nt + 3) / 4)), g2((unsigned)((size_t)a.row_chunks * d.heads * ((nt + 3) / 4) * ((nt + 3) / 4)));
    const bool full = d.length % 32 == 0;        // nothing out of range: the kernels without bounds checks
#define FF_BWD_D(KERNEL, GRID, DV)                                                                       \
    do {                                                                                                 \
        if (full && bias) hipLaunchKernelGGL((KERNEL<DV, true, true>), GRID, dim3(256), 0, st, a);       \
        else if (full) hipLaunchKernelGGL((KERNEL<DV, true, false>), GRID, dim3(256), 0, st, a);         \
        else if (bias) hipLaunchKernelGGL((KERNEL<DV, false, true>), GRID, dim3(256), 0, st, a);         \
        else hipLaunchKernelGGL((KERNEL<DV, false, false>), GRID, dim3(256), 0, st, a);                  \
    } while (0)
#define FF_BWD(KERNEL, GRID, KIND)                                                                       \
    do {                                                                                                 \
        Timed t(KIND, st);                                                                               \
        if (d.head_dim == 8) FF_BWD_D(KERNEL, GRID, 8);                                                  \
        else if (d.head_dim == 16) FF_BWD_D(KERNEL, GRID, 16);                                           \
        else FF_BWD_D(KERNEL, GRID, 32);                                                                 \
    } while (0)
    const unsigned bias_blocks = (unsigned)(((size_t)d.heads * nt * nt + 3) / 4);
    const dim3 gt(bias && bias_blocks > g1.x ? bias_blocks : g1.x, bias ? 4 : 3);      // q, k, v; the bias tiles
    {
        Timed t(KK_BWD_STATS, st);
        if (d.head_dim == 8) hipLaunchKernelGGL((k_bwd_transpose<8>), gt, dim3(256), 0, st, a);
        else if (d.head_dim == 16) hipLaunchKernelGGL((k_bwd_transpose<16>), gt, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((k_bwd_transpose<32>), gt, dim3(256), 0, st, a);
    }
    const dim3 g4((unsigned)(rh * ((nt + 3) / 4)));          // blocks of four tiles of one (row, head)
    FF_BWD(k_bwd_stats, g4, KK_BWD_STATS);
    FF_BWD(k_bwd_dq, g4, KK_BWD_DQ);
    FF_BWD(k_bwd_dkv, g4, KK_BWD_DKV);
    if (bias) {
        {
            Timed t(KK_BWD_DBIAS, st);
            hipError_t attr = hipSuccess;
#define FF_BWD_DB(DV, FV)                                                                                        \
    do {                                                                                                         \
        static const hipError_t once = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_bwd_dbias<DV, FV>), \
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kDbStage); \
        attr = once;                                                                                             \
        if (once == hipSuccess) hipLaunchKernelGGL((k_bwd_dbias<DV, FV>), g2, dim3(1024), 2 * kDbStage, st, a);  \
    } while (0)
            if (d.head_dim == 8) { if (full) FF_BWD_DB(8, true); else FF_BWD_DB(8, false); }
            else if (d.head_dim == 16) { if (full) FF_BWD_DB(16, true); else FF_BWD_DB(16, false); }
            else { if (full) FF_BWD_DB(32, true); else FF_BWD_DB(32, false); }
#undef FF_BWD_DB
            if (attr != hipSuccess) return fail(FF_EHIP, "k_bwd_dbias: dynamic LDS limit: %s", hipGetErrorString(attr));
        }
        if (a.row_chunks > 1) {
            Timed t(KK_BWD_DBIAS, st);
            hipLaunchKernelGGL(k_bwd_dbias_reduce, dim3(1024), dim3(256), 0, st, a);
        }
    }
#undef FF_BWD
#undef FF_BWD_D
    return check_launch("attention core backward");
}

}  // namespace ff
