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
//                positions (k_bwd_stats adds the one of dctx); also the row of ones that stands in for no mask
//   k_bwd_stats  forward recomputation with an online softmax: the logsumexp of every query (base 2), ctx,
//                dg, dctx and delta
//   k_bwd_dq     per query tile, over the key tiles: S^T = K Q^T and dP^T = V dctx^T (lane = query, so that
//                logsumexp and delta are lane-local), dS^T, dq^T += K^T dS^T
//   k_bwd_dkv    per key tile, over the query tiles: S = Q K^T and dP = dctx V^T (lane = key), P and dS,
//                dv^T += dctx^T P, dk^T += Q^T dS
//   k_bwd_dbias  per (head, query tile, key tile, chunk of batch rows): dS summed in registers over the rows of the
//                chunk, the chunks' partial sums added in a fixed order by a small second kernel (deterministic,
//                no atomics)
// Operands whose contraction runs over the head dim are 16-byte row reads; operands whose contraction runs
// over keys or queries ("transposed" fragments: lane = channel) are two 8-byte reads of the position-contiguous
// copies, taken in exactly the order in which the accumulator of the previous contraction leaves its values, so
// nothing moves between two contractions.  What is added to q.k (bias, -inf of masked keys) and what is
// subtracted from dP (delta) enter as the accumulators' starting values.
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
    if (blockIdx.x == 0 && blockIdx.y == 0)
        for (int n = threadIdx.x; n < a.Lp; n += 256) a.ones[n] = 1.f;
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

// The logits enter the matrix core's accumulator already holding what is added to q.k: S = (q.k + B) * scale with
// B[i][j] = bias[h][i][j] * sqrt(d) for a key that may be attended to and -inf for one that is masked or beyond L
// (exp2 of the base-2 logit then gives weight 0 without any select).  The tile B [i0 .. i0+31][j0 .. j0+31] in the
// accumulator layout with lane = query: register v = key j0 + 8(v/4) + 4hf + v%4 of query i0 + col.  The bias is
// read from memory in whole rows (a load instruction covers eight 128-byte rows; bias_rows_fetch, which can run
// tiles ahead), scaled, given the keys' -inf and turned through the wavefront's own LDS tile (bias_rows_to_tile).
// FULL: L is a multiple of 32, nothing is out of range.
template <bool FULL>
__device__ __forceinline__ void bias_rows_fetch(float4 (&rows)[4], const Args& a, int h, int i0, int j0, int lane) {
    const int c4 = (lane & 7) * 4;
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int row = 8 * n + (lane >> 3), i = i0 + row, j = j0 + c4;
        const float* p = a.bias + ((size_t)h * a.L + i) * a.L + j;
        if (FULL) {
            rows[n] = *reinterpret_cast<const float4*>(p);
        } else {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < a.L) {
                if ((a.L & 3) == 0 && j + 3 < a.L) v = *reinterpret_cast<const float4*>(p);
                else {
                    if (j < a.L) v.x = p[0];
                    if (j + 1 < a.L) v.y = p[1];
                    if (j + 2 < a.L) v.z = p[2];
                    if (j + 3 < a.L) v.w = p[3];
                }
            }
            rows[n] = v;
        }
    }
}
// keys: bit n set if key j0 + n may be attended to
__device__ __forceinline__ void bias_rows_to_tile(f32x16& b, const float4 (&rows)[4], uint32_t keys, float sqrt_d, float* tile, int lane,
                                                  int col, int hf) {
    const int c4 = (lane & 7) * 4;
    const uint32_t kb = keys >> c4;
    const float m0 = (kb & 1u) ? 0.f : -INFINITY, m1 = (kb & 2u) ? 0.f : -INFINITY;
    const float m2 = (kb & 4u) ? 0.f : -INFINITY, m3 = (kb & 8u) ? 0.f : -INFINITY;
#pragma unroll
    for (int n = 0; n < 4; ++n)
        *reinterpret_cast<float4*>(tile + (8 * n + (lane >> 3)) * kTilePitch + c4) =
            make_float4(rows[n].x * sqrt_d + m0, rows[n].y * sqrt_d + m1, rows[n].z * sqrt_d + m2, rows[n].w * sqrt_d + m3);
    // (LDS operations of one wavefront are carried out in order and the compiler keeps a load behind a store that
    // may alias it, so the lanes see each other's rows without any wait; a fence here would also wait for the
    // loads in flight and serialise the tiles)
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const float4 v = *reinterpret_cast<const float4*>(tile + col * kTilePitch + 8 * g + 4 * hf);
        b[4 * g] = v.x; b[4 * g + 1] = v.y; b[4 * g + 2] = v.z; b[4 * g + 3] = v.w;
    }
    __builtin_amdgcn_wave_barrier();
}
// the same tile with lane = key: register v = query i0 + 8(v/4) + 4hf + v%4 of key j0 + col; kterm is the lane's own
// 0 / -inf
__device__ __forceinline__ void bias_rows_to_tile_by_key(f32x16& b, const float4 (&rows)[4], float kterm, float sqrt_d, float* tile,
                                                         int lane, int col, int hf) {
    const int c4 = (lane & 7) * 4;
#pragma unroll
    for (int n = 0; n < 4; ++n)
        *reinterpret_cast<float4*>(tile + (8 * n + (lane >> 3)) * kTilePitch + c4) =
            make_float4(rows[n].x * sqrt_d, rows[n].y * sqrt_d, rows[n].z * sqrt_d, rows[n].w * sqrt_d);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int v = 0; v < 16; ++v) b[v] = tile[(8 * (v >> 2) + 4 * hf + (v & 3)) * kTilePitch + col] + kterm;
    __builtin_amdgcn_wave_barrier();
}
// the same without a bias: only the keys' 0 / -inf, straight from the mask bits
__device__ __forceinline__ void mask_tile(f32x16& b, uint32_t keys, int hf) {
#pragma unroll
    for (int v = 0; v < 16; ++v) b[v] = ((keys >> (8 * (v >> 2) + 4 * hf + (v & 3))) & 1u) ? 0.f : -INFINITY;
}

// ====================================================================================
// Staging of a 32-position tile of one (row, head) for the four wavefronts of a block, which all contract with it:
// the row-major tile of two tensors (x, y: [32][D]), their position-contiguous tiles (xT, yT: [D][32]) and two
// float vectors of the 32 positions.  The block copies 16-byte pieces global -> registers -> LDS, one tile ahead
// of the tile being worked on (two LDS stages, one barrier per tile); a wavefront reads its operand fragments
// from LDS just before the matrix instructions that use them.
constexpr int kStPitch = 80;                          // bytes per staged row: 32 bf16 + 16 bytes, 16-byte aligned
constexpr int kStRowsX = 0, kStRowsY = 32 * kStPitch, kStColsX = 64 * kStPitch, kStColsY = 96 * kStPitch;
constexpr int kStVecA = 128 * kStPitch, kStVecB = kStVecA + 128, kStBytes = kStVecB + 128;

struct TileSrc {
    const bf16_t *x, *y;         // [L][D] of the (row, head), or NULL (tile not needed: zeros)
    const bf16_t *xT, *yT;       // [D][Lp] of the (row, head), or NULL
    const float *va, *vb;        // [Lp] of the (row, head), or NULL
    int L, Lp;
};

// 16-byte piece `id` of the tile at position n0: where it comes from (NULL: zeros) and where it goes in the stage
template <int D, bool FULL>
__device__ __forceinline__ const uint4* stage_piece(const TileSrc& t, int n0, int id, int& dst) {
    constexpr int PR = D / 8, NR = 32 * PR, NC = 4 * D;
    if (id < 2 * NR) {
        const bool second = id >= NR;
        const int k = second ? id - NR : id, n = k / PR, pc = k - n * PR;
        dst = (second ? kStRowsY : kStRowsX) + n * kStPitch + pc * 16;
        const bf16_t* src = second ? t.y : t.x;
        if (!src || (!FULL && n0 + n >= t.L)) return nullptr;
        return reinterpret_cast<const uint4*>(src + (size_t)(n0 + n) * D + 8 * pc);
    }
    id -= 2 * NR;
    if (id < 2 * NC) {
        const bool second = id >= NC;
        const int k = second ? id - NC : id, e = k >> 2, pc = k & 3;
        dst = (second ? kStColsY : kStColsX) + e * kStPitch + pc * 16;
        const bf16_t* src = second ? t.yT : t.xT;
        if (!src) return nullptr;
        return reinterpret_cast<const uint4*>(src + (size_t)e * t.Lp + n0 + 8 * pc);
    }
    id -= 2 * NC;
    const bool second = id >= 8;
    const int pc = second ? id - 8 : id;
    dst = (second ? kStVecB : kStVecA) + pc * 16;
    const float* src = second ? t.vb : t.va;
    if (!src) return nullptr;
    return reinterpret_cast<const uint4*>(src + n0 + 4 * pc);
}
template <int D> constexpr int stage_pieces() { return 2 * 32 * (D / 8) + 2 * 4 * D + 16; }

// the (up to three) pieces of thread tid: requested from memory ...
template <int D, bool FULL>
__device__ __forceinline__ void stage_fetch(const TileSrc& t, int n0, int tid, uint4& r0, uint4& r1, uint4& r2) {
    constexpr int N = stage_pieces<D>();
    int dst;
    r0 = r1 = r2 = make_uint4(0, 0, 0, 0);
    if (tid < N) {
        const uint4* p = stage_piece<D, FULL>(t, n0, tid, dst);
        if (p) r0 = *p;
    }
    if (N > 256 && tid + 256 < N) {
        const uint4* p = stage_piece<D, FULL>(t, n0, tid + 256, dst);
        if (p) r1 = *p;
    }
    if (N > 512 && tid + 512 < N) {
        const uint4* p = stage_piece<D, FULL>(t, n0, tid + 512, dst);
        if (p) r2 = *p;
    }
}
// ... and put into the stage
template <int D, bool FULL>
__device__ __forceinline__ void stage_store(const TileSrc& t, int n0, int tid, unsigned char* stage, const uint4& r0, const uint4& r1,
                                            const uint4& r2) {
    constexpr int N = stage_pieces<D>();
    int dst;
    if (tid < N) {
        stage_piece<D, FULL>(t, n0, tid, dst);
        *reinterpret_cast<uint4*>(stage + dst) = r0;
    }
    if (N > 256 && tid + 256 < N) {
        stage_piece<D, FULL>(t, n0, tid + 256, dst);
        *reinterpret_cast<uint4*>(stage + dst) = r1;
    }
    if (N > 512 && tid + 512 < N) {
        stage_piece<D, FULL>(t, n0, tid + 512, dst);
        *reinterpret_cast<uint4*>(stage + dst) = r2;
    }
}
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
        stage_fetch<D, FULL>(src, 0, tid, rs[0][0], rs[0][1], rs[0][2]);                                         \
        if (kAhead == 2) stage_fetch<D, FULL>(src, n1, tid, rs[1][0], rs[1][1], rs[1][2]);                       \
        if (BIAS) {                                                                                              \
            bias_rows_fetch<FULL>(brow[0], a, h, i0a, 0, lane);                                                  \
            if (kAhead == 2) bias_rows_fetch<FULL>(brow[1], a, h, i0a, n1, lane);                                \
        }                                                                                                        \
        if (FULL || col < a.L) mk[0] = mrow[col];                                                                \
        if (kAhead == 2 && (FULL || n1 + col < a.L)) mk[1] = mrow[n1 + col];                                     \
    }                                                                                                            \
    stage_store<D, FULL>(src, 0, tid, s_stage, rs[0][0], rs[0][1], rs[0][2]);                                    \
    __syncthreads();
// (bt: what the accumulator of the logits starts from, see bias_rows_fetch.  Every load of the loop is issued on
// every path - the last two tiles ask for themselves again - because a load under a condition makes the compiler
// wait, at every later wait, also for the loads just issued.)
#define FF_BWD_Q_HEAD(P)                                                                                         \
    const int j0 = 32 * (tt + (P));                                                                              \
    const unsigned char* stage = s_stage + (P) * kStBytes;                                                       \
    constexpr int PF = kAhead == 2 ? (P) : 1 - (P);       /* the register set that receives what is requested now */ \
    const int jn = j0 + 32 * kAhead < a.L ? j0 + 32 * kAhead : j0;                                               \
    stage_fetch<D, FULL>(src, jn, tid, rs[PF][0], rs[PF][1], rs[PF][2]);                                         \
    const uint32_t keys = (uint32_t)__ballot((FULL || j0 + col < a.L) && mk[P] != 0.f);                          \
    f32x16 bt;                                                                                                   \
    if (BIAS) bias_rows_to_tile(bt, brow[P], keys, a.sqrt_d, tile, lane, col, hf);                               \
    else if (FULL && !a.mask) bt = zero16();                                                                     \
    else mask_tile(bt, keys, hf);                                                                                \
    if (BIAS) bias_rows_fetch<FULL>(brow[PF], a, h, i0a, jn, lane);                                              \
    if (FULL || jn + col < a.L) mk[PF] = mrow[jn + col];
#define FF_BWD_Q_TAIL(P)                                                                                         \
    if (j0 + 32 < a.L)                                                                                           \
        stage_store<D, FULL>(src, j0 + 32, tid, s_stage + (1 - (P)) * kStBytes, rs[1 - (P)][0], rs[1 - (P)][1], rs[1 - (P)][2]); \
    __syncthreads();

// ====================================================================================
// Block = four consecutive query tiles of one (row, head); the key-side tiles (k rows, v position-contiguous) are
// staged once per block and key tile; the bias rows and the key-mask entries of the next tile are requested
// while this one is worked on.
template <int D, bool FULL, bool BIAS>
__global__ __launch_bounds__(256) void k_bwd_stats(Args a) {
    constexpr int KS = (D + 15) / 16;
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[2 * kStBytes];
    __shared__ __attribute__((aligned(16))) float s_tile[4 * 32 * kTilePitch];
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nt = a.Lp >> 5, bpr = (nt + 3) >> 2;
    const int rh = blockIdx.x / bpr, it = (blockIdx.x - rh * bpr) * 4 + wave;
    const int r = rh / a.H, h = rh - r * a.H, i0 = it * 32, i = i0 + col;
    const bool active = it < nt;
    const size_t base = (size_t)rh * a.L * D;
    float* tile = s_tile + wave * 32 * kTilePitch;
    TileSrc src;
    src.x = a.k + base; src.y = nullptr; src.xT = nullptr; src.yT = a.vT + (size_t)rh * D * a.Lp;
    src.va = nullptr; src.vb = nullptr; src.L = a.L; src.Lp = a.Lp;
    Frag qf[KS];
    load_rows<D, FULL>(qf, a.q + base, active ? i0 : 0, a.L, col, hf);
    FF_BWD_Q_PROLOGUE

    float m = -INFINITY, l = 0.f;
    f32x16 ctx = zero16();          // ctx^T: lane = query, register v = channel 8(v/4) + 4hf + v%4
#define FF_BWD_STATS_TILE(P)                                                                                     \
    {                                                                                                            \
        FF_BWD_Q_HEAD(P)                                                                                         \
        if (active) {                                                                                            \
            Frag kf[KS], vt[2], pf[2];                                                                           \
            staged_rows<D>(kf, stage + kStRowsX, col, hf);                                                       \
            staged_cols<D>(vt, stage + kStColsY, col, hf);                                                       \
            f32x16 s = bt;                                                                                       \
            _Pragma("unroll") for (int t = 0; t < KS; ++t)                                                       \
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t].v, qf[t].v, s, 0, 0, 0);                       \
            float tmax = s[0];                                                                                   \
            _Pragma("unroll") for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, s[v]);                             \
            tmax = fmaxf(tmax, other_half(tmax)) * a.qscale2;       /* (qscale2 > 0) */                          \
            const float m_new = fmaxf(m, tmax);                                                                  \
            /* (nothing valid so far: every weight of the tile is zero and nothing is rescaled) */               \
            const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m - m_new);                    \
            float lt = 0.f;                                                                                      \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) {                                                     \
                s[v] = m_new == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(s[v] * a.qscale2 - m_new);              \
                lt += s[v];                                                                                      \
                ctx[v] *= alpha;                                                                                 \
            }                                                                                                    \
            l = l * alpha + lt;                                                                                  \
            m = m_new;                                                                                           \
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
    __shared__ __attribute__((aligned(16))) float s_tile[4 * 32 * kTilePitch];
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nt = a.Lp >> 5, bpr = (nt + 3) >> 2;
    const int rh = blockIdx.x / bpr, it = (blockIdx.x - rh * bpr) * 4 + wave;
    const int r = rh / a.H, h = rh - r * a.H, i0 = it * 32, i = i0 + col;
    const bool active = it < nt;
    const size_t base = (size_t)rh * a.L * D;
    float* tile = s_tile + wave * 32 * kTilePitch;
    TileSrc src;
    src.x = a.k + base; src.y = a.v + base; src.xT = a.kT + (size_t)rh * D * a.Lp; src.yT = nullptr;
    src.va = nullptr; src.vb = nullptr; src.L = a.L; src.Lp = a.Lp;
    Frag qf[KS], dcf[KS];
    load_rows<D, FULL>(qf, a.q + base, active ? i0 : 0, a.L, col, hf);
    load_rows<D, FULL>(dcf, a.dctx + base, active ? i0 : 0, a.L, col, hf);
    const float lse = a.lse[(size_t)rh * a.Lp + (active ? i : col)], delta = a.delta[(size_t)rh * a.Lp + (active ? i : col)];
    FF_BWD_Q_PROLOGUE

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
            f32x16 s = bt, dp = ndelta;      /* dP - delta: the accumulator starts from -delta */                \
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
template <int D, bool FULL, bool BIAS>
__global__ __launch_bounds__(256) void k_bwd_dkv(Args a) {
    constexpr int KS = (D + 15) / 16;
    __shared__ __attribute__((aligned(16))) unsigned char s_stage[2 * kStBytes];
    __shared__ __attribute__((aligned(16))) float s_tile[4 * 32 * kTilePitch];
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
    // What the accumulator of the logits starts from (see bias_rows_fetch), here with lane = key and register v =
    // query i0 + 8(v/4) + 4hf + v%4: the bias tile times sqrt(d), or -inf in every register if the lane's key is
    // masked or beyond L.  Two sets of bias rows (even and odd query tiles), requested two tiles ahead like the
    // staged tiles.
    const float kterm = key_ok ? 0.f : -INFINITY;
    const int j0a = active ? j0 : 0;
    float* tile = s_tile + wave * 32 * kTilePitch;
    float4 brow[2][4];
    uint4 rs[2][3];
    {
        const int n1 = 32 < a.L ? 32 : 0;
        stage_fetch<D, FULL>(src, 0, tid, rs[0][0], rs[0][1], rs[0][2]);
        if (kAhead == 2) stage_fetch<D, FULL>(src, n1, tid, rs[1][0], rs[1][1], rs[1][2]);
        if (BIAS) {
            bias_rows_fetch<FULL>(brow[0], a, h, 0, j0a, lane);
            if (kAhead == 2) bias_rows_fetch<FULL>(brow[1], a, h, n1, j0a, lane);
        }
    }
    stage_store<D, FULL>(src, 0, tid, s_stage, rs[0][0], rs[0][1], rs[0][2]);
    __syncthreads();

    f32x16 dk = zero16(), dv = zero16();     // dk^T, dv^T: lane = key, register = channel
#define FF_BWD_DKV_TILE(P)                                                                                       \
    {                                                                                                            \
        const int i0 = 32 * (tt + (P));                                                                          \
        const unsigned char* stage = s_stage + (P) * kStBytes;                                                   \
        constexpr int PF = kAhead == 2 ? (P) : 1 - (P);                                                          \
        const int in = i0 + 32 * kAhead < a.L ? i0 + 32 * kAhead : i0;    /* (the last tiles ask for themselves again) */ \
        stage_fetch<D, FULL>(src, in, tid, rs[PF][0], rs[PF][1], rs[PF][2]);                                     \
        f32x16 s;                                                                                                \
        if (BIAS) {                                                                                              \
            bias_rows_to_tile_by_key(s, brow[P], kterm, a.sqrt_d, tile, lane, col, hf);                          \
            bias_rows_fetch<FULL>(brow[PF], a, h, in, j0a, lane);                                                \
        } else {                                                                                                 \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) s[v] = kterm;                                         \
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
            stage_store<D, FULL>(src, i0 + 32, tid, s_stage + (1 - (P)) * kStBytes, rs[1 - (P)][0], rs[1 - (P)][1], \
                                 rs[1 - (P)][2]);                                                                \
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
template <int D, bool FULL, bool BIAS>
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
    f32x16 bt;                      // bias tile times sqrt(d) (the tile is the same for every batch row; the key mask is not)
    {
        float4 rows[4];
        bias_rows_fetch<FULL>(rows, a, h, i0, j0, lane);
        bias_rows_to_tile(bt, rows, 0xffffffffu, a.sqrt_d, s_tile + wave * 32 * kTilePitch, lane, col, hf);
    }
    f32x16 acc = zero16();          // lane = query i, register v = key j0 + 8(v/4) + 4hf + v%4
    // the operands of the next batch row are requested before this one is worked on (the last round asks for its
    // own again: a load under a condition would make every wait in the loop a wait for all loads)
    Frag qn[KS], dcn[KS], kn[KS], vn[KS];
    float lse_n, delta_n, mk_n = 1.f;
    {
        const int rh = r_begin * a.H + h;
        const size_t base = (size_t)rh * a.L * D;
        load_rows<D, FULL>(qn, a.q + base, i0, a.L, col, hf);
        load_rows<D, FULL>(dcn, a.dctx + base, i0, a.L, col, hf);
        load_rows<D, FULL>(kn, a.k + base, j0, a.L, col, hf);
        load_rows<D, FULL>(vn, a.v + base, j0, a.L, col, hf);
        lse_n = a.lse[(size_t)rh * a.Lp + i];
        delta_n = a.delta[(size_t)rh * a.Lp + i];
        if (FULL || j0 + col < a.L) mk_n = a.mrow[(size_t)r_begin * a.mstride + j0 + col];
    }
    for (int r = r_begin; r < r_end; ++r) {
        Frag qf[KS], dcf[KS], kf[KS], vf[KS];
#pragma unroll
        for (int t = 0; t < KS; ++t) { qf[t].u = qn[t].u; dcf[t].u = dcn[t].u; kf[t].u = kn[t].u; vf[t].u = vn[t].u; }
        const float lse = lse_n, delta = delta_n;
        const uint32_t keys = (uint32_t)__ballot((FULL || j0 + col < a.L) && mk_n != 0.f);
        {
            const int rn = r + 1 < r_end ? r + 1 : r, rh = rn * a.H + h;
            const size_t base = (size_t)rh * a.L * D;
            load_rows<D, FULL>(qn, a.q + base, i0, a.L, col, hf);
            load_rows<D, FULL>(dcn, a.dctx + base, i0, a.L, col, hf);
            load_rows<D, FULL>(kn, a.k + base, j0, a.L, col, hf);
            load_rows<D, FULL>(vn, a.v + base, j0, a.L, col, hf);
            lse_n = a.lse[(size_t)rh * a.Lp + i];
            delta_n = a.delta[(size_t)rh * a.Lp + i];
            if (FULL || j0 + col < a.L) mk_n = a.mrow[(size_t)rn * a.mstride + j0 + col];
        }
        f32x16 s = bt, dp;          // the accumulators start from the bias tile (-inf for this row's masked keys) and -delta
        if (!FULL || a.mask) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s[v] = ((keys >> (8 * (v >> 2) + 4 * hf + (v & 3))) & 1u) ? bt[v] : -INFINITY;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) dp[v] = -delta;
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t].v, qf[t].v, s, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t].v, dcf[t].v, dp, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] += __builtin_amdgcn_exp2f(s[v] * a.qscale2 - lse) * dp[v];
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
    return bwd::align256(Lp * 4) + 2 * bwd::align256(rh * Lp * 4) + bwd::align256(rh * d.length * d.head_dim * 2) +
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
    a.row_chunks = bias ? dbias_chunks(d) : 1;
    a.rows_per_chunk = (d.rows + a.row_chunks - 1) / a.row_chunks;
    a.dbias_part = a.row_chunks > 1 ? (float*)p : nullptr;
    a.qscale2 = kLog2e / sqrtf((float)d.head_dim);
    a.scale = 1.f / sqrtf((float)d.head_dim);
    a.sqrt_d = sqrtf((float)d.head_dim);
    const int nt = a.Lp / 32;
    const dim3 g1((unsigned)((rh * nt + 3) / 4)), g2((unsigned)(((size_t)a.row_chunks * d.heads * nt * nt + 3) / 4));
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
    const dim3 gt(g1.x, 3);
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
        FF_BWD(k_bwd_dbias, g2, KK_BWD_DBIAS);
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
