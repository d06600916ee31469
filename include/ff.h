/*
 * ff.h - C ABI of libff: Evoformer gated axial attention with pair bias on one MI355X.
 *
 * The library implements, as hand-written HIP kernels for gfx950, the attention module
 * that FastFold (arXiv 2203.00854) optimises inside AlphaFold's Evoformer:
 *
 *   LayerNorm -> Q/K/V/gate projections -> softmax(Q K^T / sqrt(d) + mask + pair bias) V
 *             -> sigmoid gate -> output projection
 *
 * in the four axial variants the Evoformer uses (Section 2.3: row-wise and column-wise
 * attention on the MSA representation, the attention bias that carries the pair
 * representation into the MSA row attention, and the "similar blocks" of the pair stack,
 * i.e. AlphaFold's triangle attention around the starting and the ending node), plus the
 * fixed row chunking used for long-sequence inference (Sections 3.2, 5.3, 6.2).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library never
 *     allocates or frees device memory (scratch memory is the caller's workspace argument)
 *     and no call depends on an earlier one.  What it keeps inside the process is
 *     bookkeeping only: device properties and per-kernel launch attributes looked up on first
 *     use (initialised once, safely under concurrent first calls), the thread-local last
 *     error and last kernel family, and the launch timer's records while that is on.
 *   - Tensors are dense, row-major, in the dtype named by the call (float32 or bfloat16).
 *     Weights have the tensor dtype.  The mask is always float32.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the default
 *     stream) and the call returns without synchronising.
 *   - Errors are returned as ff_status; nothing is launched and nothing is written to the
 *     output when an argument is rejected.  ff_last_error() gives a message (thread-local).
 *   - Arithmetic: LayerNorm statistics, softmax maxima and sums and all accumulations are
 *     float32.  In FF_BF16 the projected q/k/v/gate, the softmax weights and the gated
 *     context are rounded to bfloat16 as matrix-core operands; FF_F32 uses no bfloat16.
 */
#ifndef FF_H
#define FF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { FF_OK = 0, FF_EINVAL = 1, FF_EUNSUPPORTED = 2, FF_EWORKSPACE = 3, FF_EHIP = 4 } ff_status;
typedef enum { FF_F32 = 0, FF_BF16 = 1 } ff_dtype;

/* Which axis is attended and where the bias comes from (Section 2.3).
 * x is [n_a, n_b, c].  "batch row" = an index of the axis that is NOT attended; batch rows
 * are independent given the bias (Section 4.2).
 *   FF_MSA_ROW    x = MSA rep [N_seq, N_res, c_m]; batch row s, attention over residues j;
 *                 bias[h,i,j] = LayerNorm_z(z[i,j,:]) . w_b[h,:] from the pair rep z.
 *   FF_MSA_COL    x = MSA rep; batch row i (a residue), attention over sequences t; no bias.
 *   FF_TRI_START  x = pair rep [N_res, N_res, c_z]; batch row i, attention over k;
 *                 logits of (i; j,k) get bias[h,j,k] = LayerNorm(x[j,k,:]) . w_b[h,:].
 *   FF_TRI_END    x = pair rep; batch row j, attention over k; logits of (j; i,k) get
 *                 bias[h,k,i].  Equals FF_TRI_START applied to x with its first two axes
 *                 swapped, swapped back. */
typedef enum { FF_MSA_ROW = 0, FF_MSA_COL = 1, FF_TRI_START = 2, FF_TRI_END = 3 } ff_mode;

/* Shape of one attention module. */
typedef struct {
    int32_t mode;      /* ff_mode */
    int32_t dtype;     /* ff_dtype of x, z, out and all weights */
    int32_t n_a, n_b;  /* x and out are [n_a, n_b, c]; triangle modes need n_a == n_b */
    int32_t c;         /* channels of x (c_m for the MSA rep, c_z for the pair rep) */
    int32_t c_z;       /* channels of z; FF_MSA_ROW only, otherwise ignored */
    int32_t heads;     /* H */
    int32_t head_dim;  /* d; channel h*d + e of a projection belongs to head h */
    float   ln_eps;    /* LayerNorm epsilon, inside the square root */
} ff_attn_desc;

/* Weights, all [out, in] row-major (y = x W^T + b), dtype = desc.dtype.
 * q, k, v and the bias projection have no additive bias; the gate and the output
 * projection have one (Section 5.2 names the gate as bias + sigmoid + product). */
typedef struct {
    const void *ln_g, *ln_b;    /* [c]      LayerNorm of x                                  */
    const void *lnz_g, *lnz_b;  /* [c_z]    LayerNorm of z, FF_MSA_ROW only, else NULL      */
    const void *w_q, *w_k, *w_v;/* [H*d, c]                                                 */
    const void *w_b;            /* [H, c_z] FF_MSA_ROW; [H, c] triangle modes; NULL for COL */
    const void *w_g, *b_g;      /* [H*d, c], [H*d]  gate                                    */
    const void *w_o, *b_o;      /* [c, H*d], [c]    output projection                       */
} ff_attn_weights;

/* LayerNorm over the last axis of x [rows, c] (Section 5.2: the batch-reduction kernel the
 * paper rewrites for small hidden sizes):
 *   y = (x - mean) / sqrt(var + eps) * gamma + beta, biased variance, float32 statistics.
 * x, gamma, beta, y: device pointers of dtype dt; y may alias x.  rows >= 0, 1 <= c <= 8192.
 * Returns FF_EINVAL for bad sizes/NULL pointers, FF_EHIP if the launch fails. */
ff_status ff_layernorm(const void* x, const void* gamma, const void* beta, void* y,
                       int64_t rows, int32_t c, float eps, int32_t dt, void* hip_stream);

/* Bytes of device workspace ff_gated_attention (chunk_rows = 0) or ff_attention_chunked
 * (chunk_rows >= 1) needs for this shape: projected q,k,v,gate and the gated context of one
 * chunk of batch rows plus the bias tensor [H, L, L] in float32 - never the score tensor
 * (Section 3.2 gives its size, N_r^3 * N_head * 2 bytes, as the memory bottleneck).
 * Returns 0 if desc is invalid (ff_last_error says why). */
size_t ff_attention_workspace_bytes(const ff_attn_desc* desc, int32_t chunk_rows);

/* One gated attention module (Sections 2.1, 2.3, 5.2), all batch rows at once.
 *   x    [n_a, n_b, c]   input representation
 *   z    [n_b, n_b, c_z] pair representation, FF_MSA_ROW only; must be NULL otherwise
 *   mask [n_a, n_b] float32 of 0/1 or NULL (= all ones).  mask[a,b] == 0 removes token
 *        (a,b) as a KEY: it gets softmax weight exactly 0 (the paper's "mask" addend of
 *        the softmax input, read as minus infinity).  Queries are never masked.  A query
 *        whose keys are all masked gets zero context, so its output is b_o.
 *   out  [n_a, n_b, c]   out = (gate * context) W_o^T + b_o; no residual add, no dropout.
 *        Must not overlap x, z or ws.
 *   ws, ws_bytes  device scratch of at least ff_attention_workspace_bytes(desc, 0) bytes,
 *        256-byte aligned.
 * Returns FF_EINVAL (bad enum, non-positive size, NULL required pointer, non-NULL z outside
 * FF_MSA_ROW, n_a != n_b in a triangle mode, misaligned ws), FF_EWORKSPACE (ws too small),
 * FF_EUNSUPPORTED (a size beyond the kernels' limits: head_dim > 128, c or c_z > 8192),
 * FF_EHIP (launch failure). */
ff_status ff_gated_attention(const ff_attn_desc* desc, const ff_attn_weights* w,
                             const void* x, const void* z, const float* mask,
                             void* out, void* ws, size_t ws_bytes, void* hip_stream);

/* The same module evaluated chunk_rows batch rows at a time (Section 5.3: a chunk
 * partitions a dimension that takes no part in the computation, Y_i = F(X_i^chunk,
 * X^nonchunk); Section 6.2/6.4 use chunk size 64).  The chunked input is the batch-row
 * axis of x (and of out and mask); the non-chunked input is the bias tensor, computed once
 * before the loop.  The last chunk may be short; chunk_rows larger than the number of
 * batch rows is one chunk.  The result is bit-identical to ff_gated_attention.
 * ws must hold ff_attention_workspace_bytes(desc, chunk_rows) bytes.
 * Extra error: chunk_rows < 1 -> FF_EINVAL. */
ff_status ff_attention_chunked(const ff_attn_desc* desc, const ff_attn_weights* w,
                               const void* x, const void* z, const float* mask,
                               void* out, void* ws, size_t ws_bytes, void* hip_stream,
                               int32_t chunk_rows);

/* The module together with the residual update that closes it in the Evoformer block
 * (Section 5.2 lists "bias + dropout + add" as the last fused step of a module; dropout is
 * the identity at inference):
 *   out = x + ((gate * context) W_o^T + b_o)
 * The sum is formed in float32 and rounded to the tensor dtype once.  Arguments as for
 * ff_attention_chunked, with chunk_rows = 0 meaning all batch rows at once.  out may be x
 * itself (the representation is updated in place, saving a second [n_a, n_b, c] tensor:
 * 1 GiB at N_res = 2048) or must not overlap x at all; it must not overlap z or ws.
 * In the triangle modes the bias is taken from x as it was before the call.
 * Errors as for ff_attention_chunked; chunk_rows < 0 -> FF_EINVAL. */
ff_status ff_gated_attention_residual(const ff_attn_desc* desc, const ff_attn_weights* w,
                                      const void* x, const void* z, const float* mask,
                                      void* out, void* ws, size_t ws_bytes, void* hip_stream,
                                      int32_t chunk_rows);

/* Triangular multiplicative update of the pair representation (Section 2.3 and Figure 3: the pair
 * stack's "triangular updates module"; Section 5.2 merges its left and right projections and their
 * gates into one GEMM; Section 4.2 / Table 3 name its outgoing and incoming forms).  With
 * zn = LayerNorm_in(z):
 *   a = mask * sigmoid(zn w_ag^T + b_ag) * (zn w_ap^T + b_ap)     left,  [n, n, c]
 *   b = mask * sigmoid(zn w_bg^T + b_bg) * (zn w_bp^T + b_bp)     right, [n, n, c]
 *   g = sigmoid(zn w_g^T + b_g)                                          [n, n, c_z]
 *   incoming = 0:  t[i,j,:] = sum_k a[i,k,:] * b[j,k,:]       incoming = 1:  t[i,j,:] = sum_k a[k,i,:] * b[k,j,:]
 *   out = g * (LayerNorm_out(t) w_o^T + b_o)                  (+ z if residual = 1)
 * LayerNorms: biased variance, eps inside the root.  a, b and t are rounded to bfloat16 between
 * the kernels; g, statistics and accumulations are float32. */
typedef struct {
    int32_t dtype;      /* ff_dtype; FF_BF16 only (FF_F32 -> FF_EUNSUPPORTED) */
    int32_t incoming;   /* 0 = outgoing edges, 1 = incoming edges */
    int32_t n;          /* z and out are [n, n, c_z] */
    int32_t c_z;        /* channels of the pair representation: multiple of 32, <= 128 */
    int32_t c;          /* channels of the left / right projections: multiple of 32, <= 128 */
    float   ln_eps;
} ff_trimul_desc;

/* Weights [out, in] row-major, all with an additive bias, dtype = desc.dtype. */
typedef struct {
    const void *ln_g, *ln_b;      /* [c_z]  LayerNorm_in                   */
    const void *w_ap, *b_ap;      /* [c, c_z], [c]   left projection       */
    const void *w_ag, *b_ag;      /* [c, c_z], [c]   left gate             */
    const void *w_bp, *b_bp;      /* [c, c_z], [c]   right projection      */
    const void *w_bg, *b_bg;      /* [c, c_z], [c]   right gate            */
    const void *w_g, *b_g;        /* [c_z, c_z], [c_z]  output gate        */
    const void *lno_g, *lno_b;    /* [c]    LayerNorm_out                  */
    const void *w_o, *b_o;        /* [c_z, c], [c_z] output projection     */
} ff_trimul_weights;

/* Bytes of device workspace ff_triangle_multiplication needs (a, b and t channel-major, the
 * prepared weights); 0 if desc is invalid or unsupported (ff_last_error says why). */
size_t ff_triangle_multiplication_workspace_bytes(const ff_trimul_desc* desc);

/*   z    [n, n, c_z] pair representation, 16-byte aligned
 *   mask [n, n] float32 of 0/1 or NULL (= all ones): multiplies a and b, so a masked pair takes
 *        part in no sum over k; its own output position is still computed
 *   out  [n, n, c_z]; with residual = 1 it may be z itself (in-place update), otherwise it must
 *        not overlap z; never the workspace
 *   ws, ws_bytes  device scratch, 256-byte aligned, at least the size reported above
 * Returns FF_EINVAL / FF_EUNSUPPORTED / FF_EWORKSPACE / FF_EHIP as the attention entry points do. */
ff_status ff_triangle_multiplication(const ff_trimul_desc* desc, const ff_trimul_weights* w,
                                     const void* z, const float* mask, void* out, int32_t residual,
                                     void* ws, size_t ws_bytes, void* hip_stream);

/* Global column attention of the extra-MSA stack (Table 1 gives its size, N_extra_seq = 1024 / 5120;
 * Section 6.2 names the extra MSA among the model's optional modules; the algorithm is AlphaFold's
 * published MSA column global self-attention).  Per residue column i, with mn = LayerNorm(m):
 *   qbar[i]    = mean of mn[s,i,:] over the unmasked sequences s
 *   q[i,h,:]   = (w_q qbar[i])[h] / sqrt(head_dim)          heads x head_dim, no bias
 *   k[s,i,:]   = w_k mn[s,i],  v[s,i,:] = w_v mn[s,i]        ONE shared head of head_dim channels, no bias
 *   P[i,h,:]   = softmax over s of q[i,h] . k[s,i]           masked sequences: weight exactly 0
 *   o[i,h,:]   = sum_s P[i,h,s] v[s,i,:]
 *   out[s,i,:] = w_o (sigmoid(w_g mn[s,i] + b_g) * concat_h o[i,h]) + b_o
 * A column without unmasked sequences gets zero context (out = b_o).  The softmax and o are float32;
 * the folded weights, the normalised tokens of the k, v and query projections, k, v and the gated context
 * are bfloat16.  The gate projection takes the tokens as stored (LayerNorm's mean and scale are applied to
 * its float32 result); the LayerNorm variance is E[x^2] - mean^2 in float32, its relative rounding error
 * about 2^-22 (1 + mean^2 / variance). */
typedef struct {
    int32_t dtype;      /* ff_dtype; FF_BF16 only (FF_F32 -> FF_EUNSUPPORTED) */
    int32_t n_seq;      /* m and out are [n_seq, n_res, c] */
    int32_t n_res;
    int32_t c;          /* multiple of 32, <= 128 */
    int32_t heads;      /* heads * head_dim in {32, 64, 128} */
    int32_t head_dim;   /* 8 or 16 */
    float   ln_eps;
} ff_global_desc;

typedef struct {
    const void *ln_g, *ln_b;      /* [c]                                         */
    const void *w_q;              /* [heads*head_dim, c]                         */
    const void *w_k, *w_v;        /* [head_dim, c]                               */
    const void *w_g, *b_g;        /* [heads*head_dim, c], [heads*head_dim]       */
    const void *w_o, *b_o;        /* [c, heads*head_dim], [c]                    */
} ff_global_weights;

/* Bytes of device workspace (k and v of every token in bfloat16, one mask byte per token, partial query
 * sums, folded weights);
 * 0 if desc is invalid or unsupported (ff_last_error says why). */
size_t ff_global_column_attention_workspace_bytes(const ff_global_desc* desc);

/*   m    [n_seq, n_res, c], 16-byte aligned;  mask [n_seq, n_res] float32 of 0/1 or NULL (= all ones)
 *   out  [n_seq, n_res, c], must not overlap m or ws;  ws 256-byte aligned, at least the size above
 * Errors as for the other entry points. */
ff_status ff_global_column_attention(const ff_global_desc* desc, const ff_global_weights* w,
                                     const void* m, const float* mask, void* out,
                                     void* ws, size_t ws_bytes, void* hip_stream);

/* Backward pass of the fused attention core (Section 6.3 benchmarks the fused scale + mask + bias softmax
 * forward and backward; Table 6 reports forward and backward per Evoformer layer).  The core, per batch row r
 * and head h, with scale = 1 / sqrt(head_dim) and M(t) = 0 if t == 1 else -inf:
 *   S[r,h,i,j] = scale q[r,h,i,:] . k[r,h,j,:] + bias[h,i,j] + M(mask[r,j]);  P = softmax over j of S
 *   ctx[r,h,i,:] = sum_j P[r,h,i,j] v[r,h,j,:];   o = g * ctx          (g: the gate after its sigmoid)
 * Given dout = dLoss/do the call returns
 *   dg = dout * ctx;  with dctx = dout * g:  dv[j] = sum_i P[i,j] dctx[i];  dP[i,j] = dctx[i] . v[j];
 *   dS = P * (dP - rowsum(P * dP));  dq[i] = scale sum_j dS[i,j] k[j];  dk[j] = scale sum_i dS[i,j] q[i];
 *   dbias[h,i,j] = sum_r dS[r,h,i,j].
 * The score matrix is recomputed tile by tile, never stored (Section 3.2).  A query without unmasked keys has
 * P = 0 and all of its gradients are zero.  q, k, v, g, dout and the four gradients are bfloat16
 * [rows, heads, length, head_dim]; bias and dbias float32 [heads, length, length] (both NULL for a module without
 * bias); mask float32 [rows, length] of 0/1 or NULL.  P, dS and dctx are rounded to bfloat16 as matrix-core
 * operands; logsumexp, delta and all accumulations are float32; dbias is summed over the rows in a fixed order. */
typedef struct {
    int32_t dtype;      /* ff_dtype; FF_BF16 only */
    int32_t rows;       /* batch rows R */
    int32_t heads;      /* H */
    int32_t length;     /* attended length L (queries and keys) */
    int32_t head_dim;   /* 8, 16 or 32 */
} ff_core_desc;

/* Bytes of device workspace (logsumexp and delta per query, dctx, position-contiguous copies of q, k, v and dctx,
 * two tiled copies of the bias, partial sums of dbias over groups of rows: about six times the size of q plus a
 * few times that of the bias, never a score-sized tensor); 0 if desc is invalid or unsupported. */
size_t ff_attention_core_backward_workspace_bytes(const ff_core_desc* desc);

/* All tensor pointers are device pointers, 16-byte aligned; gradient tensors must not overlap the inputs or
 * each other; ws 256-byte aligned.  Errors as for the other entry points. */
ff_status ff_attention_core_backward(const ff_core_desc* desc, const void* q, const void* k, const void* v,
                                     const void* g, const float* bias, const float* mask, const void* dout,
                                     void* dq, void* dk, void* dv, void* dg, float* dbias,
                                     void* ws, size_t ws_bytes, void* hip_stream);

/* For callers that cannot allocate: code under HIP graph capture, tight serving loops and
 * harnesses that forbid hipMalloc, which therefore have no workspace to hand over.
 * The same module as ff_attention_chunked, with the workspace taken from a device array that is
 * part of the library's own code object (ff_static_scratch_bytes() bytes, 48 MiB; every GPU
 * the library runs on holds its copy until the process ends) and chunk_rows chosen as the
 * largest number of batch rows whose workspace fits that array.  The call allocates and
 * frees nothing and synchronises nothing; the result is bit-identical to ff_gated_attention.
 * x, z, mask, out as for ff_gated_attention.
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU
 * (different streams, different threads) race and give undefined results; calls on one
 * stream, or ordered by events, are safe.  Nothing in the array has to survive from call to
 * call and nothing in it is assumed zero.
 * Errors as for ff_attention_chunked, and FF_EWORKSPACE if even one batch row of this shape
 * needs more than the array holds (the message gives both sizes), FF_EHIP if the array's
 * device address cannot be looked up. */
ff_status ff_gated_attention_static(const ff_attn_desc* desc, const ff_attn_weights* w,
                                    const void* x, const void* z, const float* mask,
                                    void* out, void* hip_stream);

/* Size in bytes of the library's own device array used by ff_gated_attention_static. */
size_t ff_static_scratch_bytes(void);

/* Name of the kernel family the SHAPE allows: "mfma_bf16" (matrix-core path) or "generic"
 * (float32 vector path).  NULL if desc is invalid.  A call takes the matrix-core family only
 * if, in addition, x, z, out and every weight pointer are 16-byte aligned and the chunk has
 * fewer than 2^22 attention work items; ff_attention_last_path tells what a call really took. */
const char* ff_attention_path(const ff_attn_desc* desc);

/* Kernel family that the last attention call on this thread launched ("mfma_bf16" or
 * "generic"; "" before the first call or if that call was rejected before choosing).  This
 * is an observation, not a prediction: tests and the benchmark report assert on it. */
const char* ff_attention_last_path(void);

/* Launch timer, a diagnostic for benchmarks (no part of the attention path).  While it is on,
 * every kernel launch of the library is bracketed by two HIP events recorded on the launch
 * stream.  ff_profile_enable(on) clears earlier records.  ff_profile_collect waits for the
 * recorded events and returns, per kernel kind k < ff_profile_kinds(), the summed duration in
 * milliseconds and the number of launches (arrays of ff_profile_kinds() entries, host memory),
 * then clears the records.  ff_profile_name(k) names the kind.  Not thread-safe against
 * concurrent attention calls on other threads' streams beyond a mutex around the records. */
void ff_profile_enable(int32_t on);
int32_t ff_profile_kinds(void);
const char* ff_profile_name(int32_t kind);
ff_status ff_profile_collect(double* total_ms, int64_t* launches);

/* Calibration probes for the benchmark report (no part of the attention path): what this GPU
 * sustains on a bare loop of 32x32x16 bf16 matrix instructions, on a plain copy and on loops of one
 * vector instruction, so that roofline fractions can be quoted against measured as well as published
 * peaks.  Each only enqueues one kernel on hip_stream; time them with the launch timer above (kinds
 * "probe: mfma loop", "probe: copy", "probe: vector loop").
 *   ff_probe_mfma: sink = device buffer of ff_probe_sink_bytes() bytes (receives sums nobody reads);
 *                  iters >= 1 rounds of four matrix instructions per wavefront; *flop (host) receives
 *                  the floating-point operations the launch performs.
 *   ff_probe_copy: dst[i] = src[i] for `bytes` bytes (device pointers and size multiples of 16):
 *                  `bytes` read + `bytes` written.
 *   ff_probe_valu: sink as for ff_probe_mfma; iters >= 1 rounds of 16 independent instructions per
 *                  wavefront, eight wavefronts per SIMD of a 256-unit chip; kind 0: v_fma_f32, 1: v_exp_f32
 *                  (the softmax's exponential), 2: v_cvt_pk_bf16_f32 (two floats to a bfloat16 pair),
 *                  3: v_dot2c_f32_bf16 (the partial denominators); *wave_insts (host) receives the number
 *                  of wavefront-wide instructions of that kind the launch issues.  Kinds 4 .. 7 ask whether
 *                  matrix and vector instructions overlap: rounds of four independent 32x32x16 bf16 matrix
 *                  instructions with nothing (4), 16 multiply-adds (5), 32 multiply-adds (6) or 16
 *                  exponentials (7) spread between them; *wave_insts then receives the number of rounds.
 * FF_EINVAL for bad arguments, FF_EHIP if the launch fails. */
size_t ff_probe_sink_bytes(void);
ff_status ff_probe_mfma(void* sink, int32_t iters, double* flop, void* hip_stream);
ff_status ff_probe_valu(void* sink, int32_t kind, int32_t iters, double* wave_insts, void* hip_stream);
ff_status ff_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/* Message for the last non-OK status returned on this thread ("" if none). */
const char* ff_last_error(void);

/* Library version string. */
const char* ff_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FF_H */
