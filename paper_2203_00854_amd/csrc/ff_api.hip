// C ABI entry points of libff: argument checking, workspace carving, the chunk loop.
// All arithmetic of the path runs in the kernels of the other translation units.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "ff_common.h"

namespace ff {

// ---- launch timer: HIP events around kernel launches, on the launch stream -------------
static bool g_prof_on = false;
static std::mutex g_prof_mu;
struct ProfRec { int kind; hipEvent_t a, b; };
static std::vector<ProfRec> g_prof;
static std::vector<hipEvent_t> g_prof_pool;
static const char* kKindNames[KK_COUNT] = {"k_prep", "pair bias pass", "k_gemm<PROJ>", "k_attn",
                                           "k_gemm<OUT>", "k_layernorm", "generic family", "probe: mfma loop",
                                           "probe: copy", "k_tm_prep", "k_tm_proj", "k_tm_mul", "k_tm_out",
                                           "k_gca_kv", "k_gca_softmax", "k_gca_out",
                                           "k_bwd_stats", "k_bwd_dq", "k_bwd_dkv", "k_bwd_dbias", "probe: vector loop",
                                           "k_proj_attn"};

static hipEvent_t prof_event() {
    if (!g_prof_pool.empty()) {
        hipEvent_t e = g_prof_pool.back();
        g_prof_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void prof_begin(int kind, hipStream_t st) {
    if (!g_prof_on) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (g_prof.size() >= (1u << 18)) return;
    ProfRec r{kind, prof_event(), prof_event()};
    if (!r.a || !r.b) return;
    (void)hipEventRecord(r.a, st);
    g_prof.push_back(r);
}

void prof_end(int kind, hipStream_t st) {
    if (!g_prof_on) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (size_t i = g_prof.size(); i-- > 0;)
        if (g_prof[i].kind == kind) {
            (void)hipEventRecord(g_prof[i].b, st);
            return;
        }
}

static thread_local char g_err[512] = "";
static thread_local const char* g_last_path = "";     // kernel family of this thread's last attention call

ff_status fail(ff_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

ff_status check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FF_EHIP, "%s: %s", what, hipGetErrorString(e));
    return FF_OK;
}

static ff_status make_problem(const ff_attn_desc* d, Problem* p) {
    if (!d) return fail(FF_EINVAL, "desc is NULL");
    if (d->mode < FF_MSA_ROW || d->mode > FF_TRI_END) return fail(FF_EINVAL, "bad mode %d", d->mode);
    if (d->dtype != FF_F32 && d->dtype != FF_BF16) return fail(FF_EINVAL, "bad dtype %d", d->dtype);
    if (d->n_a < 1 || d->n_b < 1 || d->c < 1 || d->heads < 1 || d->head_dim < 1)
        return fail(FF_EINVAL, "non-positive size (n_a=%d n_b=%d c=%d heads=%d head_dim=%d)", d->n_a, d->n_b,
                    d->c, d->heads, d->head_dim);
    if (d->mode == FF_MSA_ROW && d->c_z < 1) return fail(FF_EINVAL, "row mode needs c_z >= 1 (got %d)", d->c_z);
    if ((d->mode == FF_TRI_START || d->mode == FF_TRI_END) && d->n_a != d->n_b)
        return fail(FF_EINVAL, "triangle modes need n_a == n_b (got %d, %d)", d->n_a, d->n_b);
    if (!(d->ln_eps >= 0.f)) return fail(FF_EINVAL, "ln_eps must be >= 0");
    if (d->head_dim > 128) return fail(FF_EUNSUPPORTED, "head_dim %d > 128", d->head_dim);
    if (d->c > 8192 || (d->mode == FF_MSA_ROW && d->c_z > 8192))
        return fail(FF_EUNSUPPORTED, "c or c_z > 8192");
    if ((int64_t)d->heads * d->head_dim > 16384) return fail(FF_EUNSUPPORTED, "heads*head_dim > 16384");
    p->mode = d->mode;
    p->dtype = d->dtype;
    p->n_a = d->n_a;
    p->n_b = d->n_b;
    p->c = d->c;
    p->c_z = d->mode == FF_MSA_ROW ? d->c_z : 0;
    p->H = d->heads;
    p->d = d->head_dim;
    p->Hd = d->heads * d->head_dim;
    p->eps = d->ln_eps;
    const bool along_b = (d->mode == FF_MSA_ROW || d->mode == FF_TRI_START);
    p->R = along_b ? d->n_a : d->n_b;
    p->L = along_b ? d->n_b : d->n_a;
    p->sr = along_b ? d->n_b : 1;
    p->sl = along_b ? 1 : d->n_b;
    p->has_bias = d->mode != FF_MSA_COL;
    return FF_OK;
}

// Both families need at most max(mfma, generic) bytes; the size reported to the caller is that
// maximum so that the family can still be chosen per call (the matrix-core kernels use 16-byte
// accesses and are only taken when every pointer is 16-byte aligned).
static size_t carve(const Problem& p, int chunk, Workspace* ws, void* base, bool fast) {
    return fast ? mfma_workspace(p, chunk, ws, base) : generic_workspace(p, chunk, ws, base);
}
static size_t workspace_need(const Problem& p, int chunk) {
    Workspace tmp;
    size_t a = generic_workspace(p, chunk, &tmp, nullptr);
    if (mfma_supported(p)) {
        size_t b = mfma_workspace(p, chunk, &tmp, nullptr);
        if (b > a) a = b;
    }
    return a;
}
static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }
static bool overlaps(const void* a, size_t an, const void* b, size_t bn) {
    return (uintptr_t)a < (uintptr_t)b + bn && (uintptr_t)b < (uintptr_t)a + an;
}

static ff_status run(const ff_attn_desc* desc, const ff_attn_weights* w, const void* x, const void* z,
                     const float* mask, void* out, void* wsp, size_t ws_bytes, void* stream_, int chunk_rows,
                     bool chunked, bool residual = false) {
    Problem p;
    ff_status st = make_problem(desc, &p);
    if (st != FF_OK) return st;
    if (chunked && chunk_rows < 1) return fail(FF_EINVAL, "chunk_rows must be >= 1 (got %d)", chunk_rows);
    if (!w) return fail(FF_EINVAL, "weights is NULL");
    if (!x || !out) return fail(FF_EINVAL, "x or out is NULL");
    if (!w->ln_g || !w->ln_b || !w->w_q || !w->w_k || !w->w_v || !w->w_g || !w->b_g || !w->w_o || !w->b_o)
        return fail(FF_EINVAL, "a required weight pointer is NULL");
    if (p.mode == FF_MSA_ROW) {
        if (!z) return fail(FF_EINVAL, "row mode needs z");
        if (!w->lnz_g || !w->lnz_b || !w->w_b) return fail(FF_EINVAL, "row mode needs lnz_g, lnz_b and w_b");
    } else {
        if (z) return fail(FF_EINVAL, "z must be NULL outside row mode");
        if (p.has_bias && !w->w_b) return fail(FF_EINVAL, "triangle modes need w_b");
    }
    const size_t esz = p.dtype == FF_F32 ? 4 : 2;
    const size_t x_bytes = (size_t)p.n_a * p.n_b * p.c * esz;
    const size_t z_bytes = (size_t)p.n_b * p.n_b * p.c_z * esz;
    // (the residual update may replace x in place: every kernel has read x, or the part of it that a
    // chunk needs, before the output projection of that chunk stores, and an element of the
    // residual is read by the very lane that stores it)
    if ((overlaps(out, x_bytes, x, x_bytes) && !(residual && out == x)) || (z && overlaps(out, x_bytes, z, z_bytes)))
        return fail(FF_EINVAL, residual ? "out must be x itself or not overlap x, and must not overlap z"
                                        : "out must not overlap x or z");
    int chunk = chunked ? (chunk_rows < p.R ? chunk_rows : p.R) : p.R;
    const size_t need = workspace_need(p, chunk);
    if (!wsp) return fail(FF_EINVAL, "workspace is NULL (%zu bytes needed)", need);
    if (((uintptr_t)wsp & 255u) != 0) return fail(FF_EINVAL, "workspace must be 256-byte aligned");
    if (ws_bytes < need) return fail(FF_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", ws_bytes, need);
    if (overlaps(out, x_bytes, wsp, need)) return fail(FF_EINVAL, "out must not overlap the workspace");

    hipStream_t stream = (hipStream_t)stream_;
    bool fast = mfma_supported(p) && mfma_chunk_ok(p, chunk) && aligned16(x) && aligned16(out) && aligned16(z);
    const void* wp[] = {w->ln_g, w->ln_b, w->lnz_g, w->lnz_b, w->w_q, w->w_k, w->w_v, w->w_b, w->w_g, w->b_g, w->w_o, w->b_o};
    for (const void* q : wp) fast = fast && aligned16(q);
    Workspace ws;
    carve(p, chunk, &ws, wsp, fast);
    g_last_path = fast ? "mfma_bf16" : "generic";
    if (fast) {
        st = mfma_prepare(p, *w, x, z, ws, stream);
    } else {
        Timed t(KK_GENERIC, stream);
        st = generic_prepare(p, *w, x, z, ws, stream);
    }
    if (st != FF_OK) return st;
    for (int r0 = 0; r0 < p.R; r0 += chunk) {
        int rows = p.R - r0 < chunk ? p.R - r0 : chunk;
        if (fast) {
            st = mfma_chunk(p, *w, x, mask, residual ? x : nullptr, out, ws, r0, rows, stream);
        } else {
            Timed t(KK_GENERIC, stream);
            st = generic_chunk(p, *w, x, mask, residual ? x : nullptr, out, ws, r0, rows, stream);
        }
        if (st != FF_OK) return st;
    }
    return FF_OK;
}

// ---- device memory of the library's own, for callers that cannot hand over a workspace -------
// ff_gated_attention_static runs the chunked path with this array as its workspace.  Every GPU the
// library runs on holds its own copy until the process ends.  In host code the array's name is only
// a handle for hipGetSymbolAddress: the device address is looked up once per device (with that
// device current) and used everywhere after that.
constexpr size_t kScratchBytes = (size_t)48 << 20;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices] = {};

static ff_status scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(FF_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(FF_EUNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(FF_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return FF_OK;
}

// largest chunk (batch rows per launch sequence) whose workspace fits `limit` bytes; 0 if not even one row does
static int largest_chunk_within(const Problem& p, size_t limit) {
    if (workspace_need(p, 1) > limit) return 0;
    int lo = 1, hi = p.R;                      // workspace_need grows with the chunk
    while (lo < hi) {
        const int mid = lo + (hi - lo + 1) / 2;
        if (workspace_need(p, mid) <= limit) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

}  // namespace ff

using namespace ff;

extern "C" {

ff_status ff_layernorm(const void* x, const void* gamma, const void* beta, void* y, int64_t rows, int32_t c,
                       float eps, int32_t dt, void* hip_stream) {
    if (dt != FF_F32 && dt != FF_BF16) return fail(FF_EINVAL, "bad dtype %d", dt);
    if (rows < 0 || c < 1 || c > 8192) return fail(FF_EINVAL, "bad size rows=%lld c=%d", (long long)rows, c);
    if (!(eps >= 0.f)) return fail(FF_EINVAL, "eps must be >= 0");
    if (rows == 0) return FF_OK;
    if (!x || !gamma || !beta || !y) return fail(FF_EINVAL, "NULL pointer");
    Timed t(KK_LAYERNORM, (hipStream_t)hip_stream);
    return layernorm_launch(x, gamma, beta, y, rows, c, eps, dt, (hipStream_t)hip_stream);
}

static ff_status check_trimul(const ff_trimul_desc* d) {
    if (!d) return fail(FF_EINVAL, "desc is NULL");
    if (d->dtype != FF_F32 && d->dtype != FF_BF16) return fail(FF_EINVAL, "bad dtype %d", d->dtype);
    if (d->n < 1 || d->c_z < 1 || d->c < 1) return fail(FF_EINVAL, "non-positive size (n=%d c_z=%d c=%d)", d->n, d->c_z, d->c);
    if (d->incoming != 0 && d->incoming != 1) return fail(FF_EINVAL, "incoming must be 0 or 1 (got %d)", d->incoming);
    if (!(d->ln_eps >= 0.f)) return fail(FF_EINVAL, "ln_eps must be >= 0");
    if (d->n > 16384) return fail(FF_EUNSUPPORTED, "n %d > 16384", d->n);
    if (!trimul_supported(d->dtype, d->c_z, d->c))
        return fail(FF_EUNSUPPORTED, "triangle multiplication: bfloat16 only, c_z and c multiples of 32 up to 128 "
                                     "(got dtype %d, c_z %d, c %d)", d->dtype, d->c_z, d->c);
    return FF_OK;
}

size_t ff_triangle_multiplication_workspace_bytes(const ff_trimul_desc* desc) {
    if (check_trimul(desc) != FF_OK) return 0;
    return trimul_workspace(desc->n, desc->c_z, desc->c);
}

ff_status ff_triangle_multiplication(const ff_trimul_desc* desc, const ff_trimul_weights* w, const void* z,
                                     const float* mask, void* out, int32_t residual, void* ws, size_t ws_bytes,
                                     void* hip_stream) {
    ff_status st = check_trimul(desc);
    if (st != FF_OK) return st;
    if (residual != 0 && residual != 1) return fail(FF_EINVAL, "residual must be 0 or 1 (got %d)", residual);
    if (!w || !z || !out) return fail(FF_EINVAL, "weights, z or out is NULL");
    const void* wp[] = {w->ln_g, w->ln_b, w->w_ap, w->b_ap, w->w_ag, w->b_ag, w->w_bp, w->b_bp, w->w_bg, w->b_bg,
                        w->w_g, w->b_g, w->lno_g, w->lno_b, w->w_o, w->b_o};
    for (const void* q : wp)
        if (!q) return fail(FF_EINVAL, "a weight pointer is NULL");
    if (!aligned16(z) || !aligned16(out)) return fail(FF_EINVAL, "z and out must be 16-byte aligned");
    const size_t z_bytes = (size_t)desc->n * desc->n * desc->c_z * 2;
    if (overlaps(out, z_bytes, z, z_bytes) && !(residual && out == z))
        return fail(FF_EINVAL, residual ? "out must be z itself or not overlap z" : "out must not overlap z");
    const size_t need = trimul_workspace(desc->n, desc->c_z, desc->c);
    if (!ws) return fail(FF_EINVAL, "workspace is NULL (%zu bytes needed)", need);
    if (((uintptr_t)ws & 255u) != 0) return fail(FF_EINVAL, "workspace must be 256-byte aligned");
    if (ws_bytes < need) return fail(FF_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", ws_bytes, need);
    if (overlaps(out, z_bytes, ws, need) || overlaps(z, z_bytes, ws, need))
        return fail(FF_EINVAL, "z and out must not overlap the workspace");
    return trimul_run(*desc, *w, z, mask, residual != 0, out, ws, (hipStream_t)hip_stream);
}

static ff_status check_global(const ff_global_desc* d) {
    if (!d) return fail(FF_EINVAL, "desc is NULL");
    if (d->dtype != FF_F32 && d->dtype != FF_BF16) return fail(FF_EINVAL, "bad dtype %d", d->dtype);
    if (d->n_seq < 1 || d->n_res < 1 || d->c < 1 || d->heads < 1 || d->head_dim < 1)
        return fail(FF_EINVAL, "non-positive size (n_seq=%d n_res=%d c=%d heads=%d head_dim=%d)", d->n_seq, d->n_res, d->c,
                    d->heads, d->head_dim);
    if (!(d->ln_eps >= 0.f)) return fail(FF_EINVAL, "ln_eps must be >= 0");
    if ((int64_t)d->n_seq * d->n_res > ((int64_t)1 << 31) - 1) return fail(FF_EUNSUPPORTED, "more than 2^31 tokens");
    if (!global_supported(*d))
        return fail(FF_EUNSUPPORTED, "global column attention: bfloat16 only, c a multiple of 32 up to 128, head_dim 8 or 16, "
                                     "heads*head_dim 32, 64 or 128 (got dtype %d, c %d, heads %d, head_dim %d)",
                    d->dtype, d->c, d->heads, d->head_dim);
    return FF_OK;
}

size_t ff_global_column_attention_workspace_bytes(const ff_global_desc* desc) {
    if (check_global(desc) != FF_OK) return 0;
    return global_workspace(*desc);
}

ff_status ff_global_column_attention(const ff_global_desc* desc, const ff_global_weights* w, const void* m,
                                     const float* mask, void* out, void* ws, size_t ws_bytes, void* hip_stream) {
    ff_status st = check_global(desc);
    if (st != FF_OK) return st;
    if (!w || !m || !out) return fail(FF_EINVAL, "weights, m or out is NULL");
    const void* wp[] = {w->ln_g, w->ln_b, w->w_q, w->w_k, w->w_v, w->w_g, w->b_g, w->w_o, w->b_o};
    for (const void* q : wp)
        if (!q) return fail(FF_EINVAL, "a weight pointer is NULL");
    if (!aligned16(m) || !aligned16(out)) return fail(FF_EINVAL, "m and out must be 16-byte aligned");
    const size_t m_bytes = (size_t)desc->n_seq * desc->n_res * desc->c * 2;
    if (overlaps(out, m_bytes, m, m_bytes)) return fail(FF_EINVAL, "out must not overlap m");
    const size_t need = global_workspace(*desc);
    if (!ws) return fail(FF_EINVAL, "workspace is NULL (%zu bytes needed)", need);
    if (((uintptr_t)ws & 255u) != 0) return fail(FF_EINVAL, "workspace must be 256-byte aligned");
    if (ws_bytes < need) return fail(FF_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", ws_bytes, need);
    if (overlaps(out, m_bytes, ws, need) || overlaps(m, m_bytes, ws, need))
        return fail(FF_EINVAL, "m and out must not overlap the workspace");
    return global_run(*desc, *w, m, mask, out, ws, (hipStream_t)hip_stream);
}

static ff_status check_core(const ff_core_desc* d) {
    if (!d) return fail(FF_EINVAL, "desc is NULL");
    if (d->dtype != FF_F32 && d->dtype != FF_BF16) return fail(FF_EINVAL, "bad dtype %d", d->dtype);
    if (d->rows < 1 || d->heads < 1 || d->length < 1 || d->head_dim < 1)
        return fail(FF_EINVAL, "non-positive size (rows=%d heads=%d length=%d head_dim=%d)", d->rows, d->heads, d->length, d->head_dim);
    if (d->length > 16384) return fail(FF_EUNSUPPORTED, "length %d > 16384", d->length);
    const int64_t tiles = (int64_t)d->rows * d->heads * ((d->length + 31) / 32);
    const int64_t btiles = (int64_t)d->heads * ((d->length + 31) / 32) * ((d->length + 31) / 32);
    if (tiles > ((int64_t)1 << 30) || btiles > ((int64_t)1 << 30)) return fail(FF_EUNSUPPORTED, "too many tiles for one launch");
    if (!core_backward_supported(*d))
        return fail(FF_EUNSUPPORTED, "attention core backward: bfloat16 only, head_dim 8, 16 or 32 (got dtype %d, head_dim %d)",
                    d->dtype, d->head_dim);
    return FF_OK;
}

size_t ff_attention_core_backward_workspace_bytes(const ff_core_desc* desc) {
    if (check_core(desc) != FF_OK) return 0;
    return core_backward_workspace(*desc);
}

ff_status ff_attention_core_backward(const ff_core_desc* desc, const void* q, const void* k, const void* v, const void* g,
                                     const float* bias, const float* mask, const void* dout, void* dq, void* dk, void* dv,
                                     void* dg, float* dbias, void* ws, size_t ws_bytes, void* hip_stream) {
    ff_status st = check_core(desc);
    if (st != FF_OK) return st;
    if (!q || !k || !v || !g || !dout || !dq || !dk || !dv || !dg) return fail(FF_EINVAL, "a required tensor pointer is NULL");
    if ((bias == nullptr) != (dbias == nullptr)) return fail(FF_EINVAL, "dbias must be given exactly when bias is");
    if (!aligned16(bias) || !aligned16(dbias)) return fail(FF_EINVAL, "bias and dbias must be 16-byte aligned");
    const void* ptrs[] = {q, k, v, g, dout, dq, dk, dv, dg};
    for (const void* t : ptrs)
        if (!aligned16(t)) return fail(FF_EINVAL, "tensor pointers must be 16-byte aligned");
    const size_t n_bytes = (size_t)desc->rows * desc->heads * desc->length * desc->head_dim * 2;
    const void* ins[] = {q, k, v, g, dout};
    void* outs[] = {dq, dk, dv, dg};
    for (void* o : outs) {
        for (const void* in : ins)
            if (overlaps(o, n_bytes, in, n_bytes)) return fail(FF_EINVAL, "a gradient tensor overlaps an input");
        for (void* o2 : outs)
            if (o != o2 && overlaps(o, n_bytes, o2, n_bytes)) return fail(FF_EINVAL, "gradient tensors overlap each other");
    }
    const size_t need = core_backward_workspace(*desc);
    if (!ws) return fail(FF_EINVAL, "workspace is NULL (%zu bytes needed)", need);
    if (((uintptr_t)ws & 255u) != 0) return fail(FF_EINVAL, "workspace must be 256-byte aligned");
    if (ws_bytes < need) return fail(FF_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", ws_bytes, need);
    return core_backward_run(*desc, q, k, v, g, bias, mask, dout, dq, dk, dv, dg, dbias, ws, (hipStream_t)hip_stream);
}

size_t ff_attention_workspace_bytes(const ff_attn_desc* desc, int32_t chunk_rows) {
    Problem p;
    if (make_problem(desc, &p) != FF_OK) return 0;
    if (chunk_rows < 0) {
        fail(FF_EINVAL, "chunk_rows must be >= 0");
        return 0;
    }
    int chunk = (chunk_rows == 0 || chunk_rows > p.R) ? p.R : chunk_rows;
    return workspace_need(p, chunk);
}

ff_status ff_gated_attention(const ff_attn_desc* desc, const ff_attn_weights* w, const void* x, const void* z,
                             const float* mask, void* out, void* ws, size_t ws_bytes, void* hip_stream) {
    return run(desc, w, x, z, mask, out, ws, ws_bytes, hip_stream, 0, false);
}

ff_status ff_attention_chunked(const ff_attn_desc* desc, const ff_attn_weights* w, const void* x, const void* z,
                               const float* mask, void* out, void* ws, size_t ws_bytes, void* hip_stream,
                               int32_t chunk_rows) {
    return run(desc, w, x, z, mask, out, ws, ws_bytes, hip_stream, chunk_rows, true);
}

ff_status ff_gated_attention_residual(const ff_attn_desc* desc, const ff_attn_weights* w, const void* x,
                                      const void* z, const float* mask, void* out, void* ws, size_t ws_bytes,
                                      void* hip_stream, int32_t chunk_rows) {
    if (chunk_rows < 0) return fail(FF_EINVAL, "chunk_rows must be >= 0 (got %d)", chunk_rows);
    return run(desc, w, x, z, mask, out, ws, ws_bytes, hip_stream, chunk_rows, chunk_rows > 0, true);
}

ff_status ff_gated_attention_static(const ff_attn_desc* desc, const ff_attn_weights* w, const void* x, const void* z,
                                    const float* mask, void* out, void* hip_stream) {
    Problem p;
    ff_status st = make_problem(desc, &p);
    if (st != FF_OK) return st;
    const int chunk = largest_chunk_within(p, kScratchBytes);
    if (chunk < 1)
        return fail(FF_EWORKSPACE, "shape too large for the static scratch: one batch row needs %zu bytes, %zu available",
                    workspace_need(p, 1), kScratchBytes);
    void* ptr = nullptr;
    st = scratch_of_current_device(&ptr);
    if (st != FF_OK) return st;
    return run(desc, w, x, z, mask, out, ptr, kScratchBytes, hip_stream, chunk, true);
}

size_t ff_static_scratch_bytes(void) { return kScratchBytes; }

const char* ff_attention_path(const ff_attn_desc* desc) {
    Problem p;
    if (make_problem(desc, &p) != FF_OK) return nullptr;
    return mfma_supported(p) ? "mfma_bf16" : "generic";
}

const char* ff_attention_last_path(void) { return g_last_path; }

void ff_profile_enable(int32_t on) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (auto& r : g_prof) {
        g_prof_pool.push_back(r.a);
        g_prof_pool.push_back(r.b);
    }
    g_prof.clear();
    g_prof_on = on != 0;
}

int32_t ff_profile_kinds(void) { return KK_COUNT; }

const char* ff_profile_name(int32_t kind) { return (kind >= 0 && kind < KK_COUNT) ? kKindNames[kind] : nullptr; }

ff_status ff_profile_collect(double* total_ms, int64_t* launches) {
    if (!total_ms || !launches) return fail(FF_EINVAL, "NULL pointer");
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (int i = 0; i < KK_COUNT; ++i) {
        total_ms[i] = 0.0;
        launches[i] = 0;
    }
    ff_status st = FF_OK;
    for (auto& r : g_prof) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess)
            st = fail(FF_EHIP, "launch timer: event read failed");
        else {
            total_ms[r.kind] += ms;
            launches[r.kind] += 1;
        }
        g_prof_pool.push_back(r.a);
        g_prof_pool.push_back(r.b);
    }
    g_prof.clear();
    return st;
}

const char* ff_last_error(void) { return g_err; }

const char* ff_version(void) { return "libff 0.1 (gfx950)"; }

}  // extern "C"
