"""GPU parity: the HIP library (through its C ABI) against the float64 CPU oracle, element by
element on the same seeded inputs.

Tolerances (the benchmark definition's): float32 max-abs 1e-4; bfloat16 max-abs 2e-2 and
relative L2 1e-2.  The oracle never rounds; the library rounds q/k/v/gate, the softmax
weights, the gated context and the output to bfloat16 in FF_BF16.
"""
import numpy as np
import pytest
import torch

import paper_2203_00854_amd as P
from oracle import evoformer_attention as O
from paper_2203_00854_amd import inputs as I
from helpers import small_spec, f64_inputs, max_abs, rel_l2

pytestmark = pytest.mark.gpu

ROW, COL, TS, TE = I.MODE_ROW, I.MODE_COL, I.MODE_TRI_START, I.MODE_TRI_END
DEV = "cuda:0"


def to_np(t):
    return t.float().cpu().numpy().astype(np.float64)


def check(got, ref, dtype, what=""):
    ma, rl = max_abs(got, ref), rel_l2(got, ref)
    print(f"{what}: max_abs={ma:.3e} rel_l2={rl:.3e}", flush=True)
    assert np.isfinite(got).all()
    if dtype == "f32":
        assert ma <= 1e-4, (what, ma)
    else:
        assert ma <= 2e-2, (what, ma)
        assert rl <= 1e-2, (what, rl)


def run_case(case, chunk_rows=None):
    desc, w, x, z, mask = P.to_device(case, DEV)
    if chunk_rows is None:
        out = P.ff_gated_attention(desc, w, x, z, mask)
    else:
        out = P.ff_attention_chunked(desc, w, x, z, mask, chunk_rows=chunk_rows)
    torch.cuda.synchronize()
    return out


def spread(n, count, step, first=3):
    """count indices below n, `step` apart modulo n (step coprime to n and odd, so that the sample
    walks through every residue modulo 8 and 64: every wavefront slot of a block, odd and even
    blocks, first and last rows of a chunk)."""
    assert np.gcd(step, n) == 1
    return sorted({(first + step * k) % n for k in range(count)})


def oracle_case(case, rows=None):
    x, z, m, w = f64_inputs(case)
    sp = case.spec
    return O.gated_attention(sp.mode, x, z, m, w, sp.heads, sp.ln_eps, rows=rows)


# ----------------------------------------------------------------------------- LayerNorm
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,c", [(1, 8), (37, 32), (1000, 64), (4099, 128), (513, 256), (129, 384), (65, 1024),
                                    (33, 100), (17, 2048), (9, 4096), (5, 7), (3, 8192)])
def test_layernorm(dtype, rows, c):
    key = I.stream_key(I.SEED, f"ln_{dtype}_{rows}_{c}", "x")
    x = I.to_storage(I.normal(key, rows * c) * 2.0 + 0.5, dtype).reshape(rows, c)
    g = I.to_storage(1 + 0.1 * I.normal(I.stream_key(I.SEED, "ln", "g"), c), dtype)
    b = I.to_storage(0.1 * I.normal(I.stream_key(I.SEED, "ln", "b"), c), dtype)
    ref = O.layer_norm(I.widen(x), I.widen(g), I.widen(b), 1e-5)

    def up(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
        return torch.from_numpy(a).to(DEV)

    y = P.ff_layernorm(up(x), up(g), up(b), 1e-5)
    torch.cuda.synchronize()
    got = to_np(y)
    if dtype == "f32":
        assert max_abs(got, ref) <= 2e-5
    else:   # one bfloat16 rounding of the result: relative 2^-9
        assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-6)


def test_layernorm_in_place_and_empty():
    x = torch.randn(64, 128, device=DEV)
    g = torch.ones(128, device=DEV)
    b = torch.zeros(128, device=DEV)
    ref = P.ff_layernorm(x, g, b)
    P.ff_layernorm(x, g, b, out=x)
    torch.cuda.synchronize()
    assert torch.equal(x, ref)
    e = torch.empty(0, 128, device=DEV)
    assert P.ff_layernorm(e, g, b).shape == (0, 128)


# ----------------------------------------------------------------------------- the five configs
def test_config1_row_fp32_tiny():
    case = I.make_case("c1_row_f32_tiny")
    check(to_np(run_case(case)), oracle_case(case), "f32", "config1")


def test_config2_row_bf16_training_crop():
    case = I.make_case("c2_row_bf16_train")
    check(to_np(run_case(case)), oracle_case(case), "bf16", "config2")


@pytest.mark.parametrize("name", ["c3_tri_start_bf16_256", "c3_tri_end_bf16_256"])
def test_config3_triangle_bf16(name):
    case = I.make_case(name)
    got = to_np(run_case(case))
    ref = oracle_case(case)
    check(got, ref, "bf16", name)
    # the residue mask leaves some batch rows without any valid key: their output is b_o
    dead = np.where(case.mask.sum(axis=1 if case.spec.mode == TS else 0) == 0)[0]
    assert len(dead) > 0
    bo = I.widen(case.weights["b_o"]).astype(np.float64)
    rows = got[dead] if case.spec.mode == TS else got[:, dead].transpose(1, 0, 2)
    assert max_abs(rows, np.broadcast_to(bo, rows.shape)) == 0.0


def test_config3_end_equals_transposed_start_on_gpu():
    """Triangle-end on z equals triangle-start on z with its first two axes swapped, swapped
    back.  The library treats both as the same problem with other strides, so this is bit-exact."""
    case_e = I.make_case("c3_tri_end_bf16_256")
    desc, w, x, z, mask = P.to_device(case_e, DEV)
    end = P.ff_gated_attention(desc, w, x, None, mask)
    desc_s = P.AttnDesc(P.FF_TRI_START, desc.dtype, desc.n_a, desc.n_b, desc.c, 0, desc.heads, desc.head_dim, desc.ln_eps)
    start_t = P.ff_gated_attention(desc_s, w, x.transpose(0, 1).contiguous(), None, mask.t().contiguous())
    torch.cuda.synchronize()
    assert torch.equal(end, start_t.transpose(0, 1))


def test_config4_column_bf16_extra_msa():
    """All 384 residue columns run on the GPU; the oracle (about 0.4 s per column on the host)
    evaluates 96 of them, 37 apart modulo 384: every position inside the attention kernel's 4-row
    blocks, odd and even blocks, the first and the last column."""
    case = I.make_case("c4_col_bf16_extra")
    got = to_np(run_case(case))
    assert P.ff_attention_last_path() == "mfma_bf16"
    rows = sorted(set(spread(384, 94, 37)) | {0, 383})
    assert {r % 8 for r in rows} == set(range(8))
    ref = oracle_case(case, rows=rows)                       # [len(rows), L, c]
    check(got[:, rows].transpose(1, 0, 2), ref, "bf16", "config4 sampled columns")


def test_config5_long_sequence_chunked_sampled_rows():
    """N_res = 2048 triangle-start, chunk = 64 rows, in the launch configuration the benchmark
    times.  The oracle evaluates 256 batch rows exactly (a batch row depends only on its own
    tokens plus the bias, which the oracle builds from all of x): eight in every chunk, at every
    position modulo 8 (the wavefront slots of the attention kernel's 8-row blocks) and modulo 64
    (first and last rows of chunks included).  Every one of the 2048 rows is then compared, bit
    for bit, with the unchunked call."""
    case = I.make_case("c5_tri_start_bf16_2048")
    desc, w, x, z, mask = P.to_device(case, DEV)
    free0 = torch.cuda.mem_get_info()[0]
    out = P.ff_attention_chunked(desc, w, x, None, None, chunk_rows=64)
    torch.cuda.synchronize()
    assert P.ff_attention_last_path() == "mfma_bf16"
    assert P.ff_attention_workspace_bytes(desc, 64) < 1 << 30
    whole = P.ff_gated_attention(desc, w, x, None, None)       # workspace 5.4 GiB: q, k, v, gate, context of all rows
    torch.cuda.synchronize()
    assert torch.equal(out, whole)
    del whole
    rows = sorted(set(spread(2048, 254, 265, first=5)) | {0, 2047})
    assert {r % 8 for r in rows} == set(range(8)) and {r // 64 for r in rows} == set(range(32))
    assert any(r % 64 == 0 for r in rows) and any(r % 64 == 63 for r in rows)
    got = to_np(out[rows])
    del out
    xw = case.widened("x")
    wts = {k: v.astype(np.float64) for k, v in case.widened_weights().items()}
    ref = O.gated_attention(TS, xw, None, None, wts, 4, 1e-5, rows=rows)
    check(got, ref, "bf16", "config5 sampled rows")
    assert free0 > 0


def test_config5_subcrop_chunked_equals_unchunked_oracle():
    """The 256-residue crop of the config-5 input through the chunked entry point (chunk 64)
    against the unchunked oracle."""
    big = I.SPECS["c5_tri_start_bf16_2048"]
    spec = I.CaseSpec("c5_subcrop", TS, "bf16", 256, 256, 128, 0, 4, 32, "none", chunk_rows=64, stream=big.name)
    case = I.make_case(spec)
    check(to_np(run_case(case, chunk_rows=64)), oracle_case(case), "bf16", "config5 sub-crop")


# ----------------------------------------------------------------------------- shapes that span tiles and leave ragged tails
SHAPES = [
    # mode, n_a, n_b, c, H, d, c_z, mask
    (ROW, 3, 70, 64, 2, 32, 24, "tail:5"),
    (ROW, 5, 129, 96, 3, 16, 40, "random:0.8"),
    (ROW, 2, 1, 32, 2, 8, 8, "none"),
    (COL, 77, 6, 64, 4, 8, 0, "tail:9"),
    (COL, 200, 3, 32, 2, 32, 0, "random:0.7"),
    (TS, 45, 45, 128, 4, 32, 0, "outer:0.9"),
    (TS, 97, 97, 64, 2, 16, 0, "none"),
    (TE, 45, 45, 128, 4, 32, 0, "outer:0.9"),
    (TE, 66, 66, 32, 1, 32, 0, "random:0.6"),
    (ROW, 4, 300, 256, 8, 32, 128, "tail:37"),
    (COL, 520, 5, 64, 8, 8, 0, "tail:100"),
    (ROW, 3, 40, 48, 3, 24, 20, "tail:3"),       # head_dim 24, channels not a power of two
    (TS, 33, 33, 100, 2, 64, 0, "none"),         # head_dim 64
    (TS, 530, 530, 32, 2, 32, 0, "tail:11"),     # 17 key tiles: the last 128-key bias group is only half there
    (ROW, 9, 700, 64, 2, 32, 16, "random:0.9"),  # 22 key tiles, nine batch rows (a ragged second block of rows)
    # many short items per persistent attention block: one bias group per item (the LDS buffers alternate from
    # item to item), four-row blocks without a bias, and six bias groups per item at d = 32
    (ROW, 1500, 40, 32, 4, 8, 16, "random:0.7"),
    (COL, 70, 1100, 32, 2, 16, 0, "tail:7"),
    (TS, 330, 330, 32, 4, 32, 0, "outer:0.9"),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode,n_a,n_b,c,H,d,c_z,mask", SHAPES)
def test_ragged_shapes(dtype, mode, n_a, n_b, c, H, d, c_z, mask):
    case = I.make_case(small_spec(mode, n_a, n_b, c, H, d, c_z=c_z, dtype=dtype, mask=mask))
    check(to_np(run_case(case)), oracle_case(case), dtype, case.spec.name)


@pytest.mark.parametrize("name", ["c2_row_bf16_train", "c3_tri_start_bf16_256", "c3_tri_end_bf16_256",
                                  "c4_col_bf16_extra", "c5_tri_start_bf16_2048"])
def test_bf16_configs_run_on_the_matrix_core_family(name):
    """The bfloat16 workloads of the benchmark must not fall back to the float32 vector family
    (device tensors from the binding are 16-byte aligned, which that family choice requires)."""
    sp = I.SPECS[name]
    desc = P.AttnDesc(sp.mode, P.FF_BF16, sp.n_a, sp.n_b, sp.c, sp.c_z, sp.heads, sp.head_dim, sp.ln_eps)
    assert P.ff_attention_path(desc) == "mfma_bf16"


def test_last_path_reports_the_family_that_really_ran():
    """The shape alone allows the matrix-core family; a weight view that is not 16-byte aligned
    sends the call to the float32 vector family, and the library says so."""
    case = I.make_case(small_spec(COL, 40, 6, 64, 4, 16, dtype="bf16", mask="tail:3"))
    desc, w, x, z, mask = P.to_device(case, DEV)
    a = P.ff_gated_attention(desc, w, x, z, mask)
    assert P.ff_attention_last_path() == "mfma_bf16"
    shifted = torch.empty(w["b_o"].numel() + 1, dtype=w["b_o"].dtype, device=DEV)
    shifted[1:] = w["b_o"]
    w2 = dict(w, b_o=shifted[1:])
    b = P.ff_gated_attention(desc, w2, x, z, mask)
    torch.cuda.synchronize()
    assert P.ff_attention_path(desc) == "mfma_bf16" and P.ff_attention_last_path() == "generic"
    check(to_np(b), to_np(a), "bf16", "generic family against matrix-core family")


def test_long_ragged_sequence_column_mode():
    """4100 attended positions (129 tiles of 32 keys, the last one ragged, 36 masked) for a few
    batch rows, head dim 32: many tiles per wavefront, a tail that is neither a multiple of 32 nor of 64."""
    case = I.make_case(small_spec(COL, 4100, 3, 64, 2, 32, dtype="bf16", mask="tail:36"))
    check(to_np(run_case(case)), oracle_case(case), "bf16", "long ragged column attention")


@pytest.mark.parametrize("mode,heads,d", [(COL, 2, 32), (TS, 2, 32), (COL, 8, 8), (TS, 4, 16)])
def test_reference_is_raised_when_late_keys_dominate(mode, heads, d):
    """The keys of the last two 32-key tiles beat everything before them by tens of log2 units
    for half of the queries (and lose by as much for the other half).  The kernel's running softmax
    reference, fixed by the first tile, has to be raised when those keys arrive.  The tokens of a
    group differ only by small noise, so the rounding of q and k is common to a group and the
    usual tolerance holds.  Head dims below 32 take the kernel's other route (the maximum of every
    tile, the next tile's contraction issued from inside the exponentials)."""
    L, late = 160, 96
    n_a, n_b = (L, 6) if mode == COL else (L, L)      # the pair representation is square
    case = I.make_case(small_spec(mode, n_a, n_b, 64, heads, d, dtype="bf16"))
    key = I.stream_key(I.SEED, "late_keys", "x")
    v = I.normal(key, 64)
    noise = I.normal(I.stream_key(I.SEED, "late_keys", "noise"), n_a * n_b * 64).reshape(n_a, n_b, 64)
    sign = np.where(np.arange(L) < late, -1.0, 1.0)
    sign = sign[:, None, None] if mode == COL else sign[None, :, None]
    case.x = I.to_storage(sign * v + 0.05 * noise, "bf16")
    for name in ("w_q", "w_k"):
        case.weights[name] = I.to_storage(5.0 * I.widen(case.weights[name]).astype(np.float64), "bf16")
    # the jump really is there: logits of the late group minus logits of the early group
    x, z, m, w = f64_inputs(case)
    xh = O.layer_norm(x, w["ln_g"], w["ln_b"], case.spec.ln_eps)
    tok = xh[:, 0] if mode == COL else xh[0]                  # [L, c]: one batch row
    q = (tok @ w["w_q"].T).reshape(L, heads, d)
    k = (tok @ w["w_k"].T).reshape(L, heads, d)
    s = np.einsum("qhe,khe->hqk", q, k) / np.sqrt(float(d)) * np.log2(np.e)
    jump = s[:, :, late:].max(axis=2) - s[:, :, :32].max(axis=2)
    assert jump.max() > 30.0
    check(to_np(run_case(case)), oracle_case(case), "bf16", f"late keys dominate, mode {mode}, d {d}")


@pytest.mark.parametrize("mode", [ROW, TS])
def test_large_token_means(mode):
    """Activations with a mean of twelve standard deviations per token.  The matrix-core family
    never subtracts the mean from x: the term -mean * (row sum of the folded weights) enters the
    contraction as bf16 hi + lo pairs and has to cancel a product that is an order of magnitude
    larger than the result."""
    n_a, n_b = (6, 96) if mode == ROW else (96, 96)
    case = I.make_case(small_spec(mode, n_a, n_b, 128, 4, 32, c_z=32, dtype="bf16", mask="tail:7"))
    off = I.normal(I.stream_key(I.SEED, "large_means", "offset"), n_a * n_b).reshape(n_a, n_b, 1)
    case.x = I.to_storage(6.0 + 2.0 * off + 0.5 * I.widen(case.x).astype(np.float64), "bf16")
    if case.z is not None:
        case.z = I.to_storage(-5.0 + 0.4 * I.widen(case.z).astype(np.float64), "bf16")
    check(to_np(run_case(case)), oracle_case(case), "bf16", f"large token means, mode {mode}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode,n_a,n_b,c,H,d,c_z,mask,chunk", [
    (ROW, 7, 70, 64, 2, 32, 24, "tail:5", 3),
    (COL, 77, 10, 64, 4, 8, 0, "tail:9", 4),
    (TS, 45, 45, 128, 4, 32, 0, "outer:0.9", 16),
    (TE, 45, 45, 128, 4, 32, 0, "random:0.8", 7),
    (TS, 20, 20, 32, 2, 8, 0, "none", 1),
    (ROW, 4, 33, 32, 2, 8, 8, "none", 100),
])
def test_chunked_is_bit_identical_to_unchunked(dtype, mode, n_a, n_b, c, H, d, c_z, mask, chunk):
    """Section 5.3: chunking a dimension that takes no part in the computation.  Batch rows
    are independent, so the chunked entry point must reproduce the unchunked bits."""
    case = I.make_case(small_spec(mode, n_a, n_b, c, H, d, c_z=c_z, dtype=dtype, mask=mask))
    a = run_case(case)
    b = run_case(case, chunk_rows=chunk)
    assert torch.equal(a, b)
    check(to_np(b), oracle_case(case), dtype, case.spec.name + f"/chunk{chunk}")


# ----------------------------------------------------------------------------- invariants on the GPU path
def test_row_mode_sequence_permutation_is_bit_exact():
    case = I.make_case(small_spec(ROW, 12, 64, 64, 4, 16, c_z=16, dtype="bf16", mask="random:0.8"))
    desc, w, x, z, mask = P.to_device(case, DEV)
    perm = torch.tensor([3, 0, 5, 1, 4, 2, 11, 10, 9, 8, 7, 6], device=DEV)
    a = P.ff_gated_attention(desc, w, x, z, mask)
    b = P.ff_gated_attention(desc, w, x[perm].contiguous(), z, mask[perm].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(a[perm], b)


def test_masked_key_content_is_irrelevant_on_gpu():
    case = I.make_case(small_spec(ROW, 4, 96, 64, 4, 16, c_z=16, dtype="bf16", mask="tail:20"))
    desc, w, x, z, mask = P.to_device(case, DEV)
    a = P.ff_gated_attention(desc, w, x, z, mask)
    x2 = x.clone()
    x2[:, 76:, :] = torch.randn_like(x2[:, 76:, :]) * 3
    b = P.ff_gated_attention(desc, w, x2, z, mask)
    torch.cuda.synchronize()
    assert torch.equal(a[:, :76], b[:, :76])


def test_fully_masked_rows_give_output_bias():
    case = I.make_case(small_spec(COL, 40, 9, 32, 2, 8, dtype="f32", mask="tail:3"))
    case.mask[:, 4] = 0.0
    got = to_np(run_case(case))
    bo = I.widen(case.weights["b_o"]).astype(np.float64)
    assert max_abs(got[:, 4], np.broadcast_to(bo, got[:, 4].shape)) == 0.0
    check(got, oracle_case(case), "f32", "fully masked column")


def test_workspace_too_small_is_an_error_not_a_fault():
    case = I.make_case(small_spec(ROW, 4, 33, 32, 2, 8, c_z=8, dtype="f32"))
    desc, w, x, z, mask = P.to_device(case, DEV)
    need = P.ff_attention_workspace_bytes(desc, 0)
    ws = torch.empty(need - 256, dtype=torch.uint8, device=DEV)
    with pytest.raises(P.FFError) as e:
        P.ff_gated_attention(desc, w, x, z, mask, ws=ws)
    assert e.value.status == 3


@pytest.mark.parametrize("mode,n_a,n_b,c,H,d,c_z,chunk", [
    (ROW, 16, 128, 128, 4, 32, 64, 0), (TS, 96, 96, 64, 2, 16, 0, 40), (COL, 200, 12, 64, 8, 8, 0, 0),
])
def test_calls_can_be_captured_in_a_hip_graph(mode, n_a, n_b, c, H, d, c_z, chunk):
    """The library only enqueues kernels on the caller's stream (no allocation, no synchronisation,
    no memset), so a call can be recorded into a HIP graph.  Every replay, with eager work and
    synchronisations in between, must reproduce the eager bits."""
    case = I.make_case(small_spec(mode, n_a, n_b, c, H, d, c_z=c_z, dtype="bf16", mask="tail:5"))
    desc, w, x, z, mask = P.to_device(case, DEV)
    ws = torch.empty(P.ff_attention_workspace_bytes(desc, chunk), dtype=torch.uint8, device=DEV)

    def call(out):
        if chunk:
            P.ff_attention_chunked(desc, w, x, z, mask, chunk_rows=chunk, out=out, ws=ws)
        else:
            P.ff_gated_attention(desc, w, x, z, mask, out=out, ws=ws)

    eager = torch.empty_like(x)
    call(eager)                                    # (also the one-time kernel attribute set-up)
    torch.cuda.synchronize()
    out = torch.zeros_like(x)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call(out)
    torch.cuda.synchronize()
    for rep in range(3):
        out.fill_(float("nan"))
        ws.random_(0, 255)                         # the workspace carries nothing from call to call
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
    x2 = x.clone()
    x.mul_(0.5)                                    # new input values through the same pointers
    ref2 = torch.empty_like(x)
    call(ref2)
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, ref2)
    assert not torch.equal(ref2, eager)
    x.copy_(x2)
