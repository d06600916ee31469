"""GPU parity of the residual update x + module(x) (ff_gated_attention_residual) against the
float64 CPU oracle, and against the library's own module output.

Tolerance.  The module output alone meets max-abs 2e-2 / relative L2 1e-2 in bfloat16.  The
update is one more float32 addition followed by the ONLY rounding to bfloat16, and that last
rounding is relative to the sum: half a unit in the last place of a bfloat16 number t is at most
2^-8 |t|.  So an element may differ from the oracle by 2e-2 + 2^-8 |x + y| (x has unit variance,
|x + y| reaches 6 at the benchmark shapes, where half an ulp alone is 1.6e-2).  float32: 1e-4
plus 2^-23 |x + y|.
"""
import numpy as np
import pytest
import torch

import paper_2203_00854_amd as P
from oracle import evoformer_attention as O
from paper_2203_00854_amd import inputs as I
from helpers import small_spec, f64_inputs, rel_l2
from test_gpu_parity import SHAPES, to_np

pytestmark = pytest.mark.gpu

ROW, COL, TS, TE = I.MODE_ROW, I.MODE_COL, I.MODE_TRI_START, I.MODE_TRI_END
DEV = "cuda:0"


def check_update(got, ref, dtype, what):
    err = np.abs(got - ref)
    allowed = (2e-2 + 2.0 ** -8 * np.abs(ref)) if dtype == "bf16" else (1e-4 + 2.0 ** -23 * np.abs(ref))
    worst = float((err - allowed).max())
    rl = rel_l2(got, ref)
    print(f"{what}: max_abs={err.max():.3e} worst margin={worst:.3e} rel_l2={rl:.3e}", flush=True)
    assert np.isfinite(got).all()
    assert worst <= 0.0, (what, worst)
    assert rl <= (1e-2 if dtype == "bf16" else 1e-5), (what, rl)


def oracle_update(case, rows=None):
    x, z, m, w = f64_inputs(case)
    sp = case.spec
    return O.gated_attention_residual(sp.mode, x, z, m, w, sp.heads, sp.ln_eps, rows=rows)


def check_against_module(upd, x, y, dtype):
    """The update holds round(x + y32) where the module output holds round(y32): the two entry
    points may differ by the two roundings only."""
    upd, x, y = to_np(upd), to_np(x), to_np(y)
    half_ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -23
    slack = half_ulp * (np.abs(y) + np.abs(upd)) * 1.01 + 1e-30
    assert (np.abs(upd - (x + y)) <= slack).all()


def run_update(case, chunk_rows=0, in_place=False):
    desc, w, x, z, mask = P.to_device(case, DEV)
    xin = x.clone() if in_place else x
    out = P.ff_gated_attention_residual(desc, w, xin, z, mask, chunk_rows=chunk_rows, in_place=in_place)
    torch.cuda.synchronize()
    if in_place:
        assert out.data_ptr() == xin.data_ptr()
    else:
        assert torch.equal(xin, x)
    return out


@pytest.mark.parametrize("name", ["c1_row_f32_tiny", "c2_row_bf16_train", "c3_tri_start_bf16_256",
                                  "c3_tri_end_bf16_256"])
def test_update_at_the_benchmark_shapes(name):
    case = I.make_case(name)
    dtype = case.spec.dtype
    desc, w, x, z, mask = P.to_device(case, DEV)
    upd = run_update(case)
    check_update(to_np(upd), oracle_update(case), dtype, name + " update")
    y = P.ff_gated_attention(desc, w, x, z, mask)
    torch.cuda.synchronize()
    check_against_module(upd, x, y, dtype)
    # in place, and chunked in place (a ragged last chunk): the same bits
    assert torch.equal(run_update(case, in_place=True), upd)
    assert torch.equal(run_update(case, chunk_rows=24, in_place=True), upd)
    assert torch.equal(run_update(case, chunk_rows=64), upd)


def test_update_column_mode_sampled_columns():
    """The extra-MSA column attention shape: every column on the GPU, 48 of them (37 apart modulo
    384: every position inside the kernel's row blocks) in the oracle."""
    case = I.make_case("c4_col_bf16_extra")
    upd = run_update(case, in_place=True)
    rows = sorted({(5 + 37 * k) % 384 for k in range(48)})
    check_update(to_np(upd)[:, rows].transpose(1, 0, 2), oracle_update(case, rows=rows), "bf16", "config4 update")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode,n_a,n_b,c,H,d,c_z,mask", SHAPES)
def test_update_ragged_shapes(dtype, mode, n_a, n_b, c, H, d, c_z, mask):
    case = I.make_case(small_spec(mode, n_a, n_b, c, H, d, c_z=c_z, dtype=dtype, mask=mask))
    upd = run_update(case)
    check_update(to_np(upd), oracle_update(case), dtype, case.spec.name + " update")
    assert torch.equal(run_update(case, in_place=True), upd)
    assert torch.equal(run_update(case, chunk_rows=5, in_place=True), upd)


def test_update_in_place_long_sequence_chunked():
    """The long-sequence use: the pair representation updated in place, 64 rows at a time, at 1024
    residues; the oracle evaluates sampled rows (a row needs only its own tokens and the bias)."""
    big = I.SPECS["c5_tri_start_bf16_2048"]
    spec = I.CaseSpec("c5_update_1024", TS, "bf16", 1024, 1024, 128, 0, 4, 32, "none", chunk_rows=64, stream=big.name)
    case = I.make_case(spec)
    upd = run_update(case, chunk_rows=64, in_place=True)
    rows = [0, 63, 64, 500, 1023]
    check_update(to_np(upd)[rows], oracle_update(case, rows=rows), "bf16", "1024-residue in-place update")


def test_partial_overlap_is_rejected():
    case = I.make_case(small_spec(ROW, 4, 33, 32, 2, 8, c_z=8, dtype="f32"))
    desc, w, x, z, mask = P.to_device(case, DEV)
    buf = torch.zeros(x.numel() + 64, dtype=x.dtype, device=DEV)
    xs = buf[:x.numel()].view_as(x).copy_(x)
    shifted = buf[64:].view_as(x)
    with pytest.raises(P.FFError) as e:
        P.ff_gated_attention_residual(desc, w, xs, z, mask, out=shifted)
    assert e.value.status == 1
