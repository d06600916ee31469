"""GPU parity of the triangular multiplicative update (ff_triangle_multiplication through the C ABI)
against the float64 oracle, element by element on the same seeded inputs.

Tolerance: relative L2 1e-2 as for the attention modules, and per element 3e-2 + 2^-8 |ref|.
The relative part is the rounding of the result itself to bfloat16 (half an ulp is up to 2^-8 of the value):
this module's outputs reach |out| = 4.7 at N_res = 256, where that last rounding alone is 1.6e-2.  The absolute
part covers the three bfloat16 roundings inside: the weights with the LayerNorm gain folded in (1.3e-2 at most
on the 259-residue case below), a and b (1.3e-2), the summed products t (0.9e-2); applied together to the
float64 oracle they give 2.29e-2 on that case (relative L2 4.4e-3), which is what the library returns to all
printed digits: the module chains two normalisations and a sum of 2 N_res products, so it is more sensitive
than the attention, whose bound of 2e-2 this replaces.  The residual form rounds z + out instead.
"""
import numpy as np
import pytest
import torch

import paper_2203_00854_amd as P
from oracle import triangle_multiplication as T
from paper_2203_00854_amd import inputs as I
from helpers import max_abs, rel_l2

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to_np(t):
    return t.float().cpu().numpy().astype(np.float64)


def oracle(case, residual=False):
    w = {k: v.astype(np.float64) for k, v in case.widened_weights().items()}
    sp = case.spec
    return T.triangle_multiplication(I.widen(case.z).astype(np.float64), case.mask, w, sp.incoming, sp.ln_eps, residual)


def check(got, ref, what, residual=False):      # (residual: same bound, the reference is z + out)
    ma, rl = max_abs(got, ref), rel_l2(got, ref)
    print(f"{what}: max_abs={ma:.3e} rel_l2={rl:.3e}", flush=True)
    assert np.isfinite(got).all()
    assert np.all(np.abs(got - ref) <= 3e-2 + 2.0 ** -8 * np.abs(ref)), (what, ma)
    assert rl <= 1e-2, (what, rl)


def run(case, residual=False, in_place=False):
    desc, w, z, mask = P.trimul_to_device(case, DEV)
    out = P.ff_triangle_multiplication(desc, w, z, mask, residual=residual, in_place=in_place)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("name", ["tm_out_bf16_256", "tm_in_bf16_256", "tm_out_bf16_384", "tm_in_bf16_384"])
def test_paper_shapes(name):
    """N_res = 256 (initial training) and 384 (fine-tuning), c_z = 128, hidden 128, residue mask with 5 % padding."""
    case = I.make_trimul_case(name)
    check(to_np(run(case)), oracle(case), name)


SHAPES = [   # n, c_z, c, mask: ragged sizes around the 32-token, 64-token and 128 x 128 tiles
    (1, 32, 32, "none"), (7, 32, 64, "random:0.7"), (33, 64, 32, "outer:0.8"), (45, 128, 128, "outer:0.9"),
    (64, 96, 64, "none"), (97, 64, 96, "random:0.9"), (130, 128, 128, "random:0.8"), (200, 32, 128, "outer:0.9"),
    (259, 128, 64, "random:0.95"),
]


@pytest.mark.parametrize("incoming", [False, True])
@pytest.mark.parametrize("n,c_z,c,mask", SHAPES)
def test_ragged_shapes(incoming, n, c_z, c, mask):
    spec = I.TriMulSpec(f"t_tm_{n}_{c_z}_{c}_{int(incoming)}_{mask}", "bf16", n, c_z, c, incoming, mask)
    case = I.make_trimul_case(spec)
    check(to_np(run(case)), oracle(case), spec.name)


@pytest.mark.parametrize("incoming", [False, True])
def test_residual_form_and_in_place(incoming):
    spec = I.TriMulSpec(f"t_tm_res_{int(incoming)}", "bf16", 150, 128, 128, incoming, "random:0.9")
    case = I.make_trimul_case(spec)
    upd = run(case, residual=True)
    check(to_np(upd), oracle(case, residual=True), spec.name, residual=True)
    assert torch.equal(run(case, residual=True, in_place=True), upd)


def test_incoming_equals_outgoing_on_the_transpose_with_sides_exchanged_bit_for_bit():
    """The library runs the incoming form as the outgoing kernels on the transposed view; exchanging the left
    and right weights and transposing input and mask by hand must give the same bits."""
    case = I.make_trimul_case(I.TriMulSpec("t_tm_transpose", "bf16", 96, 128, 128, True, "random:0.85"))
    desc, w, z, mask = P.trimul_to_device(case, DEV)
    inc = P.ff_triangle_multiplication(desc, w, z, mask)
    ws = dict(w)
    for kind in ("w", "b"):
        for s in ("p", "g"):
            ws[f"{kind}_a{s}"], ws[f"{kind}_b{s}"] = w[f"{kind}_b{s}"], w[f"{kind}_a{s}"]
    d_out = P.TriMulDesc(desc.dtype, 0, desc.n, desc.c_z, desc.c, desc.ln_eps)
    out_t = P.ff_triangle_multiplication(d_out, ws, z.transpose(0, 1).contiguous(), mask.t().contiguous())
    torch.cuda.synchronize()
    assert torch.equal(inc.transpose(0, 1), out_t)


def test_everything_masked_gives_gated_offset():
    case = I.make_trimul_case(I.TriMulSpec("t_tm_allmasked", "bf16", 40, 64, 64, False, "none"))
    case.mask = np.zeros((40, 40), np.float32)
    check(to_np(run(case)), oracle(case), "all pairs masked")


def test_long_sequence_1024_residues():
    """N_res = 1024 without a mask: the GPU computes everything, the oracle the full module (its einsum is
    1024^3 x 128 products); compared on every element."""
    spec = I.TriMulSpec("t_tm_1024", "bf16", 1024, 128, 128, False, "none", stream="tm_out_bf16_2048")
    case = I.make_trimul_case(spec)
    got = to_np(run(case))
    check(got, oracle(case), "1024 residues")


@pytest.mark.timeout(900)
def test_long_sequence_2048_residues_sampled_rows():
    """The long-sequence inference length (Section 6.2), the shape bench.py times, in the same launch configuration
    (256 x 256 product tiles): the GPU computes everything, the oracle six whole rows i of the output (rows are
    independent given a and b, which the oracle computes in full), spread over the block tiles and their edges."""
    case = I.make_trimul_case("tm_out_bf16_2048")
    rows = [0, 255, 256, 1031, 1789, 2047]
    w = {k: v.astype(np.float64) for k, v in case.widened_weights().items()}
    ref = T.triangle_multiplication(I.widen(case.z).astype(np.float64), case.mask, w, case.spec.incoming, case.spec.ln_eps,
                                    rows=rows)
    got = to_np(run(case)[rows])
    check(got, ref, "2048 residues, six rows")


def test_bad_arguments_are_status_codes():
    import ctypes as C
    from paper_2203_00854_amd import binding as B
    d = P.TriMulDesc(P.FF_F32, 0, 8, 32, 32, 1e-5)
    assert P.lib().ff_triangle_multiplication_workspace_bytes(C.byref(d)) == 0          # float32: unsupported
    d = P.TriMulDesc(P.FF_BF16, 0, 8, 48, 32, 1e-5)
    assert P.lib().ff_triangle_multiplication_workspace_bytes(C.byref(d)) == 0          # c_z not a multiple of 32
    d = P.TriMulDesc(P.FF_BF16, 0, 8, 32, 32, 1e-5)
    need = P.lib().ff_triangle_multiplication_workspace_bytes(C.byref(d))
    assert need > 0 and need % 256 == 0
    w = B.TriMulWeights()
    for n in B.TRIMUL_FIELDS:
        setattr(w, n, 0x1000)
    st = P.lib().ff_triangle_multiplication(C.byref(d), C.byref(w), 0x10000, None, 0x20000, 0, 0x100000, need - 1, None)
    assert st == B.FF_EWORKSPACE
    st = P.lib().ff_triangle_multiplication(C.byref(d), C.byref(w), 0x10000, None, 0x10000, 0, 0x100000, need, None)
    assert st == B.FF_EINVAL                                                             # out == z without residual
