"""The entry point that allocates nothing (ff_gated_attention_static): called through the raw C
ABI, compared bit for bit with ff_gated_attention on two calls in a row, the second with a
smaller input, and once more with the larger one (the library's device array keeps whatever the
call before left in it)."""
import ctypes as C

import pytest
import torch

import paper_2203_00854_amd as P
from paper_2203_00854_amd import binding as B
from paper_2203_00854_amd import inputs as I
from helpers import small_spec

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def static_call(desc, w, x, z, mask, out):
    wts = B.make_weights(w)
    ptr = lambda t: None if t is None else t.data_ptr()
    st = P.lib().ff_gated_attention_static(C.byref(desc), C.byref(wts), ptr(x), ptr(z), ptr(mask), ptr(out),
                                           torch.cuda.current_stream().cuda_stream)
    assert st == B.FF_OK, P.last_error()


def both(spec):
    case = I.make_case(spec)
    desc, w, x, z, mask = P.to_device(case, DEV)
    ref = P.ff_gated_attention(desc, w, x, z, mask)
    out = torch.full_like(x, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    static_call(desc, w, x, z, mask, out)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return ref, out, desc


def test_static_scratch_entry_point_matches_the_workspace_one():
    assert P.ff_static_scratch_bytes() == 48 << 20
    big = I.CaseSpec("static_row", I.MODE_ROW, "bf16", 96, 256, 256, 128, 8, 32, "tail:16")      # several chunks
    small = small_spec(I.MODE_TRI_START, 45, 45, 128, 4, 32, dtype="bf16", mask="outer:0.9")
    tiny_f32 = I.SPECS["c1_row_f32_tiny"]
    for spec in (big, small, tiny_f32, big):
        ref, out, desc = both(spec)
        assert torch.equal(ref, out), spec.name
    # the big case really ran in more than one chunk
    d = P.AttnDesc(P.FF_MSA_ROW, P.FF_BF16, 96, 256, 256, 128, 8, 32, 1e-5)
    assert P.ff_attention_workspace_bytes(d, 0) > P.ff_static_scratch_bytes()


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    d = P.AttnDesc(P.FF_TRI_START, P.FF_BF16, 4096, 4096, 128, 0, 4, 32, 1e-5)     # the bias alone is 256 MiB
    w = B.AttnWeights()
    st = P.lib().ff_gated_attention_static(C.byref(d), C.byref(w), 0x1000, None, None, 0x2000, None)
    assert st == B.FF_EWORKSPACE
    assert "static scratch" in P.last_error()
