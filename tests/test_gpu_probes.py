"""The calibration probes and the launch timer of the C ABI (what bench.py's calibration calls): they run, count
what they say they count, and reject bad arguments with a status code."""
import ctypes as C

import pytest
import torch

import paper_2203_00854_amd as P
from paper_2203_00854_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_probes_run_and_are_timed_by_kind():
    sink = torch.empty(P.lib().ff_probe_sink_bytes(), dtype=torch.uint8, device=DEV)
    src = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    dst = torch.zeros_like(src)
    P.ff_profile_enable(True)
    flop = P.ff_probe_mfma(sink, 100)
    insts = [P.ff_probe_valu(sink, kind, 64) for kind in range(4)]
    rounds = [P.ff_probe_valu(sink, kind, 64) for kind in range(4, 8)]
    P.ff_probe_copy(dst, src)
    torch.cuda.synchronize()
    k = P.ff_profile_collect()
    P.ff_profile_enable(False)
    assert flop == 512 * 8 * 100 * 4 * 2.0 * 32 * 32 * 16
    assert insts == [1024 * 4 * 64 * 16.0] * 4
    assert rounds == [1024 * 4 * 64.0] * 4
    assert torch.equal(dst, src)
    assert k["probe: mfma loop"][1] == 1 and k["probe: copy"][1] == 1 and k["probe: vector loop"][1] == 8
    assert all(ms > 0.0 for ms, _ in k.values())


def test_probe_arguments():
    sink = torch.empty(P.lib().ff_probe_sink_bytes(), dtype=torch.uint8, device=DEV)
    n = C.c_double(0.0)
    ptr = C.c_void_p(sink.data_ptr())
    assert P.lib().ff_probe_valu(ptr, 8, 10, C.byref(n), None) == B.FF_EINVAL
    assert P.lib().ff_probe_valu(ptr, 0, 0, C.byref(n), None) == B.FF_EINVAL
    assert P.lib().ff_probe_valu(None, 0, 10, C.byref(n), None) == B.FF_EINVAL
    assert P.lib().ff_probe_mfma(ptr, 0, C.byref(n), None) == B.FF_EINVAL
    assert P.lib().ff_probe_copy(ptr, ptr, 24, None) == B.FF_EINVAL
