"""The C-ABI library loads, exports what include/ff.h declares, and rejects bad arguments
with status codes before anything reaches the GPU.  No compute calls here."""
import ctypes as C
import os
import re

import pytest

import paper_2203_00854_amd as P
from paper_2203_00854_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "ff.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ff_[a-z_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = header_functions()
    for n in ("ff_layernorm", "ff_gated_attention", "ff_attention_chunked", "ff_gated_attention_residual",
              "ff_attention_workspace_bytes", "ff_last_error"):
        assert n in names


def test_library_exports_every_declared_symbol():
    lib = P.lib()
    for n in header_functions():
        assert hasattr(lib, n), n


def test_struct_layout_matches_header():
    assert C.sizeof(B.AttnDesc) == 9 * 4
    assert C.sizeof(B.AttnWeights) == 12 * C.sizeof(C.c_void_p)


def good_desc(**kw):
    d = dict(mode=P.FF_MSA_ROW, dtype=P.FF_BF16, n_a=8, n_b=32, c=32, c_z=16, heads=4, head_dim=8, ln_eps=1e-5)
    d.update(kw)
    return P.AttnDesc(**d)


def test_workspace_size_is_positive_and_grows_with_chunk():
    d = good_desc()
    full = P.ff_attention_workspace_bytes(d, 0)
    one = P.ff_attention_workspace_bytes(d, 1)
    assert 0 < one < full
    assert P.ff_attention_workspace_bytes(d, 10 ** 6) == full
    assert full % 256 == 0


def test_workspace_never_holds_the_score_tensor():
    """Section 3.2: the score tensor N_r^3 * N_head * 2 bytes is the memory problem.  The
    workspace for N_res=2048, H=4 chunked by 64 rows must be far below 4*2048^3*2 = 68.7 GB
    and even below one chunk of scores (64*4*2048^2*2 = 2.1 GB)."""
    d = good_desc(mode=P.FF_TRI_START, n_a=2048, n_b=2048, c=128, c_z=0, heads=4, head_dim=32)
    ws = P.ff_attention_workspace_bytes(d, 64)
    assert ws < 64 * 4 * 2048 ** 2 * 2
    assert ws < 1 << 30


@pytest.mark.parametrize("kw,status", [
    (dict(mode=9), B.FF_EINVAL), (dict(dtype=5), B.FF_EINVAL), (dict(n_a=0), B.FF_EINVAL),
    (dict(heads=-1), B.FF_EINVAL), (dict(c_z=0), B.FF_EINVAL), (dict(head_dim=256), B.FF_EUNSUPPORTED),
    (dict(mode=P.FF_TRI_START, n_a=5, n_b=6), B.FF_EINVAL), (dict(c=10000), B.FF_EUNSUPPORTED),
])
def test_bad_descriptors(kw, status):
    d = good_desc(**kw)
    assert P.lib().ff_attention_workspace_bytes(C.byref(d), 0) == 0
    assert P.last_error() != ""
    w = B.AttnWeights()
    st = P.lib().ff_gated_attention(C.byref(d), C.byref(w), 0x1000, 0x2000, None, 0x3000, 0x100000, 1 << 40, None)
    assert st == status


def _fake_weights(row=True):
    w = B.AttnWeights()
    for i, n in enumerate(B.WEIGHT_FIELDS):
        setattr(w, n, 0x10000 * (i + 1))
    if not row:
        w.lnz_g = None
        w.lnz_b = None
    return w


def test_argument_errors_before_any_launch():
    lib = P.lib()
    d = good_desc()
    w = _fake_weights()
    need = P.ff_attention_workspace_bytes(d, 0)
    X, Z, OUT, WS = 0x100000, 0x200000, 0x300000, 0x400000
    call = lambda *a: lib.ff_gated_attention(C.byref(d), *a)
    assert call(C.byref(w), None, Z, None, OUT, WS, need, None) == B.FF_EINVAL          # x NULL
    assert call(C.byref(w), X, None, None, OUT, WS, need, None) == B.FF_EINVAL          # z missing in row mode
    assert call(C.byref(w), X, Z, None, X, WS, need, None) == B.FF_EINVAL               # out aliases x
    assert call(C.byref(w), X, Z, None, OUT, None, need, None) == B.FF_EINVAL           # no workspace
    assert call(C.byref(w), X, Z, None, OUT, WS + 8, need, None) == B.FF_EINVAL         # misaligned workspace
    assert call(C.byref(w), X, Z, None, OUT, WS, need - 1, None) == B.FF_EWORKSPACE
    assert "workspace too small" in P.last_error()
    assert call(None, X, Z, None, OUT, WS, need, None) == B.FF_EINVAL                   # weights NULL
    w2 = _fake_weights()
    w2.w_b = None
    assert call(C.byref(w2), X, Z, None, OUT, WS, need, None) == B.FF_EINVAL
    dc = good_desc(mode=P.FF_MSA_COL)
    wc = _fake_weights(row=False)
    assert lib.ff_gated_attention(C.byref(dc), C.byref(wc), X, Z, None, OUT, WS, 1 << 40, None) == B.FF_EINVAL  # z given
    assert lib.ff_attention_chunked(C.byref(d), C.byref(w), X, Z, None, OUT, WS, need, None, 0) == B.FF_EINVAL
    assert "chunk_rows" in P.last_error()
    # the residual update: out may be x itself, but not a shifted view of it, and never z
    upd = lambda *a: lib.ff_gated_attention_residual(C.byref(d), C.byref(w), *a)
    assert upd(X, Z, None, X + 64, WS, need, None, 0) == B.FF_EINVAL
    assert "x itself" in P.last_error()
    assert upd(X, Z, None, Z, WS, need, None, 0) == B.FF_EINVAL
    assert upd(X, Z, None, X, WS, need, None, -1) == B.FF_EINVAL
    assert upd(X, Z, None, X, WS, need - 1, None, 0) == B.FF_EWORKSPACE     # in place passes the overlap check


def test_layernorm_argument_errors():
    lib = P.lib()
    assert lib.ff_layernorm(0x1000, 0x2000, 0x3000, 0x4000, 4, 0, 1e-5, 0, None) == B.FF_EINVAL
    assert lib.ff_layernorm(0x1000, 0x2000, 0x3000, 0x4000, -1, 8, 1e-5, 0, None) == B.FF_EINVAL
    assert lib.ff_layernorm(0x1000, 0x2000, 0x3000, 0x4000, 4, 8, 1e-5, 3, None) == B.FF_EINVAL
    assert lib.ff_layernorm(None, 0x2000, 0x3000, 0x4000, 4, 8, 1e-5, 0, None) == B.FF_EINVAL
    assert lib.ff_layernorm(None, None, None, None, 0, 8, 1e-5, 0, None) == B.FF_OK     # empty input: nothing to do


def test_path_selection_reports_a_family():
    assert P.ff_attention_path(good_desc(dtype=P.FF_F32)) == "generic"
    assert P.ff_attention_path(good_desc(n_a=128, n_b=256, c=256, c_z=128, heads=8, head_dim=32)) in ("mfma_bf16", "generic")


def test_workspace_never_holds_the_score_tensor_of_section_3_2():
    """Section 3.2 of the paper: the attention score tensor of a triangle module takes
    N_r^3 * N_head * 2 bytes, more than 20 GB over 48 layers at N_r = 384 (the fixture holds the
    paper's figures).  The formula reproduces the stated bound, and the workspace this library
    asks for at that shape stays three orders of magnitude below one layer's score tensor."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "attention_activation_memory.txt")
    row = [l.split() for l in open(path) if l.strip() and not l.startswith("#")][0]
    n_r, heads, esz, layers, stated = (int(v) for v in row)
    per_layer = n_r ** 3 * heads * esz
    assert per_layer * layers > stated
    assert per_layer * layers < 1.2 * stated            # "can exceed 20 GB": 21.7 GB
    desc = good_desc(mode=P.FF_TRI_START, n_a=n_r, n_b=n_r, c=128, c_z=0, heads=heads, head_dim=32)
    need = P.ff_attention_workspace_bytes(desc, 64)
    assert need * 8 < per_layer
    # chunking bounds it: the whole-module workspace grows with the rows, the chunked one does not
    assert P.ff_attention_workspace_bytes(desc, 0) > need


# ---- the entry points added after the attention module: layouts, workspace sizes, argument errors (no launches)
def test_struct_layouts_of_the_widened_modules():
    assert C.sizeof(B.TriMulDesc) == 6 * 4
    assert C.sizeof(B.TriMulWeights) == len(B.TRIMUL_FIELDS) * C.sizeof(C.c_void_p)
    assert C.sizeof(B.GlobalDesc) == 7 * 4
    assert C.sizeof(B.GlobalWeights) == len(B.GLOBAL_FIELDS) * C.sizeof(C.c_void_p)
    assert C.sizeof(B.CoreDesc) == 5 * 4
    text = open(os.path.join(ROOT, "include", "ff.h")).read()
    for name, fields in (("ff_trimul_weights", B.TRIMUL_FIELDS), ("ff_global_weights", B.GLOBAL_FIELDS)):
        body = re.search(r"typedef struct\s*\{([^}]*)\}\s*" + name, text, flags=re.S).group(1)
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        declared = re.findall(r"\*\s*([a-z_0-9]+)", body)
        assert tuple(declared) == tuple(fields), name        # same members, same order


def test_workspace_sizes_of_the_widened_modules():
    lib = P.lib()
    tm = B.TriMulDesc(dtype=P.FF_BF16, incoming=0, n=256, c_z=128, c=128, ln_eps=1e-5)
    ws = lib.ff_triangle_multiplication_workspace_bytes(C.byref(tm))
    # a, b and t (three bf16 tensors of n^2 c) plus the prepared weights, and nothing of order n^3
    assert 3 * 256 * 256 * 128 * 2 <= ws < 3 * 256 * 256 * 128 * 2 + (1 << 20)
    gd = B.GlobalDesc(dtype=P.FF_BF16, n_seq=1024, n_res=384, c=64, heads=8, head_dim=8, ln_eps=1e-5)
    ws = lib.ff_global_column_attention_workspace_bytes(C.byref(gd))
    assert 1024 * 384 * 16 * 2 <= ws < 1024 * 384 * 64 * 2         # k | v per token and partial sums: below the input's size
    cd = B.CoreDesc(dtype=P.FF_BF16, rows=128, heads=8, length=256, head_dim=32)
    ws = lib.ff_attention_core_backward_workspace_bytes(C.byref(cd))
    assert 0 < ws < 128 * 8 * 256 * 256 * 2                        # never a score-sized tensor
    for bad in (B.TriMulDesc(dtype=P.FF_F32, incoming=0, n=64, c_z=128, c=128, ln_eps=1e-5),
                B.TriMulDesc(dtype=P.FF_BF16, incoming=0, n=64, c_z=100, c=128, ln_eps=1e-5)):
        assert lib.ff_triangle_multiplication_workspace_bytes(C.byref(bad)) == 0
    assert lib.ff_global_column_attention_workspace_bytes(
        C.byref(B.GlobalDesc(dtype=P.FF_BF16, n_seq=64, n_res=8, c=64, heads=8, head_dim=32, ln_eps=1e-5))) == 0
    assert lib.ff_attention_core_backward_workspace_bytes(
        C.byref(B.CoreDesc(dtype=P.FF_BF16, rows=4, heads=2, length=64, head_dim=64))) == 0


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
