"""GPU parity of the one-kernel projection + attention path (sequences of 129..256 positions, head
dimension 32, 64 / 128 / 256 channels, bfloat16) against the float64 oracle, through the C ABI.

Shapes: odd numbers of batch rows (the last block has one row only), lengths that leave
wavefronts without tokens (192 padded positions) and ragged tails inside a tile, every mode,
masks that empty whole key tiles, chunked calls (row pairs that start at a chunk's first row).
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


def check(got, ref, what=""):
    ma, rl = max_abs(got, ref), rel_l2(got, ref)
    print(f"{what}: max_abs={ma:.3e} rel_l2={rl:.3e}", flush=True)
    assert np.isfinite(got).all()
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


def oracle_case(case):
    x, z, m, w = f64_inputs(case)
    sp = case.spec
    return O.gated_attention(sp.mode, x, z, m, w, sp.heads, sp.ln_eps)


SHAPES = [
    # mode, n_a, n_b, c, H, d, c_z, mask, chunk
    (ROW, 5, 130, 64, 2, 32, 48, "tail:5", None),
    (ROW, 4, 256, 256, 8, 32, 128, "random:0.8", None),
    (ROW, 7, 200, 128, 3, 32, 16, "tail:70", None),          # the last two key tiles hold no valid key
    (ROW, 19, 255, 256, 4, 32, 32, "random:0.5", 6),          # chunks of six rows, the last of one
    (COL, 200, 3, 128, 2, 32, 0, "random:0.7", None),
    (COL, 129, 33, 64, 8, 32, 0, "none", None),
    (TS, 150, 150, 128, 4, 32, 0, "outer:0.9", 16),
    (TE, 131, 131, 64, 2, 32, 0, "random:0.8", 7),
    (TS, 256, 256, 128, 4, 32, 0, "tail:3", 64),
]


@pytest.mark.parametrize("mode,n_a,n_b,c,H,d,c_z,mask,chunk", SHAPES)
def test_fused_projection_attention_shapes(mode, n_a, n_b, c, H, d, c_z, mask, chunk):
    case = I.make_case(small_spec(mode, n_a, n_b, c, H, d, c_z=c_z, dtype="bf16", mask=mask))
    got = to_np(run_case(case, chunk_rows=chunk))
    assert P.ff_attention_last_path() == "mfma_bf16"
    check(got, oracle_case(case), case.spec.name)


def test_fused_chunked_is_bit_identical_to_unchunked():
    """Section 5.3: batch rows are independent, so any chunking reproduces the same bits (here
    chunks with an odd number of rows: a row is the first of its pair in one call and the second
    in the other)."""
    case = I.make_case(small_spec(ROW, 11, 190, 128, 4, 32, c_z=16, dtype="bf16", mask="random:0.8"))
    a = run_case(case)
    b = run_case(case, chunk_rows=3)
    assert torch.equal(a, b)


def test_fused_fully_masked_rows_give_output_bias():
    """A batch row without a valid key: every key tile is skipped, the context is zero and the module
    returns the output projection's bias for that row."""
    case = I.make_case(small_spec(COL, 200, 9, 64, 2, 32, dtype="bf16", mask="tail:3"))
    case.mask[:, 4] = 0.0
    got = to_np(run_case(case))
    bo = I.widen(case.weights["b_o"]).astype(np.float64)
    assert max_abs(got[:, 4], np.broadcast_to(bo, got[:, 4].shape)) == 0.0
    check(got, oracle_case(case), "fully masked batch row")


def test_fused_masked_key_content_is_irrelevant():
    case = I.make_case(small_spec(ROW, 4, 180, 128, 4, 32, c_z=16, dtype="bf16", mask="tail:50"))
    desc, w, x, z, mask = P.to_device(case, DEV)
    a = P.ff_gated_attention(desc, w, x, z, mask)
    x2 = x.clone()
    x2[:, 130:, :] = torch.randn_like(x2[:, 130:, :]) * 3
    b = P.ff_gated_attention(desc, w, x2, z, mask)
    torch.cuda.synchronize()
    assert torch.equal(a[:, :130], b[:, :130])


@pytest.mark.parametrize("mode,n_a,n_b,c,H,d,c_z,chunk", [(ROW, 9, 200, 128, 4, 32, 32, 0), (TS, 140, 140, 64, 2, 32, 0, 48)])
def test_fused_calls_can_be_captured_in_a_hip_graph(mode, n_a, n_b, c, H, d, c_z, chunk):
    """The kernel keeps nothing in the workspace from call to call (the pad rows and columns of the
    tiled bias are rewritten by every call): replays over a workspace filled with random bytes
    reproduce the eager bits."""
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
        ws.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
