"""GPU parity at the paper's fine-tuning shapes (Table 1: N_res = 384, N_seq = 512,
N_extra_seq = 5120), bf16, all four modes, in the launch configuration bench.py times.

The library computes every batch row; the oracle evaluates a sample of them (a batch row needs
only its own tokens and the bias, Section 4.2), chosen to touch the first and last row, both
sides of every 8-row block boundary of the attention kernel and rows in the middle.
"""
import numpy as np
import pytest
import torch

import paper_2203_00854_amd as P
from paper_2203_00854_amd import inputs as I
from test_gpu_parity import check, oracle_case, run_case, to_np

pytestmark = pytest.mark.gpu

ROW, COL, TS, TE = I.MODE_ROW, I.MODE_COL, I.MODE_TRI_START, I.MODE_TRI_END


def sampled(got, mode, rows):
    return got[rows] if mode in (ROW, TS) else got[:, rows].transpose(1, 0, 2)


@pytest.mark.parametrize("name,rows", [
    ("ft_row_bf16_512x384", [0, 7, 8, 255, 256, 300, 511]),
    ("ft_col_bf16_512x384", [0, 7, 8, 191, 192, 383]),
    ("ft_tri_start_bf16_384", list(range(0, 384, 13)) + [383]),
    ("ft_tri_end_bf16_384", list(range(5, 384, 13)) + [383]),
])
def test_fine_tuning_shapes(name, rows):
    case = I.make_case(name)
    sp = case.spec
    desc = P.AttnDesc(sp.mode, P.FF_BF16, sp.n_a, sp.n_b, sp.c, sp.c_z, sp.heads, sp.head_dim, sp.ln_eps)
    assert P.ff_attention_path(desc) == "mfma_bf16"
    got = to_np(run_case(case))
    assert P.ff_attention_last_path() == "mfma_bf16"
    check(sampled(got, sp.mode, rows), oracle_case(case, rows=rows), "bf16", name)
    # chunked (a ragged last chunk) reproduces the bits
    assert torch.equal(run_case(case, chunk_rows=100), run_case(case))


def test_extra_msa_column_attention_5120_sequences():
    """160 key tiles of 32 per column, head dim 8, the last 512 sequences padding; the oracle
    materialises the 5120 x 5120 scores of each head for six columns: both sides of a boundary
    between the attention kernel's 4-row blocks, the first and last column, two in the middle at
    other positions inside their blocks."""
    case = I.make_case("ft_col_bf16_extra_5120")
    got = to_np(run_case(case))
    rows = [0, 3, 4, 190, 257, 383]
    check(sampled(got, COL, rows), oracle_case(case, rows=rows), "bf16", "extra MSA, 5120 sequences")
