"""Pins of the global-column-attention oracle (oracle/global_column_attention.py) to things other than
itself: scalar brute force, a torch float64 composition, the already pinned plain column attention oracle in
the case where the two coincide, closed forms and invariants.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import evoformer_attention as A
from oracle import global_column_attention as G
from paper_2203_00854_amd import inputs as I


def f64_case(n_seq, n_res, c, heads, d, mask="random:0.7", name=None):
    spec = I.GlobalSpec(name or f"pin_gca_{n_seq}_{n_res}_{c}_{heads}_{d}_{mask}", "f32", n_seq, n_res, c, heads, d, mask)
    case = I.make_global_case(spec)
    w = {k: v.astype(np.float64) for k, v in case.widened_weights().items()}
    return I.widen(case.m).astype(np.float64), case.mask, w


def brute_force(m, mask, w, heads, eps):
    n_seq, n_res, c = m.shape
    d = w["w_k"].shape[0]
    out = np.zeros((n_seq, n_res, c))
    for i in range(n_res):
        xs = []
        for s in range(n_seq):
            vec = list(m[s, i])
            mu = sum(vec) / c
            var = sum((t - mu) ** 2 for t in vec) / c
            xs.append([(t - mu) / math.sqrt(var + eps) * w["ln_g"][k] + w["ln_b"][k] for k, t in enumerate(vec)])
        valid = [s for s in range(n_seq) if mask is None or mask[s, i] != 0]
        o = [[0.0] * d for _ in range(heads)]
        if valid:
            qbar = [sum(xs[s][k] for s in valid) / len(valid) for k in range(c)]
            for h in range(heads):
                q = [sum(w["w_q"][h * d + e][k] * qbar[k] for k in range(c)) / math.sqrt(d) for e in range(d)]
                logit = {s: sum(q[e] * sum(w["w_k"][e][k] * xs[s][k] for k in range(c)) for e in range(d)) for s in valid}
                mx = max(logit.values())
                den = sum(math.exp(logit[s] - mx) for s in valid)
                for e in range(d):
                    o[h][e] = sum(math.exp(logit[s] - mx) / den * sum(w["w_v"][e][k] * xs[s][k] for k in range(c)) for s in valid)
        for s in range(n_seq):
            gated = []
            for h in range(heads):
                for e in range(d):
                    t = sum(w["w_g"][h * d + e][k] * xs[s][k] for k in range(c)) + w["b_g"][h * d + e]
                    gated.append(o[h][e] / (1.0 + math.exp(-t)))
            for co in range(c):
                out[s, i, co] = sum(w["w_o"][co][f] * gated[f] for f in range(heads * d)) + w["b_o"][co]
    return out


@pytest.mark.parametrize("n_seq,n_res,c,heads,d,mask", [(5, 3, 6, 2, 3, "random:0.7"), (4, 2, 8, 3, 2, "none"),
                                                         (6, 2, 4, 1, 4, "tail:2")])
def test_against_scalar_brute_force(n_seq, n_res, c, heads, d, mask):
    m, mk, w = f64_case(n_seq, n_res, c, heads, d, mask)
    assert np.max(np.abs(G.global_column_attention(m, mk, w, heads) - brute_force(m, mk, w, heads, 1e-5))) < 1e-12


def test_against_torch_float64_composition():
    n_seq, n_res, c, heads, d = 9, 4, 16, 4, 4
    m, mk, w = f64_case(n_seq, n_res, c, heads, d, "random:0.8")
    F = torch.nn.functional
    t = {k: torch.from_numpy(np.ascontiguousarray(v)) for k, v in w.items()}
    x = F.layer_norm(torch.from_numpy(m), (c,), t["ln_g"], t["ln_b"], 1e-5)                 # [s, i, c]
    mt = torch.from_numpy(mk.astype(np.float64))
    qbar = (x * mt[..., None]).sum(0) / mt.sum(0)[:, None]                                   # [i, c]
    q = F.linear(qbar, t["w_q"]).view(n_res, heads, d) * d ** -0.5
    k = F.linear(x, t["w_k"])                                                                # [s, i, d]
    v = F.linear(x, t["w_v"])
    logits = torch.einsum("ihe,sie->ihs", q, k) + torch.where(mt.t() > 0, 0.0, -torch.inf)[:, None, :]
    p = torch.softmax(logits, dim=-1)
    o = torch.einsum("ihs,sie->ihe", p, v).reshape(n_res, heads * d)
    g = torch.sigmoid(F.linear(x, t["w_g"], t["b_g"]))
    ref = F.linear(g * o[None], t["w_o"], t["b_o"])
    assert np.max(np.abs(G.global_column_attention(m, mk, w, heads) - ref.numpy())) < 1e-12


def test_equal_sequences_reduce_to_the_plain_column_attention():
    """If all sequences of a column are equal, every sequence's own query equals the averaged one, so the plain
    gated column attention (already pinned) with the single key / value head repeated for every head gives
    the same result."""
    n_seq, n_res, c, heads, d = 6, 3, 8, 2, 4
    m, _, w = f64_case(n_seq, n_res, c, heads, d, "none")
    m = np.repeat(m[:1], n_seq, axis=0)
    mask = np.ones((n_seq, n_res), np.float32)
    mask[4:, 1] = 0.0
    plain = dict(w, w_k=np.tile(w["w_k"], (heads, 1)), w_v=np.tile(w["w_v"], (heads, 1)))
    ref = A.gated_attention(A.MODE_COL, m, None, mask, plain, heads, 1e-5)
    assert np.max(np.abs(G.global_column_attention(m, mask, w, heads) - ref)) < 1e-12


def test_different_sequences_differ_from_the_plain_column_attention():
    n_seq, n_res, c, heads, d = 6, 3, 8, 2, 4
    m, mk, w = f64_case(n_seq, n_res, c, heads, d, "none")
    plain = dict(w, w_k=np.tile(w["w_k"], (heads, 1)), w_v=np.tile(w["w_v"], (heads, 1)))
    ref = A.gated_attention(A.MODE_COL, m, None, None, plain, heads, 1e-5)
    assert np.max(np.abs(G.global_column_attention(m, None, w, heads) - ref)) > 1e-3


def test_zero_query_weights_give_the_mean_value_of_unmasked_sequences():
    n_seq, n_res, c, heads, d = 7, 3, 8, 2, 4
    m, mk, w = f64_case(n_seq, n_res, c, heads, d, "random:0.7")
    w = dict(w, w_q=np.zeros_like(w["w_q"]), w_g=np.zeros_like(w["w_g"]), b_g=np.full(heads * d, 40.0))
    x = G.layer_norm(m, w["ln_g"], w["ln_b"], 1e-5)
    v = x @ w["w_v"].T
    ref = np.empty_like(m)
    for i in range(n_res):
        ok = mk[:, i] != 0
        o = v[ok, i].mean(axis=0) if ok.any() else np.zeros(d)
        ref[:, i] = np.tile(o, heads) @ w["w_o"].T + w["b_o"]
    assert np.max(np.abs(G.global_column_attention(m, mk, w, heads) - ref)) < 1e-12


def test_masked_sequences_do_not_matter_and_empty_columns_give_the_output_bias():
    n_seq, n_res, c, heads, d = 8, 4, 8, 2, 4
    m, _, w = f64_case(n_seq, n_res, c, heads, d, "none")
    mask = np.ones((n_seq, n_res), np.float32)
    mask[5:, :] = 0.0
    mask[:, 2] = 0.0
    a = G.global_column_attention(m, mask, w, heads)
    m2 = m.copy()
    m2[5:] = m2[5:] * 3.0 + 1.0
    b = G.global_column_attention(m2, mask, w, heads)
    assert np.max(np.abs(a[:5] - b[:5])) == 0.0                  # unmasked sequences see no change
    assert np.max(np.abs(a[:, 2] - w["b_o"])) == 0.0             # no unmasked sequence in column 2
    # the query average uses the unmasked sequences only: a masked sequence with a huge value would show otherwise
    m3 = m.copy()
    m3[6, 0, 0] += 50.0
    assert np.max(np.abs(G.global_column_attention(m3, mask, w, heads)[:5] - a[:5])) == 0.0


def test_sequence_permutation_equivariance_and_column_independence():
    n_seq, n_res, c, heads, d = 6, 3, 8, 2, 4
    m, mk, w = f64_case(n_seq, n_res, c, heads, d, "random:0.8")
    perm = np.array([3, 0, 5, 1, 4, 2])
    a = G.global_column_attention(m, mk, w, heads)
    b = G.global_column_attention(m[perm], mk[perm], w, heads)
    assert np.max(np.abs(a[perm] - b)) < 1e-12
    only = G.global_column_attention(m, mk, w, heads, cols=[2, 0])
    assert np.array_equal(only, a[:, [2, 0]])
