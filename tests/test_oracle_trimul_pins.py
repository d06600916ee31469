"""Pins of the triangular-multiplicative-update oracle (oracle/triangle_multiplication.py) to
things other than itself: a scalar brute force, an independent composition of torch float64
library routines, closed forms and invariants.  A dropped term, a swapped index, a transposed
operand or a missing mask in the oracle fails at least one of these.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import triangle_multiplication as T
from paper_2203_00854_amd import inputs as I


def f64_case(n, c_z, c, incoming, mask="random:0.7", name=None):
    spec = I.TriMulSpec(name or f"pin_tm_{n}_{c_z}_{c}_{int(incoming)}_{mask}", "f32", n, c_z, c, incoming, mask)
    case = I.make_trimul_case(spec)
    w = {k: v.astype(np.float64) for k, v in case.widened_weights().items()}
    return I.widen(case.z).astype(np.float64), case.mask, w


def brute_force(z, mask, w, incoming, eps):
    """Scalar loops only: every sum of the definition written out element by element."""
    n, _, cz = z.shape
    c = len(w["b_ap"])

    def ln(vec, g, b):
        mu = sum(vec) / len(vec)
        var = sum((t - mu) ** 2 for t in vec) / len(vec)
        return [(t - mu) / math.sqrt(var + eps) * g[i] + b[i] for i, t in enumerate(vec)]

    def lin(vec, wm, bv, o):
        return sum(wm[o][k] * vec[k] for k in range(len(vec))) + bv[o]

    sig = lambda t: 1.0 / (1.0 + math.exp(-t))
    a = [[None] * n for _ in range(n)]
    b = [[None] * n for _ in range(n)]
    g = [[None] * n for _ in range(n)]
    for i in range(n):
        for j in range(n):
            zn = ln(list(z[i, j]), w["ln_g"], w["ln_b"])
            m = 1.0 if mask is None else float(mask[i, j])
            a[i][j] = [m * sig(lin(zn, w["w_ag"], w["b_ag"], o)) * lin(zn, w["w_ap"], w["b_ap"], o) for o in range(c)]
            b[i][j] = [m * sig(lin(zn, w["w_bg"], w["b_bg"], o)) * lin(zn, w["w_bp"], w["b_bp"], o) for o in range(c)]
            g[i][j] = [sig(lin(zn, w["w_g"], w["b_g"], o)) for o in range(cz)]
    out = np.zeros((n, n, cz))
    for i in range(n):
        for j in range(n):
            if incoming:
                t = [sum(a[k][i][ch] * b[k][j][ch] for k in range(n)) for ch in range(c)]
            else:
                t = [sum(a[i][k][ch] * b[j][k][ch] for k in range(n)) for ch in range(c)]
            tn = ln(t, w["lno_g"], w["lno_b"])
            for o in range(cz):
                out[i, j, o] = g[i][j][o] * lin(tn, w["w_o"], w["b_o"], o)
    return out


@pytest.mark.parametrize("incoming", [False, True])
@pytest.mark.parametrize("n,c_z,c,mask", [(4, 6, 5, "random:0.7"), (5, 4, 8, "none"), (3, 8, 4, "outer:0.7")])
def test_against_scalar_brute_force(incoming, n, c_z, c, mask):
    z, m, w = f64_case(n, c_z, c, incoming, mask)
    ref = brute_force(z, m, w, incoming, 1e-5)
    got = T.triangle_multiplication(z, m, w, incoming, 1e-5)
    assert np.max(np.abs(got - ref)) < 1e-12


@pytest.mark.parametrize("incoming", [False, True])
def test_against_torch_float64_composition(incoming):
    """The same module composed from torch's float64 library routines (layer_norm, linear, sigmoid,
    einsum with its own subscript convention)."""
    z, m, w = f64_case(9, 16, 12, incoming, "random:0.8")
    F = torch.nn.functional
    t = {k: torch.from_numpy(np.ascontiguousarray(v)) for k, v in w.items()}
    zt = torch.from_numpy(z)
    zn = F.layer_norm(zt, (16,), t["ln_g"], t["ln_b"], 1e-5)
    mk = torch.from_numpy(m.astype(np.float64))[..., None]
    a = mk * torch.sigmoid(F.linear(zn, t["w_ag"], t["b_ag"])) * F.linear(zn, t["w_ap"], t["b_ap"])
    b = mk * torch.sigmoid(F.linear(zn, t["w_bg"], t["b_bg"])) * F.linear(zn, t["w_bp"], t["b_bp"])
    if incoming:
        x = torch.einsum("c k i, c k j -> i j c", a.permute(2, 0, 1), b.permute(2, 0, 1))
    else:
        x = torch.matmul(a.permute(2, 0, 1), b.permute(2, 1, 0)).permute(1, 2, 0)
    ref = torch.sigmoid(F.linear(zn, t["w_g"], t["b_g"])) * F.linear(F.layer_norm(x, (12,), t["lno_g"], t["lno_b"], 1e-5),
                                                                    t["w_o"], t["b_o"])
    got = T.triangle_multiplication(z, m, w, incoming, 1e-5)
    assert np.max(np.abs(got - ref.numpy())) < 1e-11


def open_gates(w, c, c_z):
    """Gates forced to 1 (sigmoid(40) = 1 to float64 precision)."""
    w = dict(w)
    for side in ("a", "b"):
        w[f"w_{side}g"] = np.zeros_like(w[f"w_{side}g"])
        w[f"b_{side}g"] = np.full(c, 40.0)
    w["w_g"] = np.zeros_like(w["w_g"])
    w["b_g"] = np.full(c_z, 40.0)
    return w


@pytest.mark.parametrize("incoming", [False, True])
def test_closed_form_gram_matrix(incoming):
    """Gates open, left = right = identity projection of the normalised input, no mask: per channel the
    sum over k is the Gram matrix Z_c Z_c^T (outgoing) or Z_c^T Z_c (incoming) of that channel's N x N slice."""
    n, ch = 7, 6
    z, _, w = f64_case(n, ch, ch, incoming, "none")
    w = open_gates(w, ch, ch)
    for side in ("a", "b"):
        w[f"w_{side}p"] = np.eye(ch)
        w[f"b_{side}p"] = np.zeros(ch)
    w["ln_g"], w["ln_b"] = np.ones(ch), np.zeros(ch)
    w["lno_g"], w["lno_b"] = np.ones(ch), np.zeros(ch)
    w["w_o"], w["b_o"] = np.eye(ch), np.zeros(ch)
    mu = z.mean(-1, keepdims=True)
    zn = (z - mu) / np.sqrt(z.var(-1, keepdims=True) + 1e-5)
    t = np.stack([(zn[:, :, k].T @ zn[:, :, k]) if incoming else (zn[:, :, k] @ zn[:, :, k].T) for k in range(ch)], axis=-1)
    ref = (t - t.mean(-1, keepdims=True)) / np.sqrt(t.var(-1, keepdims=True) + 1e-5)
    got = T.triangle_multiplication(z, None, w, incoming, 1e-5)
    assert np.max(np.abs(got - ref)) < 1e-10
    # the two forms differ (the Gram matrix of the rows is not that of the columns)
    other = T.triangle_multiplication(z, None, w, not incoming, 1e-5)
    assert np.max(np.abs(other - got)) > 1e-2


def test_closed_form_constant_projections_count_unmasked_pairs():
    """Left projection = constant alpha, right = constant beta, gates open: t[i,j,:] = alpha*beta times the
    number of k with mask[i,k] mask[j,k] = 1 (outgoing) or mask[k,i] mask[k,j] = 1 (incoming)."""
    n, cz, c = 6, 5, 4
    z, m, w = f64_case(n, cz, c, False, "random:0.6")
    w = open_gates(w, c, cz)
    alpha, beta = np.array([0.5, -1.0, 2.0, 0.25]), np.array([1.5, 0.5, -0.75, 3.0])
    for side, val in (("a", alpha), ("b", beta)):
        w[f"w_{side}p"] = np.zeros((c, cz))
        w[f"b_{side}p"] = val
    m64 = m.astype(np.float64)
    for incoming, cnt in ((False, m64 @ m64.T), (True, m64.T @ m64)):
        t = cnt[:, :, None] * (alpha * beta)
        tn = (t - t.mean(-1, keepdims=True)) / np.sqrt(t.var(-1, keepdims=True) + 1e-5) * w["lno_g"] + w["lno_b"]
        ref = tn @ w["w_o"].T + w["b_o"]
        got = T.triangle_multiplication(z, m, w, incoming, 1e-5)
        assert np.max(np.abs(got - ref)) < 1e-10
    assert np.abs(m64 @ m64.T - m64.T @ m64).max() > 0        # the mask tells the two forms apart


def test_incoming_is_outgoing_on_the_transposed_pair_rep_with_sides_swapped():
    """incoming(z, mask)[j, i] = outgoing(z^T, mask^T)[i, j] with the left and right weights exchanged:
    t_in[j,i] = sum_k a[k,j] b[k,i], and on the transposed input a'[p,q] = a[q,p]."""
    z, m, w = f64_case(8, 12, 10, True, "random:0.8")
    ws = dict(w)
    for kind in ("w", "b"):
        for s in ("p", "g"):
            ws[f"{kind}_a{s}"], ws[f"{kind}_b{s}"] = w[f"{kind}_b{s}"], w[f"{kind}_a{s}"]
    inc = T.triangle_multiplication(z, m, w, True)
    out_t = T.triangle_multiplication(z.transpose(1, 0, 2), m.T, ws, False)
    assert np.max(np.abs(inc.transpose(1, 0, 2) - out_t)) < 1e-12
    # without the exchange it is a different function
    plain = T.triangle_multiplication(z.transpose(1, 0, 2), m.T, w, False)
    assert np.max(np.abs(inc.transpose(1, 0, 2) - plain)) > 1e-3


@pytest.mark.parametrize("incoming", [False, True])
def test_masked_pair_contributes_to_no_sum(incoming):
    """Changing z at a masked pair (p, q) changes the output at (p, q) only (through its own gate and
    normalisation input), nowhere else."""
    z, m, w = f64_case(7, 8, 6, incoming, "random:0.7")
    p, q = [tuple(ix) for ix in np.argwhere(m == 0)][0]
    z2 = z.copy()
    z2[p, q, 0] += 3.0      # (one channel: a shift of all channels is removed by the LayerNorm)
    a = T.triangle_multiplication(z, m, w, incoming)
    b = T.triangle_multiplication(z2, m, w, incoming)
    diff = np.abs(a - b).max(-1)
    diff[p, q] = 0.0
    assert diff.max() == 0.0
    # and an unmasked pair does reach other positions
    p2, q2 = [tuple(ix) for ix in np.argwhere(m == 1)][0]
    z3 = z.copy()
    z3[p2, q2, 0] += 3.0
    d3 = np.abs(a - T.triangle_multiplication(z3, m, w, incoming)).max(-1)
    d3[p2, q2] = 0.0
    assert d3.max() > 1e-3


def test_everything_masked_gives_gated_offset():
    """a = b = 0 everywhere: t = 0, LayerNorm_out(0) = its offset, out = g * (lno_b W_o^T + b_o)."""
    z, _, w = f64_case(5, 6, 4, False, "none")
    got = T.triangle_multiplication(z, np.zeros((5, 5), np.float32), w, False)
    _, _, g = T.projections(z, None, w, 1e-5)
    assert np.max(np.abs(got - g * (w["lno_b"] @ w["w_o"].T + w["b_o"]))) < 1e-12


@pytest.mark.parametrize("incoming", [False, True])
def test_residue_permutation_equivariance(incoming):
    z, m, w = f64_case(6, 8, 8, incoming, "random:0.8")
    perm = np.array([2, 0, 5, 1, 4, 3])
    a = T.triangle_multiplication(z, m, w, incoming)
    b = T.triangle_multiplication(z[perm][:, perm], m[perm][:, perm], w, incoming)
    assert np.max(np.abs(a[perm][:, perm] - b)) < 1e-12


def test_residual_form_adds_the_input():
    z, m, w = f64_case(5, 6, 4, True, "random:0.8")
    assert np.array_equal(T.triangle_multiplication(z, m, w, True, residual=True),
                          z + T.triangle_multiplication(z, m, w, True))


def test_layer_norm_and_sigmoid_against_library():
    x = np.random.default_rng(1).normal(size=(5, 7))
    g, b = np.linspace(0.5, 1.5, 7), np.linspace(-1, 1, 7)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (7,), torch.from_numpy(g), torch.from_numpy(b), 1e-3)
    assert np.max(np.abs(T.layer_norm(x, g, b, 1e-3) - ref.numpy())) < 1e-13
    t = np.linspace(-30, 30, 13)
    assert np.max(np.abs(T.sigmoid(t) - torch.sigmoid(torch.from_numpy(t)).numpy())) < 1e-15


@pytest.mark.parametrize("incoming", [False, True])
def test_rows_option_against_scalar_brute_force(incoming):
    """rows= (only some rows i of the output, what the full-size GPU comparison uses) against the scalar loops, which
    know nothing of it; with and without the residual, and with the mask."""
    z, mask, w = f64_case(6, 32, 32, incoming, "random:0.7", name=f"pin_tm_rows_{int(incoming)}")
    ref = brute_force(z, mask, w, incoming, 1e-5)
    rows = [4, 0, 5]
    np.testing.assert_allclose(T.triangle_multiplication(z, mask, w, incoming, 1e-5, rows=rows), ref[rows], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(T.triangle_multiplication(z, mask, w, incoming, 1e-5, residual=True, rows=rows),
                               (z + ref)[rows], rtol=1e-11, atol=1e-12)
