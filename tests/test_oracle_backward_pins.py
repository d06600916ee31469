"""Pins of the attention-core backward oracle (oracle/attention_core_backward.py): its forward against the
pinned module oracle, its gradients against central finite differences of that forward and against torch
float64 autograd of an independent composition.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import attention_core_backward as B
from oracle import evoformer_attention as A


def small(R=2, H=2, L=5, d=3, seed=0, masked=True, bias=True):
    rng = np.random.default_rng(seed)
    q, k, v, do = (rng.normal(size=(R, H, L, d)) for _ in range(4))
    g = 1.0 / (1.0 + np.exp(-rng.normal(size=(R, H, L, d))))
    b = rng.normal(size=(H, L, L)) if bias else None
    m = None
    if masked:
        m = (rng.random((R, L)) < 0.7).astype(np.float32)
        m[0, 0] = 1.0
    return q, k, v, g, b, m, do


def test_forward_core_matches_the_module_oracle():
    """The forward written for this oracle against a scalar re-evaluation of the definition, and its
    probabilities against the masked softmax of the (separately pinned) module oracle."""
    R, H, L, d = 3, 2, 6, 4
    q, k, v, g, b, m, _ = small(R, H, L, d, seed=3)
    o = B.attention_core(q, k, v, g, b, m)
    # scalar re-evaluation of the definition, element by element
    for r in range(R):
        for h in range(H):
            for i in range(L):
                valid = [j for j in range(L) if m[r, j] != 0]
                s = [q[r, h, i] @ k[r, h, j] / np.sqrt(d) + b[h, i, j] for j in valid]
                w = np.exp(np.array(s) - max(s)) if valid else np.zeros(0)
                ctx = sum(wj / w.sum() * v[r, h, j] for wj, j in zip(w, valid)) if valid else np.zeros(d)
                assert np.max(np.abs(o[r, h, i] - g[r, h, i] * ctx)) < 1e-12
    # and the masked softmax of the pinned module oracle gives the same probabilities
    p = B._probabilities(q, k, b, m, 1 / np.sqrt(d))
    for r in range(R):
        s = np.einsum("hid,hjd->hij", q[r], k[r]) / np.sqrt(d) + b
        assert np.max(np.abs(A.masked_softmax(s, m[r] != 0) - p[r])) < 1e-14


@pytest.mark.parametrize("masked,bias", [(True, True), (False, True), (True, False)])
def test_gradients_against_central_finite_differences(masked, bias):
    q, k, v, g, b, m, do = small(masked=masked, bias=bias, seed=1)
    grads = B.attention_core_backward(q, k, v, g, b, m, do)
    loss = lambda q_, k_, v_, g_, b_: float((B.attention_core(q_, k_, v_, g_, b_, m) * do).sum())
    args = [q, k, v, g, b]
    eps = 1e-6
    rng = np.random.default_rng(5)
    for n, (arr, grad) in enumerate(zip(args, grads)):
        if arr is None:
            assert grad is None
            continue
        for _ in range(25):                       # 25 random coordinates of every operand
            ix = tuple(rng.integers(0, s) for s in arr.shape)
            hi = [a if a is None else a.copy() for a in args]
            lo = [a if a is None else a.copy() for a in args]
            hi[n][ix] += eps
            lo[n][ix] -= eps
            fd = (loss(*hi) - loss(*lo)) / (2 * eps)
            assert abs(fd - grad[ix]) < 1e-7 * max(1.0, abs(fd)), (n, ix, fd, grad[ix])


def test_gradients_against_torch_autograd():
    q, k, v, g, b, m, do = small(R=3, H=2, L=7, d=4, seed=2)
    t = [torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v, g, b)]
    s = torch.matmul(t[0], t[1].transpose(-1, -2)) * (4 ** -0.5) + t[4][None]
    s = s + torch.where(torch.from_numpy(m)[:, None, None, :] > 0, 0.0, -torch.inf)
    o = t[3] * torch.matmul(torch.softmax(s, dim=-1), t[2])
    (o * torch.from_numpy(do)).sum().backward()
    for mine, ref in zip(B.attention_core_backward(q, k, v, g, b, m, do), t):
        assert np.max(np.abs(mine - ref.grad.numpy())) < 1e-12


def test_fully_masked_row_has_zero_gradients_and_masked_keys_get_none():
    q, k, v, g, b, m, do = small(R=2, H=2, L=5, d=3, seed=4)
    m[1, :] = 0.0
    m[0, :] = [1, 1, 0, 1, 0]
    dq, dk, dv, dg, db = B.attention_core_backward(q, k, v, g, b, m, do)
    for t in (dq, dk, dv, dg):
        assert np.all(t[1] == 0.0)
    assert np.all(dk[0][:, [2, 4]] == 0.0) and np.all(dv[0][:, [2, 4]] == 0.0)
    assert np.all(db[:, :, [2, 4]] == 0.0)              # only row 0 contributes, and it masks keys 2 and 4
    # softmax gradients sum to zero over the keys
    assert np.max(np.abs(db.sum(axis=-1))) < 1e-12
