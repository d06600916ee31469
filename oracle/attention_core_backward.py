"""CPU oracle for the backward pass of the fused attention core (float64, numpy).

TEST INFRASTRUCTURE ONLY.  It defines what the HIP library's ff_attention_core_backward must compute; it is
imported by tests/, never by the product path, and it shares no code with the kernels.

The paper benchmarks its fused softmax (scale + mask + bias) forward AND backward (Section 6.3) and reports
forward / backward times per Evoformer layer (Table 6); training needs the gradients of the attention core
that the forward path fuses.  The core, per batch row r and head h (Sections 2.1, 5.2), with scale 1/sqrt(d)
and M(t) = 0 if t == 1 else -inf:

    S[r,h,i,j] = scale * q[r,h,i,:] . k[r,h,j,:] + bias[h,i,j] + M(mask[r,j])
    P          = softmax over j of S            (a query without unmasked keys: P = 0)
    ctx[r,h,i] = sum_j P[r,h,i,j] v[r,h,j,:]
    o          = g * ctx                        (g: the gate after its sigmoid)

Given do = dLoss/do, the chain rule gives (written out, nothing fused or tiled):

    dg   = do * ctx                 dctx = do * g
    dv[r,h,j]  = sum_i P[i,j] dctx[i]
    dP[i,j]    = dctx[i] . v[j]
    dS[i,j]    = P[i,j] * (dP[i,j] - sum_j' P[i,j'] dP[i,j'])
    dq[r,h,i]  = scale * sum_j dS[i,j] k[j]     dk[r,h,j] = scale * sum_i dS[i,j] q[i]
    dbias[h,i,j] = sum_r dS[r,h,i,j]            (the bias is shared by the batch rows)

Parity pins: tests/test_oracle_backward_pins.py (central finite differences of the forward definition, which
is written separately here and is itself checked against the pinned module oracle; torch float64 autograd).
"""
from __future__ import annotations

import numpy as np

_F = np.float64


def _probabilities(q, k, bias, mask, scale):
    """P[r,h,i,j] of the definition above; q, k [R,H,L,d], bias [H,L,L] or None, mask [R,L] or None."""
    s = scale * np.einsum("rhid,rhjd->rhij", q, k)
    if bias is not None:
        s = s + np.asarray(bias, _F)[None]
    R, H, L, _ = q.shape
    valid = np.ones((R, L), bool) if mask is None else (np.asarray(mask) != 0)
    p = np.zeros_like(s)
    for r in range(R):
        if not valid[r].any():
            continue
        sr = s[r][:, :, valid[r]]
        e = np.exp(sr - sr.max(axis=-1, keepdims=True))
        p[r][:, :, valid[r]] = e / e.sum(axis=-1, keepdims=True)
    return p


def attention_core(q, k, v, g, bias, mask):
    """Forward: o = g * softmax(scale q k^T + bias + mask) v.  All of q, k, v, g: [R, H, L, d]."""
    q, k, v, g = (np.asarray(t, _F) for t in (q, k, v, g))
    p = _probabilities(q, k, bias, mask, 1.0 / np.sqrt(q.shape[-1]))
    return g * np.einsum("rhij,rhjd->rhid", p, v)


def attention_core_backward(q, k, v, g, bias, mask, do):
    """Gradients (dq, dk, dv, dg, dbias) of sum(o * do) with respect to q, k, v, g, bias.  dbias is None if
    bias is None."""
    q, k, v, g, do = (np.asarray(t, _F) for t in (q, k, v, g, do))
    scale = 1.0 / np.sqrt(q.shape[-1])
    p = _probabilities(q, k, bias, mask, scale)
    ctx = np.einsum("rhij,rhjd->rhid", p, v)
    dg = do * ctx
    dctx = do * g
    dv = np.einsum("rhij,rhid->rhjd", p, dctx)
    dp = np.einsum("rhid,rhjd->rhij", dctx, v)
    ds = p * (dp - (p * dp).sum(axis=-1, keepdims=True))
    dq = scale * np.einsum("rhij,rhjd->rhid", ds, k)
    dk = scale * np.einsum("rhij,rhid->rhjd", ds, q)
    dbias = None if bias is None else ds.sum(axis=0)
    return dq, dk, dv, dg, dbias
