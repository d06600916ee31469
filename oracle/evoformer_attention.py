"""CPU oracle for the Evoformer gated axial attention with pair bias (float64, numpy).

TEST INFRASTRUCTURE ONLY.  This file defines what the HIP library must compute; it is
imported by tests/, by the smoke check and by the benchmark's cpu_baseline leg, never by
the product path, and it shares no code with the kernels.

It is the plain definition written out: the score matrix of every (batch row, head) is
materialised, the softmax is the textbook max / subtract / exp / sum / divide
(FastFold Section 5.2, the description of the fused softmax), nothing is tiled, fused,
chunked or computed online.  Chunking and online softmax reach exactly this result up to
rounding order, so the definition itself is the reference.

What the paper fixes and where:
  * multi-head attention = Q/K/V linear layers split into heads, scaled dot product,
    softmax, product with V, concatenation, output linear layer      (Section 2.1);
  * the Evoformer applies it along rows or along columns of a representation with two
    sequence axes; the pair representation feeds the MSA row attention through an
    attention bias, and the pair stack uses "similar blocks"          (Section 2.3);
  * the softmax input is the scaled logits plus a mask term plus a bias term
                                                                       (Section 5.2);
  * the gate is bias + sigmoid + element-wise product                 (Section 5.2, JIT fusion);
  * each module ends in bias + dropout + add, the residual update of the representation
    (Section 5.2, JIT fusion; dropout is the identity outside training).
The paper prints no equations for the four modules and defers to AlphaFold 2; the index
placement below is AlphaFold's published MSA row attention with pair bias, MSA column
attention and triangle attention around the starting / ending node.

Readings where the paper is silent (all restated in the design notes):
  * LayerNorm: biased variance, eps inside the square root, per-channel gain and offset.
  * Scale 1/sqrt(head_dim) applies to q.k only, not to bias or mask.
  * mask is 0/1; a masked key gets weight exactly 0 (additive minus infinity).  A query
    whose keys are all masked gets an all-zero weight row, so its output is b_o.
  * Padded queries are still computed.
  * q, k, v and the bias projection have no additive bias; gate and output linears do.
  * Weights are [out, in]; channel h*head_dim + e belongs to head h.

Parity pins: tests/test_oracle_pins.py (scalar brute force, an independent composition
of torch float64 library routines, closed forms, invariants).  Every function here is
pinned by at least one of them.
"""
from __future__ import annotations

import numpy as np

MODE_ROW, MODE_COL, MODE_TRI_START, MODE_TRI_END = 0, 1, 2, 3

_F = np.float64


def layer_norm(v, gamma, beta, eps):
    """LayerNorm over the last axis: (v - mean) / sqrt(var + eps) * gamma + beta with
    the biased variance (Section 3.1 classes LayerNorm as a batch reduction over the
    hidden dimension)."""
    v = np.asarray(v, dtype=_F)
    mu = v.mean(axis=-1, keepdims=True)
    var = ((v - mu) ** 2).mean(axis=-1, keepdims=True)
    return (v - mu) / np.sqrt(var + eps) * np.asarray(gamma, _F) + np.asarray(beta, _F)


def sigmoid(t):
    return 1.0 / (1.0 + np.exp(-t))


def masked_softmax(logits, key_valid):
    """Softmax over the last axis restricted to keys with key_valid == True.

    Steps as in Section 5.2: row maximum, subtract, exponentiate, sum, divide.  Masked
    keys get exactly 0.  If no key is valid the whole row is 0."""
    logits = np.asarray(logits, dtype=_F)
    key_valid = np.asarray(key_valid, dtype=bool)
    p = np.zeros_like(logits)
    if not key_valid.any():
        return p
    s = logits[..., key_valid]
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    p[..., key_valid] = e / e.sum(axis=-1, keepdims=True)
    return p


def pair_bias(mode, x, z, w, eps):
    """Attention bias b[h, p, q] (Section 2.3: the attention bias carries pair
    information into the attention).

    MSA row mode: b[h,i,j] = sum_c LN_z(z[i,j,:])_c * w_b[h,c], a LayerNorm of its own.
    Triangle modes: b[h,p,q] = sum_c LN(x[p,q,:])_c * w_b[h,c] with the module's LayerNorm.
    Column mode: no bias (returns None)."""
    if mode == MODE_COL:
        return None
    wb = np.asarray(w["w_b"], _F)
    if mode == MODE_ROW:
        src, g, b = z, w["lnz_g"], w["lnz_b"]
    else:
        src, g, b = x, w["ln_g"], w["ln_b"]
    n0, n1 = src.shape[0], src.shape[1]
    out = np.empty((wb.shape[0], n0, n1), dtype=_F)
    for p in range(n0):                                   # one row of the pair rep at a time
        out[:, p, :] = (layer_norm(src[p], g, b, eps) @ wb.T).T
    return out


def _project(xr, w, heads):
    """LayerNormed tokens [L, c] -> q, k, v, g each [L, heads, d]."""
    L = xr.shape[0]
    q = (xr @ np.asarray(w["w_q"], _F).T).reshape(L, heads, -1)
    k = (xr @ np.asarray(w["w_k"], _F).T).reshape(L, heads, -1)
    v = (xr @ np.asarray(w["w_v"], _F).T).reshape(L, heads, -1)
    g = sigmoid(xr @ np.asarray(w["w_g"], _F).T + np.asarray(w["b_g"], _F)).reshape(L, heads, -1)
    return q, k, v, g


def gated_attention(mode, x, z, mask, w, heads, eps=1e-5, rows=None):
    """Gated axial attention, one of four modes.  x: [n_a, n_b, c]; z: [n_b, n_b, c_z]
    (row mode only); mask: [n_a, n_b] of 0/1 or None; w: dict of weights.

    Returns out [n_a, n_b, c] (float64).  If rows is given, only those batch rows
    (s for row mode, i for column mode, i for triangle-start, j for triangle-end) are
    evaluated and the result is [len(rows), L, c] in that order: batch rows are
    independent given the bias (Section 4.2: attention along an axis needs nothing from
    the other rows).

    With q, k, v, g the per-head projections of LN(x) and M(t) = 0 if t == 1 else -inf:
      row:        S[s,h,i,j] = q[s,i,h].k[s,j,h]/sqrt(d) + b[h,i,j] + M(mask[s,j]); softmax over j
      column:     S[i,h,s,t] = q[s,i,h].k[t,i,h]/sqrt(d)            + M(mask[t,i]); softmax over t
      tri-start:  S[i,h,j,k] = q[i,j,h].k[i,k,h]/sqrt(d) + b[h,j,k] + M(mask[i,k]); softmax over k
      tri-end:    S[j,h,i,k] = q[i,j,h].k[k,j,h]/sqrt(d) + b[h,k,i] + M(mask[k,j]); softmax over k
    o = g * (P v) per head, out = concat_heads(o) W_o^T + b_o.
    """
    n_a, n_b, c = x.shape
    wo = np.asarray(w["w_o"], _F)
    bo = np.asarray(w["b_o"], _F)
    bias = pair_bias(mode, x, z, w, eps)
    along_b = mode in (MODE_ROW, MODE_TRI_START)          # attended axis is b
    n_rows, L = (n_a, n_b) if along_b else (n_b, n_a)
    want = range(n_rows) if rows is None else list(rows)
    res = np.empty((len(want), L, c), dtype=_F)
    for n, r in enumerate(want):
        xr = x[r, :, :] if along_b else x[:, r, :]        # the L tokens of batch row r
        xr = layer_norm(xr, w["ln_g"], w["ln_b"], eps)
        q, k, v, g = _project(xr, w, heads)
        d = q.shape[-1]
        if mask is None:
            valid = np.ones(L, dtype=bool)
        else:
            valid = (np.asarray(mask[r, :] if along_b else mask[:, r]) != 0)
        o = np.empty((L, heads, d), dtype=_F)
        for h in range(heads):
            s = (q[:, h, :] @ k[:, h, :].T) / np.sqrt(d)  # [query, key]
            if mode in (MODE_ROW, MODE_TRI_START):
                s = s + bias[h]                           # b[h, query, key]
            elif mode == MODE_TRI_END:
                s = s + bias[h].T                         # b[h, key, query]
            p = masked_softmax(s, valid)
            o[:, h, :] = g[:, h, :] * (p @ v[:, h, :])
        res[n] = o.reshape(L, heads * d) @ wo.T + bo
    if rows is not None:
        return res
    return res if along_b else res.transpose(1, 0, 2)


def gated_attention_residual(mode, x, z, mask, w, heads, eps=1e-5, rows=None):
    """The module together with the residual add that closes it in the Evoformer block:
    x + gated_attention(x) (Section 5.2 lists "bias + dropout + add" as the module's last
    fused step; b_o is the bias, dropout is the identity at inference, x is what is added).
    rows as in gated_attention: [len(rows), L, c] for the chosen batch rows."""
    y = gated_attention(mode, x, z, mask, w, heads, eps, rows)
    x = np.asarray(x, _F)
    if rows is None:
        return x + y
    rows = list(rows)
    if mode in (MODE_ROW, MODE_TRI_START):
        return x[rows, :, :] + y
    return x[:, rows, :].transpose(1, 0, 2) + y


def attention_weights(mode, x, z, mask, w, heads, eps, r, h):
    """The softmax weights P[query, key] of batch row r, head h (for invariant tests)."""
    along_b = mode in (MODE_ROW, MODE_TRI_START)
    xr = layer_norm(x[r, :, :] if along_b else x[:, r, :], w["ln_g"], w["ln_b"], eps)
    q, k, _, _ = _project(xr, w, heads)
    d = q.shape[-1]
    s = (q[:, h, :] @ k[:, h, :].T) / np.sqrt(d)
    bias = pair_bias(mode, x, z, w, eps)
    if mode in (MODE_ROW, MODE_TRI_START):
        s = s + bias[h]
    elif mode == MODE_TRI_END:
        s = s + bias[h].T
    L = xr.shape[0]
    valid = np.ones(L, bool) if mask is None else (np.asarray(mask[r, :] if along_b else mask[:, r]) != 0)
    return masked_softmax(s, valid)
