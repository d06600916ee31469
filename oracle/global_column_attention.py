"""CPU oracle for the global column attention of the extra-MSA stack (float64, numpy).

TEST INFRASTRUCTURE ONLY.  It defines what the HIP library's ff_global_column_attention must compute;
it is imported by tests/, never by the product path, and it shares no code with the kernels.

What the paper fixes: the extra-MSA stack works on N_extra_seq sequences (Table 1: 1024 in initial
training, 5120 in fine-tuning) and is one of the optional modules of the model (Section 6.2).  The
paper does not describe its column attention; it defers to AlphaFold 2, whose published "MSA column
global self-attention" is written out here.  Per residue column i, with mn = LayerNorm(m):

    qbar[i]     = mean over the unmasked sequences s of mn[s, i, :]
    q[i, h, :]  = (W_q qbar[i])[h] / sqrt(d)                 H heads of d channels, no bias
    k[s, i, :]  = W_k mn[s, i],   v[s, i, :] = W_v mn[s, i]   ONE key / value head of d channels, no bias
    P[i, h, :]  = softmax over s of q[i, h] . k[s, i]        masked sequences get weight exactly 0
    o[i, h, :]  = sum_s P[i, h, s] v[s, i, :]
    g[s, i]     = sigmoid(W_g mn[s, i] + b_g)                per sequence, H d channels
    out[s, i]   = W_o (g[s, i] * concat_h o[i, h]) + b_o

so every sequence of a column receives the same attended vector, shaped by its own gate: the cost is
linear in the number of sequences instead of quadratic.

Readings where the sources are silent (restated in the design notes):
  * the query average runs over the unmasked sequences only (sum of mask * mn divided by the number of
    unmasked sequences, no regulariser in the denominator);
  * a column without any unmasked sequence gets zero context, so its outputs are b_o (as for the other
    attention modules);
  * LayerNorm, weight layout [out, in], head-major channel split as in the other modules.

Parity pins: tests/test_oracle_global_pins.py (scalar brute force, torch float64 composition, the reduction
to the plain column attention oracle when all sequences of a column are equal, closed forms, invariants).
"""
from __future__ import annotations

import numpy as np

_F = np.float64


def layer_norm(v, gamma, beta, eps):
    v = np.asarray(v, dtype=_F)
    mu = v.mean(axis=-1, keepdims=True)
    var = ((v - mu) ** 2).mean(axis=-1, keepdims=True)
    return (v - mu) / np.sqrt(var + eps) * np.asarray(gamma, _F) + np.asarray(beta, _F)


def sigmoid(t):
    return 1.0 / (1.0 + np.exp(-t))


def global_column_attention(m, mask, w, heads, eps=1e-5, cols=None):
    """m [N_seq, N_res, c]; mask [N_seq, N_res] of 0/1 or None; returns out [N_seq, N_res, c] (float64).
    cols: evaluate only these residue columns and return [N_seq, len(cols), c] (columns are independent)."""
    m = np.asarray(m, _F)
    n_seq, n_res, c = m.shape
    wq, wk, wv = (np.asarray(w[k], _F) for k in ("w_q", "w_k", "w_v"))
    wg, bg, wo, bo = (np.asarray(w[k], _F) for k in ("w_g", "b_g", "w_o", "b_o"))
    d = wk.shape[0]
    want = range(n_res) if cols is None else list(cols)
    out = np.empty((n_seq, len(want), c), dtype=_F)
    for n, i in enumerate(want):
        x = layer_norm(m[:, i, :], w["ln_g"], w["ln_b"], eps)              # [N_seq, c]
        valid = np.ones(n_seq, bool) if mask is None else (np.asarray(mask)[:, i] != 0)
        o = np.zeros((heads, d), dtype=_F)
        if valid.any():
            qbar = x[valid].mean(axis=0)
            q = (wq @ qbar).reshape(heads, d) / np.sqrt(d)
            k = x @ wk.T                                                   # [N_seq, d]
            v = x @ wv.T
            s = q @ k[valid].T                                             # [heads, valid sequences]
            e = np.exp(s - s.max(axis=1, keepdims=True))
            p = e / e.sum(axis=1, keepdims=True)
            o = p @ v[valid]                                               # [heads, d]
        g = sigmoid(x @ wg.T + bg)                                         # [N_seq, heads * d]
        out[:, n, :] = (g * o.reshape(1, heads * d)) @ wo.T + bo
    return out
