"""CPU oracle for the triangular multiplicative update of the pair stack (float64, numpy).

TEST INFRASTRUCTURE ONLY.  It defines what the HIP library's ff_triangle_multiplication must
compute; it is imported by tests/, the smoke check and the benchmark's cpu_baseline leg, never
by the product path, and it shares no code with the kernels.

What the paper fixes: the pair representation is processed by attention blocks "with additional
triangular updates module" that "uses triangular relationships in pair information to infer and
update representations" (Section 2.3, Figure 3); the module has a left and a right projection, each
with a gate, which the paper's kernels merge into one GEMM (Section 5.2, merge GEMM); there is an
outgoing and an incoming form (Section 4.2, Table 3: two all-gathers, "incoming and outgoing").
The paper prints no equations and defers to AlphaFold 2, whose published algorithms
("triangular multiplicative update using outgoing / incoming edges") are written out here:

    zn      = LayerNorm_in(z)                                              [N, N, c_z]
    a       = mask * sigmoid(zn W_ag^T + b_ag) * (zn W_ap^T + b_ap)         [N, N, c]   left
    b       = mask * sigmoid(zn W_bg^T + b_bg) * (zn W_bp^T + b_bp)         [N, N, c]   right
    g       = sigmoid(zn W_g^T + b_g)                                      [N, N, c_z]
    outgoing:  t[i, j, :] = sum_k a[i, k, :] * b[j, k, :]
    incoming:  t[i, j, :] = sum_k a[k, i, :] * b[k, j, :]
    out     = g * (LayerNorm_out(t) W_o^T + b_o)                           [N, N, c_z]

Readings where the sources are silent (restated in the design notes):
  * every linear layer has an additive bias (AlphaFold's default linear layer);
  * both LayerNorms: biased variance, eps inside the square root, per-channel gain and offset;
  * mask is a 0/1 pair mask [N, N]; it multiplies a and b (a masked pair takes no part in any sum
    over k) but neither g nor the output position itself; None means all ones;
  * the residual form is z + out (Section 5.2: bias + dropout + add, dropout off).

Nothing is tiled, fused or reordered: the sum over k is one einsum per form.
Parity pins: tests/test_oracle_trimul_pins.py (scalar brute force, an independent torch float64
composition, closed forms, the outgoing/incoming transposition identity, mask and permutation
invariants).
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


def _linear(x, w, b):
    return x @ np.asarray(w, _F).T + np.asarray(b, _F)


def _side(zn, mask, w, side):
    """Left (side "a") or right ("b") gated projection of the normalised pair representation."""
    m = 1.0 if mask is None else np.asarray(mask, _F)[..., None]
    return m * sigmoid(_linear(zn, w[f"w_{side}g"], w[f"b_{side}g"])) * _linear(zn, w[f"w_{side}p"], w[f"b_{side}p"])


def projections(z, mask, w, eps):
    """(a, b, g) of the definition above."""
    zn = layer_norm(z, w["ln_g"], w["ln_b"], eps)
    a = _side(zn, mask, w, "a")
    b = _side(zn, mask, w, "b")
    g = sigmoid(_linear(zn, w["w_g"], w["b_g"]))
    return a, b, g


def triangle_multiplication(z, mask, w, incoming=False, eps=1e-5, residual=False, rows=None):
    """Triangular multiplicative update of the pair representation z [N, N, c_z] (float64 out).
    rows: evaluate only these rows i of the output and return [len(rows), N, c_z]: out[i] needs a of row i (outgoing)
    or of column i (incoming), all of b, and the gate of row i; nothing else of the definition changes."""
    z = np.asarray(z, _F)
    if rows is None:
        a, b, g = projections(z, mask, w, eps)
        if incoming:
            t = np.einsum("kic,kjc->ijc", a, b)
        else:
            t = np.einsum("ikc,jkc->ijc", a, b)
        out = g * _linear(layer_norm(t, w["lno_g"], w["lno_b"], eps), w["w_o"], w["b_o"])
        return z + out if residual else out
    sel = list(rows)
    zn = layer_norm(z, w["ln_g"], w["ln_b"], eps)
    mk = None if mask is None else np.asarray(mask, _F)
    b = _side(zn, mk, w, "b")
    if incoming:
        a = _side(zn[:, sel], None if mk is None else mk[:, sel], w, "a")       # a[k, i] for the wanted i
        t = np.stack([np.einsum("kc,kjc->jc", a[:, n], b) for n in range(len(sel))])
    else:
        a = _side(zn[sel], None if mk is None else mk[sel], w, "a")             # a[i, k] for the wanted i
        t = np.stack([np.einsum("kc,jkc->jc", a[n], b) for n in range(len(sel))])
    g = sigmoid(_linear(zn[sel], w["w_g"], w["b_g"]))
    out = g * _linear(layer_norm(t, w["lno_g"], w["lno_b"], eps), w["w_o"], w["b_o"])
    return z[sel] + out if residual else out
