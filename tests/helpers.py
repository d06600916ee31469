"""Helpers shared by the tests: small seeded cases and error measures."""
import numpy as np

from paper_2203_00854_amd import inputs as I


def small_spec(mode, n_a, n_b, c, heads, d, c_z=0, dtype="f32", mask="none", name=None, chunk_rows=0):
    if mode == I.MODE_ROW and c_z == 0:
        c_z = 8
    if mode != I.MODE_ROW:
        c_z = 0
    name = name or f"t_{I.MODE_NAMES[mode]}_{dtype}_{n_a}x{n_b}x{c}_h{heads}d{d}_{mask}"
    return I.CaseSpec(name, mode, dtype, n_a, n_b, c, c_z, heads, d, mask, chunk_rows=chunk_rows)


def f64_inputs(case):
    """(x, z, mask, weights) as float64 arrays holding exactly the stored values."""
    x = case.widened("x").astype(np.float64)
    z = None if case.z is None else case.widened("z").astype(np.float64)
    w = {k: v.astype(np.float64) for k, v in case.widened_weights().items()}
    return x, z, case.mask, w


def max_abs(a, b):
    return float(np.max(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64))))


def rel_l2(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))
