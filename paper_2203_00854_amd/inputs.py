"""Seeded synthetic inputs for the Evoformer gated-attention path.

This module is shared by the tests, the benchmark and the smoke check so that the CPU
oracle and the HIP library always see the very same arrays.  It holds none of the
method's arithmetic: only a counter-based random generator, dtype rounding, the
workload shapes and the mask patterns.

Generator: splitmix64 used as a counter-based generator (element i of a stream is
finalise(key + (i+1)*golden)), turned into standard normals with the Box-Muller
transform in float64.  A stream is keyed by (seed, case name, tensor name), so the
values do not depend on generation order, chunking or thread count, nor on torch's RNG.

The shapes are the ones the paper gives for AlphaFold's Evoformer (Table 1: N_r=256,
N_s=128 initial training; Table 2: hidden 256 / 8 heads for the MSA stack, hidden
128 / 4 heads for the pair stack; Section 6.2: N_r=2048 long-sequence inference with
chunk size 64).  The paper's real protein MSAs are replaced by i.i.d. N(0,1)
activations and N(0, 1/fan_in) weights.
"""
from __future__ import annotations

import hashlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

SEED = 220300854

MODE_ROW, MODE_COL, MODE_TRI_START, MODE_TRI_END = 0, 1, 2, 3
MODE_NAMES = {MODE_ROW: "msa_row", MODE_COL: "msa_col",
              MODE_TRI_START: "tri_start", MODE_TRI_END: "tri_end"}

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


# --------------------------------------------------------------------------- generator
def stream_key(seed: int, case: str, tensor: str) -> np.uint64:
    """64-bit key of one random stream."""
    h = hashlib.blake2b(f"{seed}/{case}/{tensor}".encode(), digest_size=8).digest()
    return np.uint64(int.from_bytes(h, "little"))


def _finalise(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _bits(key: np.uint64, first: int, count: int) -> np.ndarray:
    """count 64-bit words of the stream, counters first .. first+count-1."""
    with np.errstate(over="ignore"):
        ctr = np.arange(first + 1, first + count + 1, dtype=np.uint64)
        return _finalise(key + ctr * _GOLDEN)


def _uniform(key: np.uint64, first: int, count: int) -> np.ndarray:
    """Uniforms in the open interval (0, 1), 53 bits each."""
    return ((_bits(key, first, count) >> np.uint64(11)).astype(np.float64) + 0.5) * 2.0 ** -53


def _normal_pairs(key: np.uint64, first_pair: int, pairs: int) -> np.ndarray:
    """2*pairs normals: pair p (counters 2p, 2p+1) gives elements 2p (cos) and 2p+1 (sin)."""
    u = _uniform(key, 2 * first_pair, 2 * pairs)
    rad = np.sqrt(-2.0 * np.log(u[0::2]))
    ang = 2.0 * np.pi * u[1::2]
    out = np.empty(2 * pairs, dtype=np.float64)
    out[0::2] = rad * np.cos(ang)
    out[1::2] = rad * np.sin(ang)
    return out


def normal(key: np.uint64, count: int, block: int = 1 << 18, threads: int = 8) -> np.ndarray:
    """count standard normals (float64); elements 2p and 2p+1 come from counters 2p, 2p+1."""
    pairs_total = (count + 1) // 2
    out = np.empty(2 * pairs_total, dtype=np.float64)
    starts = list(range(0, pairs_total, block))

    def work(s):
        n = min(block, pairs_total - s)
        out[2 * s:2 * (s + n)] = _normal_pairs(key, s, n)

    if len(starts) <= 1:
        for s in starts:
            work(s)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, starts))
    return out[:count]


def bernoulli(key: np.uint64, count: int, p_one: float) -> np.ndarray:
    """count 0/1 draws (float32), P(1) = p_one."""
    return (_uniform(key, 0, count) < p_one).astype(np.float32)


# --------------------------------------------------------------------------- dtypes
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); result as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32, exactly."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(values_f64: np.ndarray, dtype: str) -> np.ndarray:
    """Round generated float64 values once to the case's storage type.

    "f32": float32 array.  "bf16": uint16 array of bfloat16 bit patterns (float64 is
    rounded to float32 and then to bfloat16, both nearest-even)."""
    f = values_f64.astype(np.float32)
    if dtype == "f32":
        return f
    if dtype == "bf16":
        return f32_to_bf16_bits(f)
    raise ValueError(dtype)


def widen(stored: np.ndarray) -> np.ndarray:
    """Stored tensor -> float32 array holding exactly the stored values."""
    if stored.dtype == np.uint16:
        return bf16_bits_to_f32(stored)
    return np.asarray(stored, dtype=np.float32)


# --------------------------------------------------------------------------- cases
@dataclass(frozen=True)
class CaseSpec:
    name: str
    mode: int
    dtype: str              # "f32" | "bf16"
    n_a: int                # x is [n_a, n_b, c]
    n_b: int
    c: int
    c_z: int                # channels of z (MSA row mode only, else 0)
    heads: int
    head_dim: int
    mask: str               # "none" | "tail:K" | "outer:P" | "random:P"
    chunk_rows: int = 0     # 0 = unchunked
    ln_eps: float = 1e-5
    stream: str = ""        # random-stream name; cases with the same one share their data

    @property
    def stream_name(self):
        return self.stream or self.name

    @property
    def batch_len(self):    # (R, L): independent rows, attended length
        return (self.n_a, self.n_b) if self.mode in (MODE_ROW, MODE_TRI_START) else (self.n_b, self.n_a)


@dataclass
class Case:
    spec: CaseSpec
    x: np.ndarray                       # storage dtype, [n_a, n_b, c]
    z: Optional[np.ndarray]             # storage dtype, [n_b, n_b, c_z] (row mode) or None
    mask: Optional[np.ndarray]          # float32 0/1, [n_a, n_b], or None
    weights: Dict[str, np.ndarray] = field(default_factory=dict)   # storage dtype

    def widened(self, name: str) -> np.ndarray:
        if name == "x":
            return widen(self.x)
        if name == "z":
            return widen(self.z)
        return widen(self.weights[name])

    def widened_weights(self) -> Dict[str, np.ndarray]:
        return {k: widen(v) for k, v in self.weights.items()}


# The five workloads of the benchmark definition.
SPECS = {
    "c1_row_f32_tiny": CaseSpec("c1_row_f32_tiny", MODE_ROW, "f32", 8, 32, 32, 16, 4, 8, "tail:4"),
    "c2_row_bf16_train": CaseSpec("c2_row_bf16_train", MODE_ROW, "bf16", 128, 256, 256, 128, 8, 32, "tail:16"),
    "c3_tri_start_bf16_256": CaseSpec("c3_tri_start_bf16_256", MODE_TRI_START, "bf16", 256, 256, 128, 0, 4, 32, "outer:0.95", stream="c3_tri_bf16_256"),
    "c3_tri_end_bf16_256": CaseSpec("c3_tri_end_bf16_256", MODE_TRI_END, "bf16", 256, 256, 128, 0, 4, 32, "outer:0.95", stream="c3_tri_bf16_256"),
    "c4_col_bf16_extra": CaseSpec("c4_col_bf16_extra", MODE_COL, "bf16", 1024, 384, 64, 0, 8, 8, "tail:102"),
    "c5_tri_start_bf16_2048": CaseSpec("c5_tri_start_bf16_2048", MODE_TRI_START, "bf16", 2048, 2048, 128, 0, 4, 32, "none", chunk_rows=64),
}

# The paper's second training setting (Table 1, fine-tuning: N_res = 384, N_seq = 512,
# N_extra_seq = 5120) at the same channel and head counts; padding as in the workloads above
# (a trailing tenth of the attended axis, a Bernoulli(0.95) residue mask for the pair modules).
SPECS.update({
    "ft_row_bf16_512x384": CaseSpec("ft_row_bf16_512x384", MODE_ROW, "bf16", 512, 384, 256, 128, 8, 32, "tail:38"),
    "ft_col_bf16_512x384": CaseSpec("ft_col_bf16_512x384", MODE_COL, "bf16", 512, 384, 256, 0, 8, 32, "tail:51",
                                    stream="ft_row_bf16_512x384"),
    "ft_tri_start_bf16_384": CaseSpec("ft_tri_start_bf16_384", MODE_TRI_START, "bf16", 384, 384, 128, 0, 4, 32,
                                      "outer:0.95", stream="ft_tri_bf16_384"),
    "ft_tri_end_bf16_384": CaseSpec("ft_tri_end_bf16_384", MODE_TRI_END, "bf16", 384, 384, 128, 0, 4, 32,
                                    "outer:0.95", stream="ft_tri_bf16_384"),
    "ft_col_bf16_extra_5120": CaseSpec("ft_col_bf16_extra_5120", MODE_COL, "bf16", 5120, 384, 64, 0, 8, 8, "tail:512"),
})


def make_mask(spec: CaseSpec, seed: int = SEED) -> Optional[np.ndarray]:
    """0/1 float32 mask [n_a, n_b], or None.  The entry at (a, b) says whether token
    (a, b) may be attended to as a key.

    "tail:K"   the last K positions of the attended axis are padding;
    "outer:P"  a residue vector r ~ Bernoulli(P) (square inputs), mask = r r^T;
    "random:P" i.i.d. Bernoulli(P) entries."""
    kind, _, arg = spec.mask.partition(":")
    if kind == "none":
        return None
    m = np.ones((spec.n_a, spec.n_b), dtype=np.float32)
    if kind == "tail":
        k = int(arg)
        if spec.mode in (MODE_ROW, MODE_TRI_START):
            m[:, spec.n_b - k:] = 0.0
        else:
            m[spec.n_a - k:, :] = 0.0
        return m
    if kind == "outer":
        assert spec.n_a == spec.n_b
        r = bernoulli(stream_key(seed, spec.stream_name, "mask"), spec.n_a, float(arg))
        return np.outer(r, r).astype(np.float32)
    if kind == "random":
        r = bernoulli(stream_key(seed, spec.stream_name, "mask"), spec.n_a * spec.n_b, float(arg))
        return r.reshape(spec.n_a, spec.n_b)
    raise ValueError(spec.mask)


def make_case(spec_or_name, seed: int = SEED) -> Case:
    spec = SPECS[spec_or_name] if isinstance(spec_or_name, str) else spec_or_name
    hd = spec.heads * spec.head_dim

    def gen(name, shape, scale=1.0, shift=0.0):
        n = int(np.prod(shape))
        v = normal(stream_key(seed, spec.stream_name, name), n)
        if scale != 1.0:
            v *= scale
        if shift != 0.0:
            v += shift
        return to_storage(v, spec.dtype).reshape(shape)

    c = spec.c
    x = gen("x", (spec.n_a, spec.n_b, c))
    z = None
    w: Dict[str, np.ndarray] = {}
    w["ln_g"] = gen("ln_g", (c,), 0.1, 1.0)
    w["ln_b"] = gen("ln_b", (c,), 0.1)
    if spec.mode == MODE_ROW:
        z = gen("z", (spec.n_b, spec.n_b, spec.c_z))
        w["lnz_g"] = gen("lnz_g", (spec.c_z,), 0.1, 1.0)
        w["lnz_b"] = gen("lnz_b", (spec.c_z,), 0.1)
        w["w_b"] = gen("w_b", (spec.heads, spec.c_z), spec.c_z ** -0.5)
    elif spec.mode in (MODE_TRI_START, MODE_TRI_END):
        w["w_b"] = gen("w_b", (spec.heads, c), c ** -0.5)
    for nm in ("w_q", "w_k", "w_v", "w_g"):
        w[nm] = gen(nm, (hd, c), c ** -0.5)
    w["b_g"] = to_storage(np.ones(hd), spec.dtype)
    w["w_o"] = gen("w_o", (c, hd), hd ** -0.5)
    w["b_o"] = gen("b_o", (c,), 0.1)
    return Case(spec, x, z, make_mask(spec, seed), w)


# --------------------------------------------------------------------------- triangular multiplicative update
TRIMUL_WEIGHTS = ("ln_g", "ln_b", "w_ap", "b_ap", "w_ag", "b_ag", "w_bp", "b_bp", "w_bg", "b_bg", "w_g", "b_g",
                  "lno_g", "lno_b", "w_o", "b_o")


@dataclass(frozen=True)
class TriMulSpec:
    """Pair-stack triangular multiplicative update (Section 2.3, Figure 3): z is [n, n, c_z],
    the left/right projections have c channels.  mask as in CaseSpec ("none" | "outer:P" | "random:P")."""
    name: str
    dtype: str
    n: int
    c_z: int
    c: int
    incoming: bool
    mask: str = "none"
    ln_eps: float = 1e-5
    stream: str = ""

    @property
    def stream_name(self):
        return self.stream or self.name


@dataclass
class TriMulCase:
    spec: TriMulSpec
    z: np.ndarray
    mask: Optional[np.ndarray]
    weights: Dict[str, np.ndarray] = field(default_factory=dict)

    def widened_weights(self) -> Dict[str, np.ndarray]:
        return {k: widen(v) for k, v in self.weights.items()}


# Pair-stack shapes of the paper (Table 1: N_res 256 initial training, 384 fine-tuning; Table 2: pair
# hidden 128) and the long-sequence inference length of Section 6.2.
TRIMUL_SPECS = {
    "tm_out_bf16_256": TriMulSpec("tm_out_bf16_256", "bf16", 256, 128, 128, False, "outer:0.95", stream="tm_bf16_256"),
    "tm_in_bf16_256": TriMulSpec("tm_in_bf16_256", "bf16", 256, 128, 128, True, "outer:0.95", stream="tm_bf16_256"),
    "tm_out_bf16_384": TriMulSpec("tm_out_bf16_384", "bf16", 384, 128, 128, False, "outer:0.95", stream="tm_bf16_384"),
    "tm_in_bf16_384": TriMulSpec("tm_in_bf16_384", "bf16", 384, 128, 128, True, "outer:0.95", stream="tm_bf16_384"),
    "tm_out_bf16_2048": TriMulSpec("tm_out_bf16_2048", "bf16", 2048, 128, 128, False, "none"),
}


def make_trimul_case(spec_or_name, seed: int = SEED) -> TriMulCase:
    """Activations N(0,1); weights N(0, 1/fan_in); gate biases 1; other biases 0.1 N(0,1); LayerNorm gains
    1 + 0.1 N(0,1), offsets 0.1 N(0,1)."""
    spec = TRIMUL_SPECS[spec_or_name] if isinstance(spec_or_name, str) else spec_or_name

    def gen(name, shape, scale=1.0, shift=0.0):
        v = normal(stream_key(seed, spec.stream_name, name), int(np.prod(shape)))
        return to_storage(v * scale + shift, spec.dtype).reshape(shape)

    cz, c, n = spec.c_z, spec.c, spec.n
    w: Dict[str, np.ndarray] = {}
    w["ln_g"] = gen("ln_g", (cz,), 0.1, 1.0)
    w["ln_b"] = gen("ln_b", (cz,), 0.1)
    for side in ("a", "b"):
        w[f"w_{side}p"] = gen(f"w_{side}p", (c, cz), cz ** -0.5)
        w[f"b_{side}p"] = gen(f"b_{side}p", (c,), 0.1)
        w[f"w_{side}g"] = gen(f"w_{side}g", (c, cz), cz ** -0.5)
        w[f"b_{side}g"] = to_storage(np.ones(c), spec.dtype)
    w["w_g"] = gen("w_g", (cz, cz), cz ** -0.5)
    w["b_g"] = to_storage(np.ones(cz), spec.dtype)
    w["lno_g"] = gen("lno_g", (c,), 0.1, 1.0)
    w["lno_b"] = gen("lno_b", (c,), 0.1)
    w["w_o"] = gen("w_o", (cz, c), c ** -0.5)
    w["b_o"] = gen("b_o", (cz,), 0.1)
    z = gen("z", (n, n, cz))
    kind, _, arg = spec.mask.partition(":")
    mask = None
    if kind == "outer":
        r = bernoulli(stream_key(seed, spec.stream_name, "mask"), n, float(arg))
        mask = np.outer(r, r).astype(np.float32)
    elif kind == "random":
        mask = bernoulli(stream_key(seed, spec.stream_name, "mask"), n * n, float(arg)).reshape(n, n)
    elif kind != "none":
        raise ValueError(spec.mask)
    return TriMulCase(spec, z, mask, w)


# --------------------------------------------------------------------------- global column attention (extra-MSA stack)
@dataclass(frozen=True)
class GlobalSpec:
    """MSA column global attention: m is [n_seq, n_res, c]; H heads of d channels for the query and
    the gate, one shared key / value head of d channels.  mask as in CaseSpec ("none" | "tail:K" | "random:P"),
    "tail" padding the last K sequences."""
    name: str
    dtype: str
    n_seq: int
    n_res: int
    c: int
    heads: int
    head_dim: int
    mask: str = "none"
    ln_eps: float = 1e-5
    stream: str = ""

    @property
    def stream_name(self):
        return self.stream or self.name


@dataclass
class GlobalCase:
    spec: GlobalSpec
    m: np.ndarray
    mask: Optional[np.ndarray]
    weights: Dict[str, np.ndarray] = field(default_factory=dict)

    def widened_weights(self) -> Dict[str, np.ndarray]:
        return {k: widen(v) for k, v in self.weights.items()}


# Extra-MSA shapes of the paper (Table 1: N_extra_seq 1024 / 5120, N_res 256 / 384) with AlphaFold's
# extra-MSA channel count (64) and 8 heads of 8 channels, as in the column-attention workload.
GLOBAL_SPECS = {
    "gca_bf16_1024x384": GlobalSpec("gca_bf16_1024x384", "bf16", 1024, 384, 64, 8, 8, "tail:102"),
    "gca_bf16_5120x384": GlobalSpec("gca_bf16_5120x384", "bf16", 5120, 384, 64, 8, 8, "tail:512"),
}


def make_global_case(spec_or_name, seed: int = SEED) -> GlobalCase:
    spec = GLOBAL_SPECS[spec_or_name] if isinstance(spec_or_name, str) else spec_or_name

    def gen(name, shape, scale=1.0, shift=0.0):
        v = normal(stream_key(seed, spec.stream_name, name), int(np.prod(shape)))
        return to_storage(v * scale + shift, spec.dtype).reshape(shape)

    c, hd, d = spec.c, spec.heads * spec.head_dim, spec.head_dim
    w: Dict[str, np.ndarray] = {}
    w["ln_g"] = gen("ln_g", (c,), 0.1, 1.0)
    w["ln_b"] = gen("ln_b", (c,), 0.1)
    w["w_q"] = gen("w_q", (hd, c), c ** -0.5)
    w["w_k"] = gen("w_k", (d, c), c ** -0.5)
    w["w_v"] = gen("w_v", (d, c), c ** -0.5)
    w["w_g"] = gen("w_g", (hd, c), c ** -0.5)
    w["b_g"] = to_storage(np.ones(hd), spec.dtype)
    w["w_o"] = gen("w_o", (c, hd), hd ** -0.5)
    w["b_o"] = gen("b_o", (c,), 0.1)
    m = gen("m", (spec.n_seq, spec.n_res, c))
    kind, _, arg = spec.mask.partition(":")
    mask = None
    if kind == "tail":
        mask = np.ones((spec.n_seq, spec.n_res), np.float32)
        mask[spec.n_seq - int(arg):, :] = 0.0
    elif kind == "random":
        mask = bernoulli(stream_key(seed, spec.stream_name, "mask"), spec.n_seq * spec.n_res, float(arg)).reshape(
            spec.n_seq, spec.n_res)
    elif kind != "none":
        raise ValueError(spec.mask)
    return GlobalCase(spec, m, mask, w)


# --------------------------------------------------------------------------- attention core (for its backward pass)
@dataclass(frozen=True)
class CoreSpec:
    """Operands of the fused attention core: q, k, v, g, do are [rows, heads, length, head_dim]; bias is
    [heads, length, length] float32 (or absent), mask [rows, length] ("none" | "tail:K" | "random:P")."""
    name: str
    rows: int
    heads: int
    length: int
    head_dim: int
    has_bias: bool = True
    mask: str = "none"
    stream: str = ""

    @property
    def stream_name(self):
        return self.stream or self.name


@dataclass
class CoreCase:
    spec: CoreSpec
    tensors: Dict[str, np.ndarray] = field(default_factory=dict)   # q, k, v, g, do: bf16 bit patterns; bias: float32
    mask: Optional[np.ndarray] = None


# the attention cores of the paper's training shapes (Table 1 / Table 2): MSA row attention (128 rows, 8 heads of
# 32, 256 residues, pair bias) and triangle attention (256 rows, 4 heads of 32, 256 residues)
CORE_SPECS = {
    "core_row_256": CoreSpec("core_row_256", 128, 8, 256, 32, True, "tail:16"),
    "core_tri_256": CoreSpec("core_tri_256", 256, 4, 256, 32, True, "random:0.95"),
}


def make_core_case(spec_or_name, seed: int = SEED) -> CoreCase:
    """q, k, v ~ N(0,1) (what the projections of normalised activations give), g = sigmoid of N(1,1), bias ~ N(0,1),
    do ~ N(0,1); all but the bias rounded to bfloat16."""
    spec = CORE_SPECS[spec_or_name] if isinstance(spec_or_name, str) else spec_or_name
    shape = (spec.rows, spec.heads, spec.length, spec.head_dim)
    n = int(np.prod(shape))

    def gen(name, count):
        return normal(stream_key(seed, spec.stream_name, name), count)

    t: Dict[str, np.ndarray] = {}
    for name in ("q", "k", "v", "do"):
        t[name] = to_storage(gen(name, n), "bf16").reshape(shape)
    t["g"] = to_storage(1.0 / (1.0 + np.exp(-(gen("g", n) + 1.0))), "bf16").reshape(shape)
    if spec.has_bias:
        t["bias"] = gen("bias", spec.heads * spec.length * spec.length).astype(np.float32).reshape(
            spec.heads, spec.length, spec.length)
    kind, _, arg = spec.mask.partition(":")
    mask = None
    if kind == "tail":
        mask = np.ones((spec.rows, spec.length), np.float32)
        mask[:, spec.length - int(arg):] = 0.0
    elif kind == "random":
        mask = bernoulli(stream_key(seed, spec.stream_name, "mask"), spec.rows * spec.length, float(arg)).reshape(
            spec.rows, spec.length)
    elif kind != "none":
        raise ValueError(spec.mask)
    return CoreCase(spec, t, mask)
