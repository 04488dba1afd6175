"""Seeded synthetic inputs for msGeMM (arxiv 2310.06178).

This module only *makes bytes*: 4-bit (and 8-bit) weight codes, activations,
scales, value maps and the table of benchmark shapes.  It holds none of the method's arithmetic (no
decoding of codes, no products, no tables), so both the CPU oracle's tests and
the HIP path's tests can feed the very same arrays to the two sides.

Storage conventions (the paper fixes none of them; Section 4 only asks that the
d codes of a group be adjacent in a row-major M):
  codes  uint8 [m][k/2]; byte t of row i = column 2t in bits 3:0, column 2t+1
         in bits 7:4.
  X      [b][k]: one activation vector (a column of the paper's k x b matrix X)
         per row, so it is contiguous.  fp32 / fp16 as numpy dtypes, bf16 as
         uint16 bit patterns, int8 as int8.
  scales float16 [m][k/scale_group].
"""
from __future__ import annotations

import numpy as np

# The five benchmark configurations (LLM-shaped GeMMs), then the paper's own
# shapes -- the two GeMMs of the GPT-3 MLP block, Section 5 -- as a second
# workload ("mlp1", "mlp2": one activation vector; "_b16": a batch of 16).  The
# paper gives no data for them either: same recipe, seeds 11 and 12.
CONFIGS = {
    "cfg1":  dict(m=1024,  k=1024, b=1,  x="f32",  y="f32",  scale_group=0,   d=2, seed=0),
    "cfg2":  dict(m=16384, k=4096, b=1,  x="f16",  y="f16",  scale_group=0,   d=2, seed=2),
    "cfg3a": dict(m=14336, k=4096, b=8,  x="f16",  y="f16",  scale_group=128, d=2, seed=3),
    "cfg3b": dict(m=14336, k=4096, b=16, x="f16",  y="f16",  scale_group=128, d=2, seed=3),
    "cfg4":  dict(m=8192,  k=8192, b=16, x="i8",   y="i32",  scale_group=0,   d=2, seed=4),
    "cfg5":  dict(m=28672, k=8192, b=64, x="bf16", y="bf16", scale_group=128, d=2, seed=5,
                  outliers=True),
    "mlp1":     dict(m=12288, k=49152, b=1,  x="f16", y="f16", scale_group=0, d=2, seed=11),
    "mlp2":     dict(m=49152, k=12288, b=1,  x="f16", y="f16", scale_group=0, d=2, seed=12),
    "mlp1_b16": dict(m=12288, k=49152, b=16, x="f16", y="f16", scale_group=0, d=2, seed=11),
    "mlp2_b16": dict(m=49152, k=12288, b=16, x="f16", y="f16", scale_group=0, d=2, seed=12),
    "mlp1_b64": dict(m=12288, k=49152, b=64, x="f16", y="f16", scale_group=0, d=2, seed=11),
    "mlp2_b64": dict(m=49152, k=12288, b=64, x="f16", y="f16", scale_group=0, d=2, seed=12),
    # 1.2 GB of codes: where the fixed costs of a launch no longer show (same recipe, seed 13)
    "big1":     dict(m=49152, k=49152, b=1,  x="f16", y="f16", scale_group=0, d=2, seed=13),
}
PAPER_SHAPES = {"mlp1": (12288, 49152), "mlp2": (49152, 12288)}

_STREAM_CODES, _STREAM_X, _STREAM_SCALES, _STREAM_OUTLIER = 1, 2, 3, 4


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(stream)])


def pack_nibbles(nib: np.ndarray) -> np.ndarray:
    """[m][k] array of 4-bit patterns (0..15) -> uint8 [m][k/2] in the layout above."""
    nib = np.asarray(nib)
    if nib.ndim != 2 or nib.shape[1] % 2:
        raise ValueError("need [m][k] with k even")
    if nib.min() < 0 or nib.max() > 15:
        raise ValueError("patterns must be 0..15")
    nib = nib.astype(np.uint8)
    return np.ascontiguousarray(nib[:, 0::2] | (nib[:, 1::2] << 4))


def make_codes(m: int, k: int, seed: int) -> np.ndarray:
    """i.i.d. uniform 4-bit patterns (values uniform over [-8,7]), packed."""
    if k % 2:
        raise ValueError("k must be even")
    return _rng(seed, _STREAM_CODES).integers(0, 256, size=(m, k // 2), dtype=np.uint8)


def make_codes8(m: int, k: int, seed: int) -> np.ndarray:
    """8-bit weight codes, uint8 [m][k], uniform over the bit patterns except the
    two that an E4M3 value map reads as NaN (0x7f, 0xff become 0x7e, 0xfe)."""
    c = _rng(seed, 5).integers(0, 256, size=(m, k), dtype=np.uint8)
    c[(c & 0x7f) == 0x7f] -= 1
    return c


def fp8_e4m3_values() -> np.ndarray:
    """The value of each 8-bit pattern in the OCP 8-bit floating point format
    E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities,
    S.1111.111 is NaN).  A value map is an input of the method, like the codes:
    this is the data format's definition, not arithmetic of the method."""
    v = np.empty(256, dtype=np.float64)
    for p in range(256):
        sign = -1.0 if p & 0x80 else 1.0
        e, f = (p >> 3) & 15, p & 7
        if e == 15 and f == 7:
            v[p] = np.nan
        elif e == 0:
            v[p] = sign * f * 2.0 ** -9
        else:
            v[p] = sign * (1.0 + f / 8.0) * 2.0 ** (e - 7)
    return v


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 bit patterns, nearest-even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def make_x(k: int, b: int, dtype: str, seed: int, outliers: bool = False) -> np.ndarray:
    """Activations [b][k].  Floats: N(0,1) drawn in fp64 then cast; with
    ``outliers`` each element is independently multiplied by 10 with probability
    0.01 before the cast.  int8: uniform over [-128,127]."""
    if dtype == "i8":
        return _rng(seed, _STREAM_X).integers(-128, 128, size=(b, k), dtype=np.int8)
    x = _rng(seed, _STREAM_X).standard_normal(size=(b, k))
    if outliers:
        hit = _rng(seed, _STREAM_OUTLIER).random(size=(b, k)) < 0.01
        x = np.where(hit, 10.0 * x, x)
    if dtype == "f32":
        return x.astype(np.float32)
    if dtype == "f16":
        return x.astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x.astype(np.float32))
    raise ValueError(dtype)


def make_scales(m: int, k: int, scale_group: int, seed: int) -> np.ndarray:
    """fp16 scales ~ U[0.005, 0.02], one per row per ``scale_group`` columns."""
    if scale_group <= 0 or k % scale_group:
        raise ValueError("k must be a multiple of scale_group")
    q = _rng(seed, _STREAM_SCALES).uniform(0.005, 0.02, size=(m, k // scale_group))
    return q.astype(np.float16)


def make_config(name: str, m: int | None = None):
    """All inputs of a named configuration; ``m`` overrides the row count (row
    subsets of the full problem for quick checks use the same generator)."""
    cfg = dict(CONFIGS[name])
    if m is not None:
        cfg["m"] = int(m)
    codes = make_codes(cfg["m"], cfg["k"], cfg["seed"])
    X = make_x(cfg["k"], cfg["b"], cfg["x"], cfg["seed"], cfg.get("outliers", False))
    scales = None
    if cfg["scale_group"]:
        scales = make_scales(cfg["m"], cfg["k"], cfg["scale_group"], cfg["seed"])
    return cfg, codes, X, scales


# --- the paper's running example (Sections 2, 3.1, 3.2): 12 x 4 x 1, d = 2 ----
# Row 0 is the one the text prints, M(0,:) = {2,4,3,5}, given there as the bit
# patterns 0010 0100 0011 0101.  The other rows and x were only in a figure that
# is not available, so they are filled in here: row 1 is all 1000 (the paper's
# pattern for -8), row 2 all 1111 (its pattern for -1), rows 3..11 seeded
# patterns; x takes small dyadic values so every sum is exact in any float type.
WORKED_EXAMPLE_ROW0_PATTERNS = (0b0010, 0b0100, 0b0011, 0b0101)
WORKED_EXAMPLE_X = (0.5, -1.25, 2.0, 0.75)


def make_worked_example():
    nib = _rng(12, _STREAM_CODES).integers(0, 16, size=(12, 4))
    nib[0, :] = WORKED_EXAMPLE_ROW0_PATTERNS
    nib[1, :] = 0b1000
    nib[2, :] = 0b1111
    x = np.asarray([WORKED_EXAMPLE_X], dtype=np.float32)
    return nib.astype(np.uint8), pack_nibbles(nib), x
