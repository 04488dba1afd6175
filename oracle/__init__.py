"""msGeMM CPU oracle -- TEST INFRASTRUCTURE ONLY.

Thin numpy front-end over ``msgemm_oracle.c`` (plain C, fp64 / int32), plus the
paper's operation-count formulas.  Only ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py`` may import this package; the HIP
product path never does and shares no code with it.

Every function names the passage of arxiv 2310.06178 it follows.  The bf16
output tolerance used by the tests is a reading of this build, not something
the paper fixes: parity unpinned for that tolerance only.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "msgemm_oracle.c")
_LIB = os.path.join(_HERE, "libmsgemm_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, dbl, vp, ci = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_int
        lib.msgemm_oracle_decode.argtypes = [ctypes.c_uint]
        lib.msgemm_oracle_decode.restype = ci
        lib.msgemm_oracle_encode.argtypes = [ci]
        lib.msgemm_oracle_encode.restype = ctypes.c_uint
        lib.msgemm_oracle_num_threads.restype = ci
        lib.msgemm_oracle_set_threads.argtypes = [ci]
        lib.msgemm_oracle_gemm_f64.argtypes = [i64, i64, i64, vp, vp, i64, vp, i64, vp, i64]
        lib.msgemm_oracle_gemm_f64_values.argtypes = [i64, i64, i64, vp, vp, vp, i64, vp, i64, vp, i64]
        lib.msgemm_oracle_gemm_f64_codes8.argtypes = [i64, i64, i64, vp, vp, vp, i64, vp, i64, vp, i64]
        lib.msgemm_oracle_lut_build_f64_values.argtypes = [i64, i64, ci, i64, vp, vp, i64, vp]
        lib.msgemm_oracle_gemm_i32.argtypes = [i64, i64, i64, vp, vp, i64, vp, i64]
        lib.msgemm_oracle_lut_groups.argtypes = [i64, ci, i64]
        lib.msgemm_oracle_lut_groups.restype = i64
        lib.msgemm_oracle_lut_build_f64.argtypes = [i64, i64, ci, i64, vp, i64, vp]
        lib.msgemm_oracle_lut_build_i32.argtypes = [i64, i64, ci, vp, i64, vp]
        lib.msgemm_oracle_lut_consume_f64.argtypes = [i64, i64, i64, ci, vp, vp, i64, vp, vp, i64]
        lib.msgemm_oracle_lut_consume_i32.argtypes = [i64, i64, i64, ci, vp, vp, vp, i64]
        lib.msgemm_oracle_f64_to_f16_bits.argtypes = [dbl]
        lib.msgemm_oracle_f64_to_f16_bits.restype = ctypes.c_uint16
        lib.msgemm_oracle_f64_to_bf16_bits.argtypes = [dbl]
        lib.msgemm_oracle_f64_to_bf16_bits.restype = ctypes.c_uint16
        lib.msgemm_oracle_round_f16.argtypes = [vp, vp, i64]
        lib.msgemm_oracle_round_bf16.argtypes = [vp, vp, i64]
        lib.msgemm_oracle_round_f32.argtypes = [vp, vp, i64]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle: {what} rejected its arguments (rc={rc})")


def num_threads() -> int:
    return int(_load().msgemm_oracle_num_threads())


def set_threads(n: int) -> None:
    _load().msgemm_oracle_set_threads(int(n))


def decode(nibble: int) -> int:
    """b(.) of Section 3.1: 4-bit pattern -> int4 value."""
    return int(_load().msgemm_oracle_decode(int(nibble)))


def encode(value: int) -> int:
    """b-hat(.) of Section 3.2: int4 value -> 4-bit pattern."""
    r = int(_load().msgemm_oracle_encode(int(value)))
    if r > 15:
        raise ValueError(f"{value} is not an int4 value")
    return r


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)


def f16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def _as_f64_cols(X) -> np.ndarray:
    X = np.asarray(X)
    if X.ndim == 1:
        X = X[None, :]
    return np.ascontiguousarray(X, dtype=np.float64)


def _values16(codebook):
    if codebook is None:
        return None
    v = np.ascontiguousarray(codebook, dtype=np.float64)
    if v.shape != (16,):
        raise ValueError("a codebook has 16 values, one per bit pattern")
    return v


def gemm_f64(codes, X, scales=None, scale_group: int = 0, codebook=None) -> np.ndarray:
    """Direct decode-and-multiply GeMM in fp64 (Section 3.2, first line of the
    y(i) equation; Section 3.3 for the per-block scales).  ``codebook``: 16
    values replacing b(.) of Section 3.1, indexed by bit pattern (None = the
    paper's two's complement).

    codes: uint8 [m][k/2]; X: [b][k] (each row one activation vector, i.e. one
    column of the paper's X); scales: [m][k/scale_group] or None.
    Returns Y as fp64 [b][m].
    """
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    X = _as_f64_cols(X)
    m, k = codes.shape[0], codes.shape[1] * 2
    b = X.shape[0]
    if X.shape[1] != k:
        raise ValueError("X must be [b][k]")
    s = None
    if scale_group:
        s = np.ascontiguousarray(scales, dtype=np.float64)
        if s.shape != (m, k // scale_group):
            raise ValueError("scales must be [m][k/scale_group]")
    Y = np.empty((b, m), dtype=np.float64)
    v = _values16(codebook)
    _check(_load().msgemm_oracle_gemm_f64_values(m, k, b, _ptr(codes), _ptr(v), _ptr(s), int(scale_group),
                                                 _ptr(X), k, _ptr(Y), m), "gemm_f64")
    return Y


def gemm_f64_codes8(codes8, X, values256, scales=None, scale_group: int = 0) -> np.ndarray:
    """The direct GeMM for 8-bit weights (Section 2 names an 8-bit floating-point
    weight matrix as another possible datatype): y = sum_j values256[code(i, j)] x(j),
    per-block scales as in Section 3.3.  codes8: uint8 [m][k]; values256: the
    value of each of the 256 bit patterns; X: [b][k].  Returns fp64 [b][m]."""
    codes8 = np.ascontiguousarray(codes8, dtype=np.uint8)
    X = _as_f64_cols(X)
    m, k = codes8.shape
    b = X.shape[0]
    if X.shape[1] != k:
        raise ValueError("X must be [b][k]")
    v = np.ascontiguousarray(values256, dtype=np.float64)
    if v.shape != (256,):
        raise ValueError("values256 has one value per 8-bit pattern")
    s = None
    if scale_group:
        s = np.ascontiguousarray(scales, dtype=np.float64)
        if s.shape != (m, k // scale_group):
            raise ValueError("scales must be [m][k/scale_group]")
    Y = np.empty((b, m), dtype=np.float64)
    _check(_load().msgemm_oracle_gemm_f64_codes8(m, k, b, _ptr(codes8), _ptr(v), _ptr(s), int(scale_group),
                                                 _ptr(X), k, _ptr(Y), m), "gemm_f64_codes8")
    return Y


def gemm_i32(codes, X) -> np.ndarray:
    """int8 activations, int32 accumulation (same definition, integer types)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    X = np.asarray(X)
    if X.dtype != np.int8:
        raise ValueError("X must be int8")
    if X.ndim == 1:
        X = X[None, :]
    X = np.ascontiguousarray(X)
    m, k = codes.shape[0], codes.shape[1] * 2
    b = X.shape[0]
    if X.shape[1] != k:
        raise ValueError("X must be [b][k]")
    Y = np.empty((b, m), dtype=np.int32)
    _check(_load().msgemm_oracle_gemm_i32(m, k, b, _ptr(codes), _ptr(X), k, _ptr(Y), m),
           "gemm_i32")
    return Y


def lut_groups(k: int, d: int, scale_group: int = 0) -> int:
    """Last dimension of L: k/d groups (Section 3.1), restarted per scale block."""
    g = int(_load().msgemm_oracle_lut_groups(int(k), int(d), int(scale_group)))
    if g < 0:
        raise ValueError("bad k / d / scale_group")
    return g


def lut_build(X, d: int, scale_group: int = 0, codebook=None) -> np.ndarray:
    """Phase 1 (Section 3.1): L[j][idx][c] = sum_r b(i_r) X(j d + r, c), with
    idx = sum_r i_r << 4r.  int8 X gives int32 entries, anything else fp64."""
    X = np.asarray(X)
    if X.ndim == 1:
        X = X[None, :]
    b, k = X.shape
    G = lut_groups(k, d, scale_group)
    E = 16 ** d
    if X.dtype == np.int8:
        if scale_group:
            raise ValueError("int8 path has no scales")
        X = np.ascontiguousarray(X)
        L = np.empty((G, E, b), dtype=np.int32)
        _check(_load().msgemm_oracle_lut_build_i32(k, b, d, _ptr(X), k, _ptr(L)), "lut_build_i32")
        return L
    X = _as_f64_cols(X)
    L = np.empty((G, E, b), dtype=np.float64)
    v = _values16(codebook)
    _check(_load().msgemm_oracle_lut_build_f64_values(k, b, d, int(scale_group), _ptr(v), _ptr(X), k, _ptr(L)),
           "lut_build_f64")
    return L


def lut_consume(codes, L, d: int, scales=None, scale_group: int = 0) -> np.ndarray:
    """Phase 2 (Section 3.2, second line of the y(i) equation): gather the table
    entry addressed by each row's d adjacent codes and add."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    m, k = codes.shape[0], codes.shape[1] * 2
    L = np.ascontiguousarray(L)
    G, E, b = L.shape
    if G != lut_groups(k, d, scale_group) or E != 16 ** d:
        raise ValueError("L has the wrong shape")
    if L.dtype == np.int32:
        Y = np.empty((b, m), dtype=np.int32)
        _check(_load().msgemm_oracle_lut_consume_i32(m, k, b, d, _ptr(codes), _ptr(L), _ptr(Y), m),
               "lut_consume_i32")
        return Y
    if L.dtype != np.float64:
        raise ValueError("L must be fp64 or int32")
    s = None
    if scale_group:
        s = np.ascontiguousarray(scales, dtype=np.float64)
    Y = np.empty((b, m), dtype=np.float64)
    _check(_load().msgemm_oracle_lut_consume_f64(m, k, b, d, _ptr(codes), _ptr(s), int(scale_group),
                                                 _ptr(L), _ptr(Y), m), "lut_consume_f64")
    return Y


def round_to(Y64: np.ndarray, dtype: str) -> np.ndarray:
    """One round-to-nearest-even from fp64 to the output type.  'f16' and
    'bf16' return uint16 bit patterns, 'f32' float32."""
    Y64 = np.ascontiguousarray(Y64, dtype=np.float64)
    lib = _load()
    if dtype == "f32":
        out = np.empty(Y64.shape, dtype=np.float32)
        lib.msgemm_oracle_round_f32(_ptr(Y64), _ptr(out), Y64.size)
    elif dtype == "f16":
        out = np.empty(Y64.shape, dtype=np.uint16)
        lib.msgemm_oracle_round_f16(_ptr(Y64), _ptr(out), Y64.size)
    elif dtype == "bf16":
        out = np.empty(Y64.shape, dtype=np.uint16)
        lib.msgemm_oracle_round_bf16(_ptr(Y64), _ptr(out), Y64.size)
    else:
        raise ValueError(dtype)
    return out


def rel_l2(y, y_ref) -> float:
    """||y - y_ref||_2 / ||y_ref||_2 over the whole output, in fp64."""
    y = np.asarray(y, dtype=np.float64).ravel()
    r = np.asarray(y_ref, dtype=np.float64).ravel()
    den = float(np.sqrt(np.sum(r * r)))
    num = float(np.sqrt(np.sum((y - r) ** 2)))
    return num / den if den > 0 else num


# --- the paper's cost model (Section 4, Section 4.2, Section 5) --------------

def ops_lut(k: int, d: int, b: int = 1) -> int:
    """C(L) = 16^d * k per activation vector (Section 4)."""
    return (16 ** d) * k * b


def ops_consume(m: int, k: int, d: int, b: int = 1):
    """C(y) = (k/d - 1) * m per activation vector (Section 4)."""
    return (k / d - 1) * m * b


def ops_msgemm(m: int, k: int, d: int, b: int = 1):
    """C(msGeMM) = (16^d k + (k/d - 1) m) b (Section 4.2)."""
    return ops_lut(k, d, b) + ops_consume(m, k, d, b)


def ops_naive(m: int, k: int, b: int = 1) -> int:
    """C(GeMM) = m k b (Section 4.2)."""
    return m * k * b


def mem_accesses(m: int, k: int, b: int = 1) -> int:
    """k b + m k elements, identical for both methods (Section 4.2)."""
    return k * b + m * k


def speedup(m: int, k: int, d: int) -> float:
    """C(GeMM) / C(msGeMM) (Section 5); independent of b."""
    return ops_naive(m, k) / ops_msgemm(m, k, d)
