"""Pins for the CPU oracle: everything here checks ``oracle/`` against something
other than itself -- values the paper prints, hand-worked numbers, closed forms,
brute force written out in Python, and library routines (numpy matmul / numpy
and torch conversions) applied to weights decoded with the paper's printed
value table.  No GPU needed."""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2310_06178_amd import inputs

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


# The value of each 4-bit pattern, from the golden file that restates Section 3.1.
PAPER_B = {int(r[0], 2): int(r[1]) for r in _read_golden("int4_value_map.txt")}
PAPER_B_ARR = np.array([PAPER_B[i] for i in range(16)], dtype=np.int64)


def unpack_independent(codes):
    """Test-side unpacking: byte t -> column 2t (low nibble), 2t+1 (high nibble)."""
    m, kb = codes.shape
    nib = np.empty((m, kb * 2), dtype=np.int64)
    for t in range(kb):
        nib[:, 2 * t] = codes[:, t] % 16
        nib[:, 2 * t + 1] = codes[:, t] // 16
    return nib


def decoded_weights(codes):
    return PAPER_B_ARR[unpack_independent(codes)]


# --------------------------------------------------------------------------
# b(.) and b-hat(.)

def test_value_map_matches_paper():
    assert len(PAPER_B) == 16
    for pattern, value in PAPER_B.items():
        assert oracle.decode(pattern) == value
        assert oracle.encode(value) == pattern
    # the pairs the paper prints verbatim
    assert oracle.decode(0b0000) == 0 and oracle.decode(0b0001) == 1
    assert oracle.decode(0b0111) == 7 and oracle.decode(0b1000) == -8
    assert oracle.decode(0b1111) == -1
    assert oracle.encode(-1) == 0b1111
    with pytest.raises(ValueError):
        oracle.encode(8)


# --------------------------------------------------------------------------
# the running example

def test_worked_example():
    g = {r[0]: r[1:] for r in _read_golden("worked_example_12x4x1.txt")}
    nib, codes, x = inputs.make_worked_example()
    assert codes.shape == (int(g["m"][0]), int(g["k"][0]) // 2)
    assert [int(p, 2) for p in g["row0_patterns"]] == list(nib[0])
    assert [PAPER_B[int(p, 2)] for p in g["row0_patterns"]] == [int(v) for v in g["row0_values"]]
    assert [float(v) for v in g["x"]] == list(x[0])
    d = int(g["d"][0])
    y = oracle.gemm_f64(codes, x)
    assert y.shape == (1, 12)
    assert y[0, 0] == float(g["y0"][0])
    L = oracle.lut_build(x, d)
    # "L has a size of 2^4 x 2^4 x 2" -- stored [group][16*16][b]
    assert L.shape == (int(g["lut_shape"][2]), int(g["lut_shape"][0]) * int(g["lut_shape"][1]), 1)
    # L(i0, i1, j) with i0 the first (least significant) digit
    e0 = L[0, 0b0010 | (0b0100 << 4), 0]
    e1 = L[1, 0b0011 | (0b0101 << 4), 0]
    assert e0 == float(g["L_0010_0100_0"][0])
    assert e1 == float(g["L_0011_0101_1"][0])
    assert e0 + e1 == float(g["y0"][0])
    y_lut = oracle.lut_consume(codes, L, d)
    assert np.array_equal(y_lut, y)
    # the filled-in rows: all 1000 -> -8 * sum(x); all 1111 -> -sum(x)
    sx = sum(float(v) for v in g["x"])
    assert y[0, 1] == -8 * sx and y[0, 2] == -sx


# --------------------------------------------------------------------------
# decode, nibble order, row stride, X / Y orientation: one-hot probes

def test_unit_vector_probe_all_codes():
    # 16 x 2 matrix: column 0 runs through all patterns, column 1 is reversed
    nib = np.stack([np.arange(16), np.arange(15, -1, -1)], axis=1)
    codes = inputs.pack_nibbles(nib)
    X = np.eye(2, dtype=np.float64)  # X[c] = e_c : b = 2 one-hot vectors
    Y = oracle.gemm_f64(codes, X)
    assert Y.shape == (2, 16)
    assert list(Y[0]) == [PAPER_B[i] for i in range(16)]
    assert list(Y[1]) == [PAPER_B[15 - i] for i in range(16)]
    Yi = oracle.gemm_i32(codes, np.eye(2, dtype=np.int8))
    assert list(Yi[0]) == [PAPER_B[i] for i in range(16)]
    assert list(Yi[1]) == [PAPER_B[15 - i] for i in range(16)]


def test_unit_vector_probe_random_matrix():
    m, k = 37, 24
    codes = inputs.make_codes(m, k, seed=11)
    W = decoded_weights(codes)
    X = np.eye(k, dtype=np.float64) * 3.0  # b = k probes
    Y = oracle.gemm_f64(codes, X)
    assert np.array_equal(Y, 3.0 * W.T)
    Yi = oracle.gemm_i32(codes, (np.eye(k) * -5).astype(np.int8))
    assert np.array_equal(Yi, -5 * W.T)


# --------------------------------------------------------------------------
# library cross-checks: the method reduces to a textbook matmul

@pytest.mark.parametrize("m,k,b", [(64, 48, 3), (130, 256, 16), (1, 2, 1), (257, 130, 5)])
def test_int_path_vs_numpy_int64_matmul(m, k, b):
    codes = inputs.make_codes(m, k, seed=m + k)
    X = inputs.make_x(k, b, "i8", seed=b)
    W = decoded_weights(codes)
    ref = (W @ X.astype(np.int64).T).T
    Y = oracle.gemm_i32(codes, X)
    assert Y.dtype == np.int32
    assert np.array_equal(Y.astype(np.int64), ref)


@pytest.mark.parametrize("m,k,b,sg", [(64, 48, 3, 0), (130, 256, 4, 128), (33, 384, 2, 128),
                                      (20, 64, 2, 64), (20, 64, 2, 2)])
def test_float_path_vs_numpy_fp64_matmul(m, k, b, sg):
    codes = inputs.make_codes(m, k, seed=7)
    X = inputs.make_x(k, b, "f16", seed=8).astype(np.float64)
    W = decoded_weights(codes).astype(np.float64)
    scales = None
    if sg:
        scales = inputs.make_scales(m, k, sg, seed=9)
        W = W * np.repeat(scales.astype(np.float64), sg, axis=1)
    ref = (W @ X.T).T
    Y = oracle.gemm_f64(codes, X, scales, sg)
    assert oracle.rel_l2(Y, ref) < 1e-13
    assert np.allclose(Y, ref, rtol=1e-11, atol=1e-11)


def test_x_and_y_orientation_not_transposed():
    # asymmetric everything: a transposed operand or swapped nibble order changes the result
    nib = np.array([[1, 2, 3, 4], [5, 6, 7, 8], [9, 10, 11, 12]])
    codes = inputs.pack_nibbles(nib)
    X = np.array([[1.0, 10.0, 100.0, 1000.0], [2.0, 0.0, 0.0, 0.0]])
    Y = oracle.gemm_f64(codes, X)
    w = [[PAPER_B[v] for v in row] for row in nib]
    for c in range(2):
        for i in range(3):
            assert Y[c, i] == sum(w[i][j] * X[c, j] for j in range(4))


# --------------------------------------------------------------------------
# closed forms

@pytest.mark.parametrize("pattern,factor", [(0b0001, 1), (0b1000, -8), (0b1111, -1), (0b0111, 7),
                                            (0b0000, 0)])
def test_constant_code_matrices(pattern, factor):
    m, k, b = 9, 40, 3
    codes = inputs.pack_nibbles(np.full((m, k), pattern))
    X = inputs.make_x(k, b, "f32", seed=3).astype(np.float64)
    Y = oracle.gemm_f64(codes, X)
    for c in range(b):
        # same summation order as a plain left-to-right sum of x scaled exactly
        s = 0.0
        for j in range(k):
            s += factor * X[c, j]
        assert np.all(Y[c] == s)
    Xi = inputs.make_x(k, b, "i8", seed=4)
    Yi = oracle.gemm_i32(codes, Xi)
    for c in range(b):
        assert np.all(Yi[c] == factor * int(Xi[c].astype(np.int64).sum()))


def test_ones_activation_gives_row_sums():
    m, k = 50, 64
    codes = inputs.make_codes(m, k, seed=21)
    W = decoded_weights(codes)
    Y = oracle.gemm_i32(codes, np.ones((1, k), dtype=np.int8))
    assert np.array_equal(Y[0], W.sum(axis=1))


def test_int_linearity():
    m, k = 40, 96
    codes = inputs.make_codes(m, k, seed=5)
    rng = np.random.default_rng(6)
    x1 = rng.integers(-60, 60, size=(2, k), dtype=np.int8)
    x2 = rng.integers(-60, 60, size=(2, k), dtype=np.int8)
    y12 = oracle.gemm_i32(codes, (x1 + x2).astype(np.int8))
    assert np.array_equal(y12, oracle.gemm_i32(codes, x1) + oracle.gemm_i32(codes, x2))


# --------------------------------------------------------------------------
# scales (Section 3.3)

def test_scale_invariants():
    m, k, b, sg = 24, 256, 3, 128
    codes = inputs.make_codes(m, k, seed=31)
    X = inputs.make_x(k, b, "f16", seed=32).astype(np.float64)
    ones = np.ones((m, k // sg), dtype=np.float16)
    y_plain = oracle.gemm_f64(codes, X)
    # q == 1 : per-block sums added block by block; equal to the plain sum up to
    # the regrouping of the additions
    y_ones = oracle.gemm_f64(codes, X, ones, sg)
    assert np.allclose(y_ones, y_plain, rtol=1e-13, atol=1e-12)
    q = inputs.make_scales(m, k, sg, seed=33)
    y_q = oracle.gemm_f64(codes, X, q, sg)
    y_2q = oracle.gemm_f64(codes, X, (2 * q.astype(np.float64)), sg)
    assert np.array_equal(y_2q, 2 * y_q)  # doubling is exact in binary floating point
    # one scale per row (scale_group = k) is the per-row q(i) of Section 3.3
    q_row = inputs.make_scales(m, k, k, seed=34)
    y_row = oracle.gemm_f64(codes, X, q_row, k)
    assert np.array_equal(y_row, y_plain * q_row.astype(np.float64).T)
    # a scale confined to block 1 only touches block 1's columns
    q01 = np.zeros((m, 2)); q01[:, 1] = 1.0
    X0 = X.copy(); X0[:, :sg] = 0.0
    assert np.array_equal(oracle.gemm_f64(codes, X, q01, sg), oracle.gemm_f64(codes, X0))


# --------------------------------------------------------------------------
# the LUT itself (Section 3.1), by brute force over every code combination

@pytest.mark.parametrize("d", [1, 2, 3, 4])
def test_lut_enumeration_brute_force(d):
    x = [0.5, -1.25, 2.0, 0.75][:d]
    L = oracle.lut_build(np.array([x]), d)
    assert L.shape == (1, 16 ** d, 1)
    for digits in itertools.product(range(16), repeat=d):
        idx = sum(digits[r] << (4 * r) for r in range(d))
        expect = 0.0
        for r in range(d):
            expect += PAPER_B[digits[r]] * x[r]
        assert L[0, idx, 0] == expect
    # enumeration matrix: k = d, m = 16^d, row i carries the digits of i, so
    # y(i) must be table entry i -- through the direct path, which builds no table
    nib = np.array([[(i >> (4 * r)) & 15 for r in range(d)] + [0] * (d % 2)
                    for i in range(16 ** d)])
    xk = np.array([x + [0.0] * (d % 2)])
    y = oracle.gemm_f64(inputs.pack_nibbles(nib), xk)
    assert np.array_equal(y[0], L[0, :, 0])


@pytest.mark.parametrize("d", [1, 2, 3])
def test_lut_enumeration_int(d):
    x = np.array([[-128, 127, 77][:d]], dtype=np.int8)
    xk = np.concatenate([x, np.zeros((1, d % 2), dtype=np.int8)], axis=1)
    L = oracle.lut_build(xk[:, :d] if d % 2 == 0 else xk, d)
    for digits in itertools.product(range(16), repeat=d):
        idx = sum(digits[r] << (4 * r) for r in range(d))
        assert L[0, idx, 0] == sum(PAPER_B[digits[r]] * int(x[0, r]) for r in range(d))


def test_lut_shape_and_groups():
    # 16^d * k/d entries (Section 4); short last group when d does not divide k
    assert oracle.lut_groups(4, 2) == 2
    assert oracle.lut_groups(4096, 3) == 1366
    assert oracle.lut_groups(4096, 2, 128) == 2048
    assert oracle.lut_groups(256, 3, 128) == 2 * 43  # groups restart per scale block
    assert oracle.lut_build(np.zeros((5, 12)), 3).shape == (4, 4096, 5)
    with pytest.raises(ValueError):
        oracle.lut_groups(8, 5)


# --------------------------------------------------------------------------
# LUT formulation == direct sum (Section 3.2, the two lines of the y(i) equation)

@pytest.mark.parametrize("d", [1, 2, 3, 4])
@pytest.mark.parametrize("m,k,b,sg", [(19, 48, 2, 0), (7, 10, 1, 0), (33, 256, 3, 128),
                                      (5, 26, 2, 0), (12, 64, 2, 16)])
def test_lut_equals_direct_float(d, m, k, b, sg):
    if d == 4 and k > 64:
        pytest.skip("table of 16^4 entries per group: kept to small k")
    codes = inputs.make_codes(m, k, seed=100 + d)
    X = inputs.make_x(k, b, "f32", seed=200 + d).astype(np.float64)
    scales = inputs.make_scales(m, k, sg, seed=300) if sg else None
    direct = oracle.gemm_f64(codes, X, scales, sg)
    L = oracle.lut_build(X, d, sg)
    via_lut = oracle.lut_consume(codes, L, d, scales, sg)
    assert np.allclose(via_lut, direct, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("d", [1, 2, 3, 4])
@pytest.mark.parametrize("m,k,b", [(19, 48, 2), (7, 10, 1), (40, 62, 3)])
def test_lut_equals_direct_int_and_d_invariance(d, m, k, b):
    codes = inputs.make_codes(m, k, seed=400)
    X = inputs.make_x(k, b, "i8", seed=401)
    direct = oracle.gemm_i32(codes, X)
    via_lut = oracle.lut_consume(codes, oracle.lut_build(X, d), d)
    assert np.array_equal(via_lut, direct)  # identical for every d, incl. d = 1


# --------------------------------------------------------------------------
# cost model (Sections 4, 4.2, 5)

def test_speedup_closed_forms():
    for name, d, value in _read_golden("mlp_speedup_closed_forms.txt"):
        m, k = inputs.PAPER_SHAPES[name]
        assert abs(oracle.speedup(m, k, int(d)) - float(value)) < 1e-6


def test_cost_model_identities():
    m, k, b = 12288, 49152, 7
    for d in (1, 2, 3, 4):
        assert oracle.ops_lut(k, d) == 2 ** (4 * d) * k
        assert oracle.ops_msgemm(m, k, d, b) == b * (2 ** (4 * d) * k + (k / d - 1) * m)
    assert oracle.ops_naive(m, k, b) == m * k * b
    assert oracle.mem_accesses(m, k, b) == k * b + m * k


def test_mem_accesses_on_the_worked_example():
    """Section 4.2 counts k*b elements of X plus m*k elements of M for either method.  On the paper's
    running example (m = 12, k = 4, b = 1) that is the 4 activations and the 48 codes: 52, counted by hand;
    swapping m and k, or dropping the X term, gives another number."""
    assert oracle.mem_accesses(12, 4, 1) == 52
    assert oracle.mem_accesses(12, 4, 3) == 60      # two more activation vectors: 8 more elements
    assert oracle.mem_accesses(4, 12, 1) == 60      # not symmetric in m and k


def test_ops_on_the_worked_example():
    """Section 4 on the running example at d = 2: the table has 16^2 entries for each of the k/d = 2 groups,
    each built from d = 2 products (512 entries, 16^d * k = 1024 operations as the paper counts them), and a row
    adds k/d - 1 = 1 time: 12 additions."""
    assert oracle.ops_lut(4, 2) == 1024
    assert oracle.ops_consume(12, 4, 2) == 12
    assert oracle.ops_naive(12, 4) == 48


# --------------------------------------------------------------------------
# the error measure of every floating-point parity assertion

def test_rel_l2_hand_worked():
    """||y - ref|| / ||ref|| on vectors small enough to do by hand: y = (3, 4), ref = (0, 5): the difference is
    (3, -1), its norm sqrt(10), the reference's norm 5.  A wrong denominator (||y|| is also 5 here, so a second
    case tells them apart), a missing square root or a sum of absolute values all give other numbers."""
    assert abs(oracle.rel_l2([3.0, 4.0], [0.0, 5.0]) - np.sqrt(10.0) / 5.0) < 1e-15
    # ||y|| = 10, ||ref|| = 5, difference (6, 3): sqrt(45) / 5 = 3 / sqrt(5)
    assert abs(oracle.rel_l2([6.0, 8.0], [0.0, 5.0]) - 3.0 / np.sqrt(5.0)) < 1e-15
    assert oracle.rel_l2([1.0, 2.0, 3.0], [1.0, 2.0, 3.0]) == 0.0
    # the whole output counts as one vector, whatever its shape
    assert abs(oracle.rel_l2(np.array([[3.0], [4.0]]), np.array([[0.0], [5.0]])) - np.sqrt(10.0) / 5.0) < 1e-15
    # a zero reference: the absolute error (nothing to divide by)
    assert oracle.rel_l2([3.0, 4.0], [0.0, 0.0]) == 5.0
    # not symmetric: the reference is the second argument
    assert abs(oracle.rel_l2([0.0, 5.0], [3.0, 4.0]) - np.sqrt(10.0) / 5.0) < 1e-15
    assert abs(oracle.rel_l2([0.0, 10.0], [3.0, 4.0]) - np.sqrt(45.0) / 5.0) < 1e-15
    # fp32 inputs are widened, not compared in fp32: 1 + 2^-30 is not 1
    assert oracle.rel_l2(np.array([1.0 + 2.0 ** -30]), np.array([1.0], dtype=np.float32)) == 2.0 ** -30


# --------------------------------------------------------------------------
# output rounding: against numpy (fp16) and torch (bf16) conversions

def test_round_f16_exhaustive_values_and_ties():
    h = np.arange(0x0000, 0x7C00, dtype=np.uint16)  # all finite non-negative halves
    v = h.view(np.float16).astype(np.float64)
    assert np.array_equal(oracle.round_to(v, "f16"), h)
    assert np.array_equal(oracle.round_to(-v, "f16"), h | 0x8000)
    mid = (v[:-1] + v[1:]) / 2  # exact ties: must go to the even neighbour
    even = np.where(h[:-1] % 2 == 0, h[:-1], h[1:])
    assert np.array_equal(oracle.round_to(mid, "f16"), even)
    assert np.array_equal(oracle.round_to(np.nextafter(mid, np.inf), "f16"), h[1:])
    assert np.array_equal(oracle.round_to(np.nextafter(mid, -np.inf), "f16"), h[:-1])
    # numpy's own double -> half conversion agrees on all of the above and on noise
    rng = np.random.default_rng(0)
    noise = rng.standard_normal(200000) * np.exp(rng.uniform(-20, 12, 200000))
    with np.errstate(over="ignore"):
        for arr in (mid, noise):
            assert np.array_equal(oracle.round_to(arr, "f16"), arr.astype(np.float16).view(np.uint16))
    assert list(oracle.round_to(np.array([65519.9, 65520.0, 1e9, -1e9, np.inf]), "f16")) == \
        [0x7BFF, 0x7C00, 0x7C00, 0xFC00, 0x7C00]


def test_round_bf16_vs_torch_and_ties():
    rng = np.random.default_rng(1)
    f = (rng.standard_normal(300000) * np.exp(rng.uniform(-60, 60, 300000))).astype(np.float32)
    want = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.round_to(f.astype(np.float64), "bf16"), want)
    # ties and their neighbours, built from consecutive bf16 values
    hb = np.arange(0x0001, 0x7F7F, 97, dtype=np.uint16)
    lo = oracle.bf16_bits_to_f64(hb)
    hi = oracle.bf16_bits_to_f64(hb + 1)
    mid = (lo + hi) / 2
    even = np.where(hb % 2 == 0, hb, hb + 1)
    assert np.array_equal(oracle.round_to(mid, "bf16"), even)
    # a double just above a tie must round up even though float(mid+eps) == mid
    assert np.array_equal(oracle.round_to(np.nextafter(mid, np.inf), "bf16"), hb + 1)
    assert np.array_equal(oracle.round_to(np.nextafter(mid, -np.inf), "bf16"), hb)
    assert np.array_equal(oracle.round_to(lo, "bf16"), hb)


def test_round_f32_is_numpy_cast():
    rng = np.random.default_rng(2)
    v = rng.standard_normal(10000) * 1e3
    assert np.array_equal(oracle.round_to(v, "f32"), v.astype(np.float32))


# --------------------------------------------------------------------------
# the input generators hand out what the configs say

def test_generators_are_seeded_and_shaped():
    cfg, codes, X, scales = inputs.make_config("cfg3a", m=64)
    cfg2, codes2, X2, scales2 = inputs.make_config("cfg3a", m=64)
    assert np.array_equal(codes, codes2) and np.array_equal(X, X2) and np.array_equal(scales, scales2)
    assert codes.shape == (64, 2048) and X.shape == (8, 4096) and X.dtype == np.float16
    assert scales.shape == (64, 32) and scales.dtype == np.float16
    assert 0.00499 < float(scales.min()) and float(scales.max()) < 0.02001  # fp16-rounded ends
    nib = unpack_independent(inputs.make_codes(256, 256, seed=0))
    counts = np.bincount(nib.ravel(), minlength=16)
    assert counts.min() > 0.9 * nib.size / 16 and counts.max() < 1.1 * nib.size / 16
    xb = inputs.make_x(4096, 64, "bf16", seed=5, outliers=True)
    assert xb.dtype == np.uint16
    xf = oracle.bf16_bits_to_f64(xb)
    assert 1.0 < xf.std() < 1.8  # N(0,1) plus 1 % of x10 outliers: var = 0.99 + 0.01*100
    xi = inputs.make_x(8192, 16, "i8", seed=4)
    assert xi.min() == -128 and xi.max() == 127


# --------------------------------------------------------------------------
# other 16-value encodings of the codes: only b(.) changes (Sections 2 and 3.1)

UINT4 = np.arange(16, dtype=np.float64)
# a made-up non-uniform, asymmetric table (dyadic values: every product below is exact)
NONUNIFORM = np.array([0.0, 0.125, 0.25, 0.5, 1.0, 1.5, 2.5, 4.0,
                       -6.0, -3.0, -2.0, -1.25, -0.75, -0.375, -0.1875, -0.0625])


def test_codebook_default_is_the_papers_b():
    codes = inputs.make_codes(33, 40, seed=21)
    X = inputs.make_x(40, 3, "f32", seed=22)
    sc = inputs.make_scales(33, 40, 8, seed=23)
    paper = PAPER_B_ARR.astype(np.float64)
    assert np.array_equal(oracle.gemm_f64(codes, X, sc, 8), oracle.gemm_f64(codes, X, sc, 8, codebook=paper))
    assert np.array_equal(oracle.lut_build(X, 3, 8), oracle.lut_build(X, 3, 8, codebook=paper))


@pytest.mark.parametrize("table", [UINT4, NONUNIFORM])
def test_codebook_unit_vector_probe(table):
    nib = np.stack([np.arange(16), np.arange(15, -1, -1)], axis=1)
    Y = oracle.gemm_f64(inputs.pack_nibbles(nib), np.eye(2), codebook=table)
    assert list(Y[0]) == list(table) and list(Y[1]) == list(table[::-1])


@pytest.mark.parametrize("table", [UINT4, NONUNIFORM])
def test_codebook_vs_numpy_matmul(table):
    m, k, b, sg = 70, 96, 4, 32
    codes = inputs.make_codes(m, k, seed=31)
    X = inputs.make_x(k, b, "f32", seed=32).astype(np.float64)
    sc = inputs.make_scales(m, k, sg, seed=33).astype(np.float64)
    W = table[unpack_independent(codes)] * np.repeat(sc, sg, axis=1)  # independently decoded and scaled
    ref = X @ W.T
    got = oracle.gemm_f64(codes, X, sc, sg, codebook=table)
    assert np.max(np.abs(got - ref)) <= 1e-12 * np.max(np.abs(ref))


def test_uint4_differs_from_twos_complement_by_sixteen_on_high_patterns():
    # pattern p as unsigned is p, as two's complement p - 16 [p >= 8]
    m, k = 50, 64
    codes = inputs.make_codes(m, k, seed=41)
    x = np.round(inputs.make_x(k, 1, "f32", seed=42).astype(np.float64) * 8) / 8  # dyadic: exact sums
    high = (unpack_independent(codes) >= 8).astype(np.float64)
    diff = oracle.gemm_f64(codes, x, codebook=UINT4) - oracle.gemm_f64(codes, x)
    assert np.array_equal(diff, 16.0 * (x @ high.T))


@pytest.mark.parametrize("d", [1, 2, 3])
def test_codebook_lut_enumeration(d):
    x = [0.5, -1.25, 2.0][:d]
    L = oracle.lut_build(np.array([x]), d, codebook=NONUNIFORM)
    for digits in itertools.product(range(16), repeat=d):
        idx = sum(digits[r] << (4 * r) for r in range(d))
        assert L[0, idx, 0] == sum(NONUNIFORM[digits[r]] * x[r] for r in range(d))
    # consuming that table equals the direct sum with the same value map
    codes = inputs.make_codes(19, 12, seed=51)
    X = np.array([[0.5, -1.25, 2.0, 0.75, -0.5, 1.5, 0.25, -2.0, 1.0, 3.0, -0.125, 0.375]])
    direct = oracle.gemm_f64(codes, X, codebook=NONUNIFORM)
    via = oracle.lut_consume(codes, oracle.lut_build(X, d, codebook=NONUNIFORM), d)
    assert np.array_equal(direct, via)


# ---------------------------------------------------------------------------
# the linearity remark of Section 4.1 as an invariant of the oracle's tables

@pytest.mark.parametrize("d", [1, 2, 3])
def test_table_of_complemented_codes_follows_from_the_other_half(d):
    """Two's complement has b(~i) = -1 - b(i), so complementing every code of an
    index gives L(~idx, j) = -S(j) - L(idx, j) with S(j) the sum of the group's
    activations; S(j) itself is the entry whose codes are all 0001 (b = 1).  A
    dropped term or a wrong sign in the table builder breaks this for some idx."""
    k, b = 12 * d, 2
    X = inputs.make_x(k, b, "f32", seed=40 + d).astype(np.float64)
    L = oracle.lut_build(X, d)
    E = 16 ** d
    ones = sum(1 << (4 * r) for r in range(d))
    S = L[:, ones, :]
    assert np.allclose(S, X.reshape(b, k // d, d).sum(axis=2).T, rtol=0, atol=1e-12)
    idx = np.arange(E)
    assert np.allclose(L[:, (~idx) & (E - 1), :], -S[:, None, :] - L[:, idx, :], rtol=0, atol=1e-9)
    # an unsigned map (value = pattern) has value(~i) = 15 - value(i)
    Lu = oracle.lut_build(X, d, codebook=np.arange(16, dtype=np.float64))
    assert np.allclose(Lu[:, (~idx) & (E - 1), :], 15.0 * S[:, None, :] - Lu[:, idx, :], rtol=0, atol=1e-9)


# ---------------------------------------------------------------------------
# 8-bit weights: one code byte per element, a 256-entry value map (Section 2)

def test_e4m3_value_map_against_the_format_definition():
    v = inputs.fp8_e4m3_values()
    assert v[0x00] == 0.0 and v[0x80] == 0.0 and np.signbit(v[0x80])
    assert v[0x38] == 1.0 and v[0xb8] == -1.0 and v[0x40] == 2.0 and v[0x3c] == 1.5
    assert v[0x01] == 2.0 ** -9 and v[0x07] == 7 * 2.0 ** -9 and v[0x08] == 2.0 ** -6   # subnormals, smallest normal
    assert v[0x7e] == 448.0 and v[0xfe] == -448.0                                        # largest finite
    assert np.isnan(v[0x7f]) and np.isnan(v[0xff]) and np.isfinite(np.delete(v, [0x7f, 0xff])).all()
    assert np.all(np.diff(v[:0x7f]) > 0)                                                  # monotone in the pattern
    codes = inputs.make_codes8(64, 96, seed=3)
    assert codes.dtype == np.uint8 and not np.any((codes & 0x7f) == 0x7f)


def test_codes8_gemm_against_library_matmul_and_probes():
    m, k, b, sg = 37, 96, 3, 32
    codes = inputs.make_codes8(m, k, seed=4)
    X = inputs.make_x(k, b, "f32", seed=5).astype(np.float64)
    v = inputs.fp8_e4m3_values()
    S = inputs.make_scales(m, k, sg, seed=6).astype(np.float64)
    W = v[codes]
    # dequantise, then a library matmul (blocks scaled one by one)
    want = np.zeros((b, m))
    for g in range(k // sg):
        want += (W[:, g * sg:(g + 1) * sg] @ X[:, g * sg:(g + 1) * sg].T).T * S[:, g][None, :]
    got = oracle.gemm_f64_codes8(codes, X, v, S, sg)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-12)
    # a unit vector reads one column of the dequantised matrix back
    for j in (0, 31, 95):
        e = np.zeros((1, k)); e[0, j] = 1.0
        assert np.array_equal(oracle.gemm_f64_codes8(codes, e, v)[0], W[:, j])
    # value = pattern: plain integer arithmetic
    ints = oracle.gemm_f64_codes8(codes, np.round(X * 8), np.arange(256.0))
    assert np.array_equal(ints, (codes.astype(np.int64) @ np.round(X * 8).astype(np.int64).T).T.astype(np.float64))
    # a transposed operand, a dropped block or an index off by one changes the result
    assert not np.allclose(got, oracle.gemm_f64_codes8(codes[:, ::-1].copy(), X, v, S, sg))
