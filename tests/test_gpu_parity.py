"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.

Bars (written out here): int8 -> int32 bit-exact; relative L2 error over the
whole output <= 1e-5 for fp32, <= 2e-3 for fp16 output, <= 1.6e-2 for bf16
output (the bf16 figure is this build's reading: 8x the fp16 bound for an 8x
coarser output format; the paper fixes no tolerance)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_06178_amd import binding as B
from paper_2310_06178_amd import inputs, torch_io

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 1.6e-2}
Y_OF_X = {"f32": "f32", "f16": "f16", "bf16": "bf16", "i8": "i32"}


def x_to_f64(X, xd):
    if xd == "bf16":
        return oracle.bf16_bits_to_f64(X)
    return X.astype(np.float64)


def oracle_y(codes, X, xd, scales, sg):
    if xd == "i8":
        return oracle.gemm_i32(codes, X)
    return oracle.gemm_f64(codes, x_to_f64(X, xd), scales, sg)


U_OUT = {"f32": 2.0 ** -24, "f16": 2.0 ** -11, "bf16": 2.0 ** -8}   # half an ulp of the output type, relative
ABS_FLOOR = {"f32": 2.0 ** -149, "f16": 2.0 ** -24, "bf16": 2.0 ** -133}     # one subnormal step of the output type
ABS_B = [float(abs(oracle.decode(i))) for i in range(16)]              # |b(.)| of Section 3.1


def elem_bound(codes, X, xd, scales, sg, table16=False, codebook=None, values256=None):
    """Per-output bound on |y_gpu - y_oracle| apart from the output rounding, from the arithmetic of the
    HIP path: S(i,c) = sum_j |q(i, block of j)| |w(i,j)| |x(j,c)| (the oracle's direct sum, Section 3.2 first
    line, fed with magnitudes) times
      * n * 2^-24 for at most n = k + 64 fp32 additions / scale multiplications per output in any order, plus
      * the rounding of a table entry: 2^-22 for fp32 entries (at most four roundings of 2^-24 at d = 4),
        2^-9 for fp16 entries (value map, product and sum each rounded to fp16: 3 * 2^-11, rounded up).
    A rigorous bound, so a correct kernel cannot fail it; an output with a wrong or missing term does as soon
    as that term exceeds it."""
    if xd == "i8":
        return None
    Xa = np.abs(x_to_f64(X, xd))
    sa = None if scales is None else np.abs(scales.astype(np.float64))
    if values256 is not None:
        S = oracle.gemm_f64_codes8(codes, Xa, np.abs(np.asarray(values256, dtype=np.float64)), sa, sg)
        k = codes.shape[1]
    else:
        cb = ABS_B if codebook is None else [abs(float(v)) for v in codebook]
        S = oracle.gemm_f64(codes, Xa, sa, sg, codebook=cb)
        k = codes.shape[1] * 2
    return ((k + 64) * 2.0 ** -24 + (2.0 ** -9 if table16 else 2.0 ** -22)) * 1.01 * S


def check(y_gpu_host, y_ref, xd, what="", bound=None):
    """int8: bit-exact.  Floats: the relative L2 error over the whole output within TOL, every element finite,
    and every element within half an ulp of the output type plus `bound` (elem_bound) of the oracle's value."""
    if xd == "i8":
        assert y_gpu_host.dtype == np.int32
        assert np.array_equal(y_gpu_host, y_ref), f"{what}: int32 result differs"
        return 0.0
    y = torch_io.to_f64(y_gpu_host)
    assert np.all(np.isfinite(y)), f"{what}: non-finite output"
    err = oracle.rel_l2(y, y_ref)
    assert err <= TOL[xd], f"{what}: rel L2 {err:.3e} > {TOL[xd]:.1e}"
    assert bound is not None, f"{what}: floating-point comparison without a per-element bound"
    tol = U_OUT[xd] * 1.01 * np.abs(y_ref) + bound + ABS_FLOOR[xd]
    excess = np.abs(y - y_ref) / tol
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 1.0, (f"{what}: element {worst} is off by {abs(y[worst] - y_ref[worst]):.3e}, "
                                  f"{excess[worst]:.2f}x its bound ({np.count_nonzero(excess > 1.0)} elements over)")
    return err


def run_gpu(codes, X, xd, scales, sg, d, variant, ldx_pad=0, ldy_pad=0, use_phases=False, options=None):
    m, k = codes.shape[0], codes.shape[1] * 2
    b = X.shape[0]
    yd = Y_OF_X[xd]
    if ldx_pad:
        Xp = np.zeros((b, k + ldx_pad), dtype=X.dtype)
        Xp[:, :k] = X
        # poison the padding: it must never be read into the result
        Xp[:, k:] = 77 if xd != "bf16" else 0x4300
        X = Xp
    dX = torch_io.to_device(X, xd)
    dC = torch_io.to_device(codes, "codes")
    dS = torch_io.to_device(scales, "scales")
    plan = B.msgemm_plan(m, k, b, xd, yd, d, sg, dC, dS, variant, options=options)
    try:
        info = B.msgemm_plan_get_info(plan)
        Y = torch_io.empty_output(b, m, yd, ldy=m + ldy_pad)
        Y.fill_(-3)
        if use_phases:
            L = torch.empty(B.msgemm_lut_bytes(plan) // 4, dtype=torch.int32, device="cuda:0")
            B.msgemm_build_lut(plan, dX, k + ldx_pad, L)
            B.msgemm_consume_lut(plan, L, Y, m + ldy_pad)
        else:
            B.msgemm_run(plan, dX, k + ldx_pad, Y, m + ldy_pad)
        torch.cuda.synchronize()
        out = torch_io.to_host(Y)
    finally:
        B.msgemm_destroy(plan)
    if ldy_pad:
        pad = out[:, m:]
        if out.dtype == np.uint16:
            assert np.all(pad == torch_io.to_host(torch.full((1,), -3, dtype=torch.bfloat16))[0])
        else:
            assert np.all(pad == -3), "output padding was written"
        out = np.ascontiguousarray(out[:, :m])
    return out, info


# ---------------------------------------------------------------------------
# two-launch variant: every d, dtype, ragged shapes, scale block sizes

SMALL = [
    # m, k, b, xd, sg
    (12, 4, 1, "f32", 0),
    (300, 520, 3, "f32", 0),
    (257, 384, 5, "f16", 128),
    (64, 256, 2, "bf16", 64),
    (131, 130, 4, "i8", 0),
    (40, 64, 2, "f16", 16),
    (1, 2, 1, "f32", 0),
    (70, 132, 16, "f16", 0),
    (33, 96, 35, "f32", 32),
]


@pytest.mark.parametrize("d", [1, 2, 3, 4])
@pytest.mark.parametrize("m,k,b,xd,sg", SMALL)
def test_global_lut_variant_small(m, k, b, xd, sg, d):
    if d == 4 and k > 400:
        pytest.skip("16^4 entries per group: keep k small")
    codes = inputs.make_codes(m, k, seed=m * 7 + k)
    X = inputs.make_x(k, b, xd, seed=k + b)
    scales = inputs.make_scales(m, k, sg, seed=5) if sg else None
    ref = oracle_y(codes, X, xd, scales, sg)
    out, info = run_gpu(codes, X, xd, scales, sg, d, B.VARIANT_GLOBAL_LUT, ldx_pad=6, ldy_pad=3)
    assert info["variant"] == B.VARIANT_GLOBAL_LUT and info["d"] == d
    check(out, ref, xd, f"global d={d}", elem_bound(codes, X, xd, scales, sg))
    out2, _ = run_gpu(codes, X, xd, scales, sg, d, B.VARIANT_GLOBAL_LUT, use_phases=True)
    assert np.array_equal(out2, out), "phases called separately differ from msgemm_run"


def test_worked_example_on_gpu():
    _, codes, x = inputs.make_worked_example()
    ref = oracle.gemm_f64(codes, x)
    for variant in (B.VARIANT_GLOBAL_LUT, B.VARIANT_AUTO):
        out, _ = run_gpu(codes, x, "f32", None, 0, 2, variant)
        assert np.array_equal(out.astype(np.float64), ref)  # dyadic inputs: exact
        assert out[0, 0] == 5.75


@pytest.mark.parametrize("b", [3, 16, 40])  # from 16 columns on the floating-point tables are built on the matrix cores
@pytest.mark.parametrize("d", [1, 2, 3])
@pytest.mark.parametrize("xd,sg", [("f32", 0), ("f16", 128), ("i8", 0), ("bf16", 0)])
def test_build_lut_matches_phase1_reference(xd, sg, d, b):
    m, k = 8, 256
    codes = inputs.make_codes(m, k, seed=1)
    X = inputs.make_x(k, b, xd, seed=2)
    scales = inputs.make_scales(m, k, sg, seed=3) if sg else None
    dC, dS = torch_io.to_device(codes, "codes"), torch_io.to_device(scales, "scales")
    dX = torch_io.to_device(X, xd)
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], d, sg, dC, dS, B.VARIANT_GLOBAL_LUT)
    try:
        info = B.msgemm_plan_get_info(plan)
        G = oracle.lut_groups(k, d, sg)
        assert info["lut_groups"] == G
        assert B.msgemm_lut_bytes(plan) == G * 16 ** d * b * 4
        if xd == "i8":
            L = torch.empty((G, 16 ** d, b), dtype=torch.int32, device="cuda:0")
        else:
            L = torch.empty((G, 16 ** d, b), dtype=torch.float32, device="cuda:0")
        B.msgemm_build_lut(plan, dX, k, L)
        torch.cuda.synchronize()
        Lh = L.cpu().numpy()
    finally:
        B.msgemm_destroy(plan)
    if xd == "i8":
        assert np.array_equal(Lh, oracle.lut_build(X, d))
    else:
        ref = oracle.lut_build(x_to_f64(X, xd), d, sg)
        # each entry is at most d roundings away from the exact value
        scale = np.abs(ref).max()
        assert np.max(np.abs(Lh.astype(np.float64) - ref)) <= d * 2.0 ** -23 * scale
        if xd != "f32" and d <= 2:
            # fp16/bf16 inputs: products exact, one rounding of the sum
            assert np.array_equal(Lh, ref.astype(np.float32))


@pytest.mark.parametrize("xd,b,half", [("f16", 20, 0), ("f32", 16, 1), ("bf16", 3, 0)])
def test_build_lut_depth_four(xd, b, half):
    """d = 4: 65536 combinations per group (k = 18: four full groups and one of two columns), plain and
    matrix-core builders, full and half tables."""
    m, k, d = 8, 18, 4
    codes = inputs.make_codes(m, k, seed=1)
    X = inputs.make_x(k, b, xd, seed=2)
    dX = torch_io.to_device(X, xd)
    variant = B.VARIANT_GLOBAL_LUT_HALF if half else B.VARIANT_GLOBAL_LUT
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], d, 0, torch_io.to_device(codes, "codes"), None, variant)
    try:
        G, E = oracle.lut_groups(k, d, 0), 16 ** d
        assert G == 5
        stored = E // 2 if half else E
        L = torch.empty(B.msgemm_lut_bytes(plan) // 4, dtype=torch.float32, device="cuda:0")
        B.msgemm_build_lut(plan, dX, k, L)
        torch.cuda.synchronize()
        Lh = L.cpu().numpy()[: G * stored * b].reshape(G, stored, b)
    finally:
        B.msgemm_destroy(plan)
    ref = oracle.lut_build(x_to_f64(X, xd), d, 0)[:, :stored, :]
    assert np.max(np.abs(Lh.astype(np.float64) - ref)) <= d * 2.0 ** -23 * np.abs(ref).max()


# ---------------------------------------------------------------------------
# argument checking through the ABI (no kernel is launched for any of these)

def test_plan_rejects_bad_arguments():
    dC = torch.zeros(64 * 32, dtype=torch.uint8, device="cuda:0")
    dS = torch.ones(64, dtype=torch.float16, device="cuda:0")

    def rc(*a, **kw):
        status, handle = B.msgemm_plan(*a, check=False, **kw)
        assert handle is None or status == B.OK
        if status == B.OK:
            B.msgemm_destroy(handle)
        return status

    assert rc(64, 64, 1, "f32", "f32", 2, 0, dC) == B.OK
    assert rc(0, 64, 1, "f32", "f32", 2, 0, dC) == B.ERR_INVALID_ARG      # empty m
    assert rc(64, 0, 1, "f32", "f32", 2, 0, dC) == B.ERR_INVALID_ARG      # empty k
    assert rc(64, 64, 0, "f32", "f32", 2, 0, dC) == B.ERR_INVALID_ARG     # empty batch
    assert rc(64, 63, 1, "f32", "f32", 2, 0, dC) == B.ERR_INVALID_ARG     # odd k
    assert rc(64, 64, 1, "f32", "f32", 5, 0, dC) == B.ERR_INVALID_ARG     # d > 4
    assert rc(64, 64, 1, "f32", "f16", 2, 0, dC) == B.ERR_INVALID_ARG     # dtype pair
    assert rc(64, 64, 1, "f32", "f32", 2, 0, None) == B.ERR_INVALID_ARG   # null codes
    assert rc(64, 64, 1, "f32", "f32", 2, 48, dC, dS) == B.ERR_INVALID_ARG  # k % group
    assert rc(64, 64, 1, "f32", "f32", 4, 2, dC, dS) == B.ERR_INVALID_ARG   # group < d
    assert rc(64, 64, 1, "f32", "f32", 2, 32, dC, None) == B.ERR_INVALID_ARG  # scales missing
    assert rc(64, 64, 1, "i8", "i32", 2, 32, dC, dS) == B.ERR_INVALID_ARG   # int8 has no scales
    assert rc(64, 64, 1, "f32", "f32", 4, 0, dC, None, B.VARIANT_FUSED_LDS) == B.ERR_UNSUPPORTED
    assert rc(64, 64, 3, "f32", "f32", 3, 0, dC, None, B.VARIANT_FUSED_LDS) == B.ERR_UNSUPPORTED   # d = 3 in LDS: b <= 2

    plan = B.msgemm_plan(64, 64, 1, "f32", "f32", 2, 0, dC)
    try:
        X = torch.zeros(64, device="cuda:0")
        Y = torch.zeros(64, device="cuda:0")
        with pytest.raises(B.MsgemmError):
            B.msgemm_run(plan, X, 63, Y, 64)   # ldx < k
        with pytest.raises(B.MsgemmError):
            B.msgemm_run(plan, X, 64, Y, 10)   # ldy < m
        with pytest.raises(B.MsgemmError):
            B.msgemm_run(plan, None, 64, Y, 64)
    finally:
        B.msgemm_destroy(plan)
    B.msgemm_destroy(None)  # allowed


# ---------------------------------------------------------------------------
# fused LDS variant (d = 2): tiles, ragged tails, k-tile reduction

FUSED_SMALL = [
    # m, k, b, xd, sg   -- k/2 = groups; 64 groups per k-tile, 256 rows per panel
    (12, 4, 1, "f32", 0),        # far smaller than one tile
    (300, 520, 3, "f32", 0),     # 2 panels (ragged), 5 k-tiles (ragged)
    (2049, 1024, 1, "f16", 128),  # 9 panels, one row in the last
    (513, 512, 2, "bf16", 256),  # scale block spans two k-tiles
    (700, 768, 2, "i8", 0),
    (4100, 256, 1, "f16", 0),    # more panels than wavefronts per workgroup
]


@pytest.mark.parametrize("m,k,b,xd,sg", FUSED_SMALL)
def test_fused_variant_small(m, k, b, xd, sg):
    codes = inputs.make_codes(m, k, seed=m + 3 * k)
    X = inputs.make_x(k, b, xd, seed=k + b + 1)
    scales = inputs.make_scales(m, k, sg, seed=6) if sg else None
    ref = oracle_y(codes, X, xd, scales, sg)
    out, info = run_gpu(codes, X, xd, scales, sg, 2, B.VARIANT_FUSED_LDS, ldx_pad=10, ldy_pad=5)
    assert info["variant"] == B.VARIANT_FUSED_LDS and info["d"] == 2
    assert info["split_k"] == -(-(k // 2) // info["tile_groups"])
    check(out, ref, xd, "fused", elem_bound(codes, X, xd, scales, sg))
    if xd == "i8":
        out_g, _ = run_gpu(codes, X, xd, scales, sg, 2, B.VARIANT_GLOBAL_LUT)
        assert np.array_equal(out, out_g)


BATCHED = [
    # m, k, b, xd, sg, variant   -- 32 groups per k-tile, 8 (16-bit entries) or 4 (fp32) columns per pass
    (300, 520, 5, "f16", 0, B.VARIANT_FUSED_LDS16),     # ragged everything, one partial column pass
    (1025, 1024, 8, "f16", 128, B.VARIANT_FUSED_LDS16),  # scale block = two k-tiles
    (513, 512, 11, "bf16", 64, B.VARIANT_FUSED_LDS16),   # scale block = one k-tile, two column passes
    (700, 768, 16, "i8", 0, B.VARIANT_FUSED_LDS16),
    (260, 130, 3, "i8", 0, B.VARIANT_FUSED_LDS16),
    (300, 520, 6, "f32", 0, B.VARIANT_FUSED_LDS),        # fp32 entries, 4 columns per pass
    (515, 256, 4, "f32", 128, B.VARIANT_FUSED_LDS),
    (300, 520, 5, "f16", 0, B.VARIANT_FUSED_LDS),        # full-width entries on request: column at a time
]


@pytest.mark.parametrize("m,k,b,xd,sg,variant", BATCHED)
def test_fused_variant_batched(m, k, b, xd, sg, variant):
    codes = inputs.make_codes(m, k, seed=2 * m + k)
    X = inputs.make_x(k, b, xd, seed=k + 7 * b)
    scales = inputs.make_scales(m, k, sg, seed=9) if sg else None
    ref = oracle_y(codes, X, xd, scales, sg)
    out, info = run_gpu(codes, X, xd, scales, sg, 2, variant, ldx_pad=4, ldy_pad=7)
    assert info["variant"] == variant
    check(out, ref, xd, "fused batched", elem_bound(codes, X, xd, scales, sg, table16=variant == B.VARIANT_FUSED_LDS16))
    if variant == B.VARIANT_FUSED_LDS16:
        assert info["col_chunk"] == 8
        # the library's own choice for a batch this small: a pass of the single-column kernels per column
        # (full-width entries), where the scale blocks allow it (whole k-tiles of 128 columns)
        out_auto, info_auto = run_gpu(codes, X, xd, scales, sg, 2, B.VARIANT_AUTO)
        if sg % 128 == 0:
            assert info_auto["variant"] == B.VARIANT_FUSED_LDS and info_auto["col_chunk"] == 1
            check(out_auto, ref, xd, "fused batched, library's choice", elem_bound(codes, X, xd, scales, sg))
        else:
            assert info_auto["variant"] == B.VARIANT_FUSED_LDS16
            assert np.array_equal(out_auto, out)


PIPELINED_CASES = [
    # m, k, b, xd, sg, rows per lane, panels per workgroup (0: chosen), segments (0: chosen)
    (300, 520, 5, "f16", 0, 8, 0, 0),        # ragged rows, columns and last k-tile (17 k-tiles of 32 columns)
    (1025, 1024, 8, "f16", 128, 8, 0, 0),    # 3 panels of 512 rows, scale block = 4 k-tiles
    (513, 512, 11, "bf16", 64, 8, 0, 4),     # two column passes, scale block = 2 k-tiles, 4 segments
    (700, 768, 16, "i8", 0, 8, 0, 1),        # one segment of 24 k-tiles: written straight to Y
    (260, 130, 3, "i8", 0, 8, 0, 0),
    (5000, 640, 9, "f16", 32, 8, 8, 5),      # 10 panels: two row blocks of 8 wavefronts; scale block = one k-tile
    (2100, 384, 8, "f16", 128, 8, 2, 3),     # 5 panels, two per workgroup: idle wavefronts that only build
    (1025, 1024, 8, "f16", 128, 4, 0, 0),    # 16 wavefronts, 256-row panels
    (700, 768, 16, "i8", 0, 4, 4, 6),
    (300, 520, 13, "bf16", 0, 4, 0, 0),
    (3000, 256, 7, "f16", 64, 4, 16, 2),     # 12 panels in one workgroup of 16 wavefronts
]


@pytest.mark.parametrize("m,k,b,xd,sg,lb,ppw,segments", PIPELINED_CASES)
def test_batched_pipelined_form(m, k, b, xd, sg, lb, ppw, segments):
    """The batched kernel that builds the next table while it gathers from the current one
    (chosen by itself only for large problems), forced on small shapes; twice on one plan."""
    options = {"batched_form": 2, "rows_per_lane": lb, "panels_per_workgroup": ppw, "batched_segments": segments}
    codes = inputs.make_codes(m, k, seed=m + 5 * k)
    scales = inputs.make_scales(m, k, sg, seed=8) if sg else None
    dC = torch_io.to_device(codes, "codes")
    dS = torch_io.to_device(scales, "scales")
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS, B.VARIANT_FUSED_LDS16, options=options)
    try:
        info = B.msgemm_plan_get_info(plan)
        assert info["tile_groups"] == 16 and info["col_chunk"] == 8
        assert info["tile_rows"] % (64 * lb) == 0
        if segments:
            assert info["split_k"] == segments
        for rep in range(2):
            X = inputs.make_x(k, b, xd, seed=41 + rep)
            Xp = np.zeros((b, k + 6), dtype=X.dtype)
            Xp[:, :k] = X
            Xp[:, k:] = 77 if xd != "bf16" else 0x4300  # poison: must never reach the result
            dX = torch_io.to_device(Xp, xd)
            Y = torch_io.empty_output(b, m, Y_OF_X[xd], ldy=m + 3)
            Y.fill_(-3)
            B.msgemm_run(plan, dX, k + 6, Y, m + 3)
            torch.cuda.synchronize()
            out = torch_io.to_host(Y)
            check(np.ascontiguousarray(out[:, :m]), oracle_y(codes, X, xd, scales, sg), xd, f"pipelined call {rep}",
                  elem_bound(codes, X, xd, scales, sg, table16=True))
            minus3 = torch_io.to_host(torch.full((1,), -3, dtype=Y.dtype))[0]
            assert np.all(out[:, m:] == minus3), "output padding was written"
    finally:
        B.msgemm_destroy(plan)


DEALT_CASES = [
    # m, k, b, xd, sg, partial sums per output expected (the most runs a row block is cut into)
    (12288, 3200, 16, "f16", 0, 34),     # 3 row blocks x 100 k-tiles over 128 workgroups a pass: shares of 3 cross row blocks
    (9000, 3840, 60, "bf16", 128, 10),   # scale blocks of 4 k-tiles, last row block of 2 panels, ragged last pass
    (8292, 4096, 16, "i8", 0, 44),       # integer sums; 17 panels: the third row block has one
    (4097, 4096, 64, "f16", 128, 16),    # 2 row blocks x 32 scale blocks over 32 workgroups: shares of 2, no crossing
    (4500, 5120, 30, "bf16", 64, 0),     # partial sums small enough for the static array (scale blocks of 2 k-tiles)
]


@pytest.mark.parametrize("m,k,b,xd,sg,runs", DEALT_CASES)
def test_batched_pipelined_k_tiles_dealt(m, k, b, xd, sg, runs):
    """The pipelined batched kernel with the k-tiles of all row blocks dealt evenly over the workgroups (option
    batched_deal = 2): a workgroup's share may end one row block and begin the next.  Against the oracle, twice on one
    plan, and through the entry point that keeps its partial sums in the shared static array (whose unused slots hold
    whatever the last call left: row blocks are cut into different numbers of shares)."""
    options = {"batched_form": 2, "batched_deal": 2}
    codes = inputs.make_codes(m, k, seed=m + 3 * k)
    scales = inputs.make_scales(m, k, sg, seed=9) if sg else None
    dC = torch_io.to_device(codes, "codes")
    dS = torch_io.to_device(scales, "scales")
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS, B.VARIANT_FUSED_LDS16, options=options)
    try:
        info = B.msgemm_plan_get_info(plan)
        assert info["tile_groups"] == 16 and info["tile_rows"] == 4096
        if runs:
            assert info["split_k"] == runs
        static_fits = info["split_k"] * -(-b // 8) * 8 * -(-m // 512) * 512 * 4 <= 16 << 20
        assert static_fits == (runs == 0)
        for rep in range(3 if static_fits else 2):
            X = inputs.make_x(k, b, xd, seed=51 + rep)
            dX = torch_io.to_device(X, xd)
            Y = torch_io.empty_output(b, m, Y_OF_X[xd], ldy=m + 3)
            Y.fill_(-3)
            if rep == 2:
                # the static array first takes the partial sums of another problem of the same extent (equal segments,
                # as many as this plan has slots): the slots that a row block of this plan does not use then hold
                # numbers, and the second launch must not add them
                k2 = max(sg, 32) * info["split_k"]  # one scale block (or k-tile) per segment
                codes2 = inputs.make_codes(m, k2, seed=77)
                scales2 = inputs.make_scales(m, k2, sg, seed=78) if sg else None
                other = B.msgemm_plan(m, k2, b, xd, Y_OF_X[xd], 2, sg, torch_io.to_device(codes2, "codes"),
                                      torch_io.to_device(scales2, "scales"), B.VARIANT_FUSED_LDS16,
                                      options={"batched_form": 2, "batched_deal": 1, "batched_segments": info["split_k"]})
                try:
                    assert B.msgemm_plan_get_info(other)["split_k"] == info["split_k"]
                    B.msgemm_run_static(other, torch_io.to_device(inputs.make_x(k2, b, xd, seed=99), xd), k2, Y, m + 3)
                finally:
                    B.msgemm_destroy(other)
                Y.fill_(-3)
                B.msgemm_run_static(plan, dX, k, Y, m + 3)
            else:
                B.msgemm_run(plan, dX, k, Y, m + 3)
            torch.cuda.synchronize()
            out = torch_io.to_host(Y)
            check(np.ascontiguousarray(out[:, :m]), oracle_y(codes, X, xd, scales, sg), xd, f"dealt, call {rep}",
                  elem_bound(codes, X, xd, scales, sg, table16=True))
            minus3 = torch_io.to_host(torch.full((1,), -3, dtype=Y.dtype))[0]
            assert np.all(out[:, m:] == minus3), "output padding was written"
    finally:
        B.msgemm_destroy(plan)


def test_fused_lds16_not_for_fp32():
    dC = torch.zeros(64 * 32, dtype=torch.uint8, device="cuda:0")
    status, handle = B.msgemm_plan(64, 64, 4, "f32", "f32", 2, 0, dC, None, B.VARIANT_FUSED_LDS16, check=False)
    assert status == B.ERR_UNSUPPORTED and handle is None


def test_batched_scale_blocks_of_32_columns_use_the_pipelined_form():
    """Scale blocks of 32 columns are one k-tile of the pipelined batched form (the other form's k-tiles are 64)."""
    m, k, b = 700, 512, 9
    codes = inputs.make_codes(m, k, seed=4)
    X = inputs.make_x(k, b, "f16", seed=5)
    scales = inputs.make_scales(m, k, 32, seed=6)
    out, info = run_gpu(codes, X, "f16", scales, 32, 0, B.VARIANT_AUTO, ldx_pad=2, ldy_pad=1)
    assert info["variant"] == B.VARIANT_FUSED_LDS16 and info["tile_groups"] == 16
    check(out, oracle_y(codes, X, "f16", scales, 32), "f16", "scale blocks of 32", elem_bound(codes, X, "f16", scales, 32, table16=True))


def test_fused_scale_group_not_tileable_falls_back():
    m, k, b = 64, 256, 2
    codes = inputs.make_codes(m, k, seed=1)
    X = inputs.make_x(k, b, "f16", seed=2)
    scales = inputs.make_scales(m, k, 32, seed=3)  # a k-tile covers at least 64 columns
    out, info = run_gpu(codes, X, "f16", scales, 32, 0, B.VARIANT_AUTO)
    assert info["variant"] == B.VARIANT_GLOBAL_LUT
    check(out, oracle_y(codes, X, "f16", scales, 32), "f16", "fallback", elem_bound(codes, X, "f16", scales, 32))


REDUCE_CASES = [
    # m, k, b, xd, sg
    (2049, 1024, 1, "f16", 128),   # 8 k-tiles, 9 panels
    (300, 8320, 1, "f32", 0),      # 65 k-tiles: more flags per panel than lanes in a wavefront
    (700, 768, 2, "i8", 0),        # two column passes share the row blocks
    (4100, 512, 1, "bf16", 256),   # more panels than wavefronts per workgroup, scale block = two k-tiles
]


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("m,k,b,xd,sg", REDUCE_CASES)
def test_fused_k_tile_reduction_modes(m, k, b, xd, sg, mode):
    """Both ways of adding the k-tile partial sums (1: second launch, 2: inside the
    launch) against the oracle, twice on the same plan: the arrival flags of the
    in-launch reduction must be down again after a launch."""
    codes = inputs.make_codes(m, k, seed=m + k)
    scales = inputs.make_scales(m, k, sg, seed=4) if sg else None
    dC = torch_io.to_device(codes, "codes")
    dS = torch_io.to_device(scales, "scales")
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS, B.VARIANT_FUSED_LDS,
                         options={"reduce_mode": mode, "k_tiles_per_workgroup": 1})
    try:
        assert B.msgemm_plan_get_info(plan)["split_k"] == -(-(k // 2) // 64)
        for rep in range(2):
            X = inputs.make_x(k, b, xd, seed=31 + rep)
            dX = torch_io.to_device(X, xd)
            Y = torch_io.empty_output(b, m, Y_OF_X[xd])
            Y.fill_(-3)
            B.msgemm_run(plan, dX, k, Y, m)
            torch.cuda.synchronize()
            check(torch_io.to_host(Y), oracle_y(codes, X, xd, scales, sg), xd, f"reduce mode {mode} call {rep}",
                  elem_bound(codes, X, xd, scales, sg))
    finally:
        B.msgemm_destroy(plan)


LONG_K_CASES = [
    # m, k, b, xd, sg, k-tiles per workgroup, panels per workgroup (0: the library's choice)
    (700, 1024, 1, "f16", 128, 3, 0),     # 8 k-tiles in runs of 3, 3, 2
    (300, 8320, 1, "f32", 0, 7, 0),       # 65 k-tiles in runs of 7: ten segments, the last two tiles long
    (4100, 1280, 2, "i8", 0, 4, 16),      # 17 panels: two per wavefront and a second row block; two column passes
    (2300, 768, 1, "bf16", 256, 2, 16),   # 9 panels: one wavefront with two; scale block = two k-tiles
    (515, 640, 1, "f16", 128, 5, 0),      # one run holds all 5 k-tiles: written straight to Y
    (1000, 512, 1, "f16", 128, 2, 4),     # fewer panels than streaming wavefronts: idle wavefronts
]


@pytest.mark.parametrize("mode", [1, 2, 3])
@pytest.mark.parametrize("m,k,b,xd,sg,tps,ppw", LONG_K_CASES)
def test_fused_long_k_form(m, k, b, xd, sg, tps, ppw, mode):
    """The single-column kernel that runs through several k-tiles per workgroup
    (two table buffers, sums kept in registers), forced on small shapes; the three
    reductions over the segments (second launch, trailing workgroups, the producing
    workgroups themselves); twice on one plan."""
    codes = inputs.make_codes(m, k, seed=m + k + tps)
    scales = inputs.make_scales(m, k, sg, seed=6) if sg else None
    dC = torch_io.to_device(codes, "codes")
    dS = torch_io.to_device(scales, "scales")
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS, B.VARIANT_FUSED_LDS,
                         options={"k_tiles_per_workgroup": tps, "reduce_mode": mode, "panels_per_workgroup": ppw})
    try:
        ktiles = -(-(k // 2) // 64)
        assert B.msgemm_plan_get_info(plan)["split_k"] == -(-ktiles // tps)
        for rep in range(2):
            X = inputs.make_x(k, b, xd, seed=77 + rep)
            dX = torch_io.to_device(X, xd)
            Y = torch_io.empty_output(b, m, Y_OF_X[xd], ldy=m + 3)
            Y.fill_(-3)
            B.msgemm_run(plan, dX, k, Y, m + 3)
            torch.cuda.synchronize()
            out = torch_io.to_host(Y)
            check(np.ascontiguousarray(out[:, :m]), oracle_y(codes, X, xd, scales, sg), xd,
                  f"long-k tps {tps} reduce mode {mode} call {rep}", elem_bound(codes, X, xd, scales, sg))
    finally:
        B.msgemm_destroy(plan)


WIDE_CASES = [
    # m, k, b, xd, sg, panels per workgroup (0: the library's choice)
    (2049, 1024, 1, "f16", 128, 4),    # 8 k-tiles in pairs, 9 panels: three row groups, the last with one panel
    (300, 8320, 1, "f32", 0, 0),       # 65 k-tiles: 33 slices, the last with one table only
    (700, 768, 2, "i8", 0, 2),         # two column passes; two panels for four wavefronts per table: idle ones
    (4100, 512, 1, "bf16", 256, 8),    # 17 panels, 8 per workgroup: two per wavefront; scale block = the two k-tiles
    (515, 256, 1, "f16", 128, 1),      # one slice: written straight to Y
    (1030, 640, 1, "f16", 128, 3),     # five k-tiles: three slices; row groups of three panels (768 outputs over 3 readers)
]


@pytest.mark.parametrize("mode", [1, 3])
@pytest.mark.parametrize("m,k,b,xd,sg,ppw", WIDE_CASES)
def test_fused_wide_form_two_tables(m, k, b, xd, sg, ppw, mode):
    """The single-column kernel with the tables of two k-tiles per workgroup (a whole unit of codes in flight per
    wavefront, the two tables' sums joined through LDS), forced on small shapes; the sums over the slices added by a
    second launch (1) or by the workgroups that produced them (3); twice on one plan: flags must be down again."""
    codes = inputs.make_codes(m, k, seed=m + k + ppw)
    scales = inputs.make_scales(m, k, sg, seed=6) if sg else None
    dC = torch_io.to_device(codes, "codes")
    dS = torch_io.to_device(scales, "scales")
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS, B.VARIANT_FUSED_LDS,
                         options={"k_tiles_per_workgroup": 2, "reduce_mode": mode, "panels_per_workgroup": ppw})
    try:
        ktiles = -(-(k // 2) // 64)
        info = B.msgemm_plan_get_info(plan)
        assert info["split_k"] == -(-ktiles // 2)
        if ppw:
            assert info["tile_rows"] == 256 * ppw
        for rep in range(2):
            X = inputs.make_x(k, b, xd, seed=91 + rep)
            dX = torch_io.to_device(X, xd)
            Y = torch_io.empty_output(b, m, Y_OF_X[xd], ldy=m + 3)
            Y.fill_(-3)
            B.msgemm_run(plan, dX, k, Y, m + 3)
            torch.cuda.synchronize()
            out = torch_io.to_host(Y)
            check(np.ascontiguousarray(out[:, :m]), oracle_y(codes, X, xd, scales, sg), xd,
                  f"wide form, reduce mode {mode}, call {rep}", elem_bound(codes, X, xd, scales, sg))
            minus3 = torch_io.to_host(torch.full((1,), -3, dtype=Y.dtype))[0]
            assert np.all(out[:, m:] == minus3), "output padding was written"
        assert B.msgemm_plan_check(plan) == B.OK
    finally:
        B.msgemm_destroy(plan)


@pytest.mark.parametrize("options", [
    {"k_tiles_per_workgroup": 1},                               # wide form, one table: readers in the producing workgroups
    {"k_tiles_per_workgroup": 2, "panels_per_workgroup": 4},    # wide form, two tables
    {"k_tiles_per_workgroup": 3, "reduce_mode": 2},             # long-k form: trailing reducer workgroups
    {"k_tiles_per_workgroup": 3, "reduce_mode": 3},             # long-k form: readers in the producing workgroups
])
def test_in_launch_reduction_give_up_is_reported(options):
    """A reduction inside the launch whose producers never announce their partial sums (forced from the host: the
    announcement is skipped and the poll bound is tiny, so every kernel still runs to its end) must not pass for a
    result: the plan's check reports it once, clears the state, and the next check is clean."""
    m, k = 2049, 1024
    codes = inputs.make_codes(m, k, seed=3)
    X = inputs.make_x(k, 1, "f16", seed=4)
    dC, dX = torch_io.to_device(codes, "codes"), torch_io.to_device(X, "f16")
    Y = torch_io.empty_output(1, m, "f16")
    plan = B.msgemm_plan(m, k, 1, "f16", "f16", 2, 0, dC, None, B.VARIANT_FUSED_LDS,
                         options=dict(options, poll_limit=8, skip_publish=1))
    try:
        assert B.msgemm_plan_get_info(plan)["split_k"] > 1
        assert B.msgemm_plan_check(plan) == B.OK       # nothing has run yet
        B.msgemm_run(plan, dX, k, Y, m)
        assert B.msgemm_plan_check(plan) == B.ERR_INCOMPLETE
        assert B.msgemm_plan_check(plan) == B.OK       # reported once, then cleared
        B.msgemm_run(plan, dX, k, Y, m)
        assert B.msgemm_plan_check(plan) == B.ERR_INCOMPLETE
    finally:
        B.msgemm_destroy(plan)
    # the same problem without the test aid is complete and right
    plan = B.msgemm_plan(m, k, 1, "f16", "f16", 2, 0, dC, None, B.VARIANT_FUSED_LDS, options=dict(options))
    try:
        B.msgemm_run(plan, dX, k, Y, m)
        assert B.msgemm_plan_check(plan) == B.OK
        check(torch_io.to_host(Y), oracle_y(codes, X, "f16", None, 0), "f16", "after the give-up test",
              elem_bound(codes, X, "f16", None, 0))
    finally:
        B.msgemm_destroy(plan)


@pytest.mark.parametrize("form,xd", [(1, "f16"), (2, "bf16"), (1, "i8")])
def test_batched_segments_added_in_the_launch(form, xd):
    """Batches, on request (reduce_mode 3): the k-segments' sums are added by the workgroups of the launch that made
    them (the grid fits the device at once).  Against the oracle over repeated calls on one plan (the parity of a
    launch tags its sums), beside the default second launch, and the host-forced give-up is reported."""
    m, k, b, sg = 1300, 2048, 11, (0 if xd == "i8" else 128)
    codes = inputs.make_codes(m, k, seed=21)
    scales = inputs.make_scales(m, k, sg, seed=5) if sg else None
    dC, dS = torch_io.to_device(codes, "codes"), torch_io.to_device(scales, "scales")
    base = {"batched_form": form, "batched_segments": 4}
    outs = {}
    for mode in (3, 0):
        plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS, B.VARIANT_FUSED_LDS16, options=dict(base, reduce_mode=mode))
        try:
            assert B.msgemm_plan_get_info(plan)["split_k"] == 4
            for rep in range(3):
                X = inputs.make_x(k, b, xd, seed=30 + rep)
                dX = torch_io.to_device(X, xd)
                Y = torch_io.empty_output(b, m, Y_OF_X[xd], ldy=m + 1)
                Y.fill_(-3)
                B.msgemm_run(plan, dX, k, Y, m + 1)
                torch.cuda.synchronize()
                assert B.msgemm_plan_check(plan) == B.OK
                out = torch_io.to_host(Y)
                check(np.ascontiguousarray(out[:, :m]), oracle_y(codes, X, xd, scales, sg), xd,
                      f"batched, reduce mode {mode}, call {rep}", elem_bound(codes, X, xd, scales, sg, table16=True))
                minus3 = torch_io.to_host(torch.full((1,), -3, dtype=Y.dtype))[0]
                assert np.all(out[:, m:] == minus3), "output padding was written"
            outs[mode] = out
        finally:
            B.msgemm_destroy(plan)
    if xd == "i8":
        assert np.array_equal(outs[0], outs[3])
    # the give-up: partial sums are never stored, the poll bound is tiny
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS, B.VARIANT_FUSED_LDS16,
                         options=dict(base, reduce_mode=3, poll_limit=8, skip_publish=1))
    try:
        assert B.msgemm_plan_check(plan) == B.OK
        B.msgemm_run(plan, dX, k, Y, m + 1)
        assert B.msgemm_plan_check(plan) == B.ERR_INCOMPLETE
        assert B.msgemm_plan_check(plan) == B.OK
    finally:
        B.msgemm_destroy(plan)


XCD_LOCAL_CASES = [
    # form, m, k, b, xd, panels per workgroup, segments
    (1, 2000, 2048, 11, "f16", 1, 4),     # 8 row blocks x 2 column passes: a row block's passes share an XCD
    (1, 3700, 1024, 8, "bf16", 2, 8),     # 15 panels in 8 row blocks: the last one has a single panel
    (1, 1000, 2048, 13, "i8", 1, 4),      # 4 row blocks x 2 passes: the pairs are dealt over the XCDs
    (1, 1300, 1536, 27, "f16", 1, 3),     # 6 row blocks x 4 passes = 24 pairs, ragged rows, ragged last pass
    (2, 3700, 2048, 16, "bf16", 1, 4),    # pipelined form, 8 panels of 512 rows
    (2, 2500, 1024, 5, "i8", 1, 16),      # 5 row blocks: no even deal, the second launch adds
]


@pytest.mark.parametrize("form,m,k,b,xd,ppw,segments", XCD_LOCAL_CASES)
def test_batched_segments_added_inside_an_xcd(form, m, k, b, xd, ppw, segments):
    """Batches, reduce_mode 4: all workgroups of a (row block, column pass) run on one XCD and hand their sums over
    through its L2 (plain stores, an arrival count kept by L2 atomics).  Against the oracle over repeated calls on one
    plan (the count runs on over the launches); integer results equal the second launch's; the host-forced give-up
    is reported where the mode applies -- which also shows that it was taken -- and the plan works again afterwards."""
    sg = 0 if xd == "i8" else 128
    codes = inputs.make_codes(m, k, seed=m + b)
    scales = inputs.make_scales(m, k, sg, seed=5) if sg else None
    dC, dS = torch_io.to_device(codes, "codes"), torch_io.to_device(scales, "scales")
    base = {"batched_form": form, "batched_segments": segments, "panels_per_workgroup": ppw}
    panel_rows = 256 if form == 1 else 512
    row_blocks, passes = -(-(-(-m // panel_rows)) // ppw), -(-b // 8)
    applies = (row_blocks % 8 == 0) or (row_blocks * passes) % 8 == 0
    outs = {}
    for mode in (4, 1):
        plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS, B.VARIANT_FUSED_LDS16, options=dict(base, reduce_mode=mode))
        try:
            assert B.msgemm_plan_get_info(plan)["split_k"] == segments
            for rep in range(4):
                X = inputs.make_x(k, b, xd, seed=40 + rep)
                dX = torch_io.to_device(X, xd)
                Y = torch_io.empty_output(b, m, Y_OF_X[xd], ldy=m + 3)
                Y.fill_(-3)
                B.msgemm_run(plan, dX, k, Y, m + 3)
                torch.cuda.synchronize()
                assert B.msgemm_plan_check(plan) == B.OK
                out = torch_io.to_host(Y)
                check(np.ascontiguousarray(out[:, :m]), oracle_y(codes, X, xd, scales, sg), xd,
                      f"batched, reduce mode {mode}, call {rep}", elem_bound(codes, X, xd, scales, sg, table16=True))
                minus3 = torch_io.to_host(torch.full((1,), -3, dtype=Y.dtype))[0]
                assert np.all(out[:, m:] == minus3), "output padding was written"
            outs[mode] = out
        finally:
            B.msgemm_destroy(plan)
    if xd == "i8":
        assert np.array_equal(outs[1], outs[4])
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS, B.VARIANT_FUSED_LDS16,
                         options=dict(base, reduce_mode=4, poll_limit=8, skip_publish=1))
    try:
        assert B.msgemm_plan_check(plan) == B.OK
        B.msgemm_run(plan, dX, k, Y, m + 3)
        assert B.msgemm_plan_check(plan) == (B.ERR_INCOMPLETE if applies else B.OK)
        assert B.msgemm_plan_check(plan) == B.OK
    finally:
        B.msgemm_destroy(plan)


DEPTH3_CASES = [
    # m, k, b, xd, segments (0: the library's choice)
    (12, 4, 1, "f32", 0),          # the worked example's shape: one full group and one of a single column
    (300, 520, 1, "f32", 0),       # 174 groups: the last of one column; ragged rows
    (2049, 1024, 1, "f16", 0),     # four sub-panels per wavefront, two row blocks
    (700, 4096, 2, "bf16", 5),     # config 2's k (1366 groups, short last group), two columns, five segments
    (131, 130, 1, "i8", 0),        # integer tables
    (600, 768, 2, "i8", 3),
    (515, 98, 1, "f16", 1),        # a single segment: written straight to Y
]


@pytest.mark.parametrize("half", [0, 1])
@pytest.mark.parametrize("m,k,b,xd,segments", DEPTH3_CASES)
def test_depth_three_tables_in_lds(m, k, b, xd, segments, half):
    """d = 3 with the tables in LDS (16 KiB per group, 8 groups per k-tile; with half tables, Section 4.1, 16 groups):
    on request only.  Against the oracle, twice on one plan."""
    codes = inputs.make_codes(m, k, seed=m + k + half)
    dC = torch_io.to_device(codes, "codes")
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 3, 0, dC, None, B.VARIANT_FUSED_LDS,
                         options={"half_tables_in_lds": half, "batched_segments": segments})
    try:
        info = B.msgemm_plan_get_info(plan)
        assert info["variant"] == B.VARIANT_FUSED_LDS and info["d"] == 3 and info["tile_groups"] == (16 if half else 8)
        assert info["lut_groups"] == -(-k // 3)
        if segments:
            assert info["split_k"] == segments
        assert B.msgemm_plan_set_codebook(plan, UINT4, check=False) == B.ERR_UNSUPPORTED
        for rep in range(2):
            X = inputs.make_x(k, b, xd, seed=17 + rep)
            dX = torch_io.to_device(X, xd)
            Y = torch_io.empty_output(b, m, Y_OF_X[xd], ldy=m + 2)
            Y.fill_(-3)
            B.msgemm_run(plan, dX, k, Y, m + 2)
            torch.cuda.synchronize()
            out = torch_io.to_host(Y)
            bnd = elem_bound(codes, X, xd, None, 0)
            check(np.ascontiguousarray(out[:, :m]), oracle_y(codes, X, xd, None, 0), xd, f"d = 3 in LDS, half {half}, call {rep}",
                  None if bnd is None else (2 * bnd if half else bnd))
            minus3 = torch_io.to_host(torch.full((1,), -3, dtype=Y.dtype))[0]
            assert np.all(out[:, m:] == minus3), "output padding was written"
        if xd != "i8" and k % 64 == 0:
            # the dense comparison kernel reads rows: the plan makes its row-major copy from the run layout on this
            # first call (the workspace grows by exactly that copy), so this also checks that layout's inverse
            before = B.msgemm_plan_get_info(plan)["workspace_bytes"]
            Y = torch_io.empty_output(b, m, Y_OF_X[xd], ldy=m)
            B.msgemm_dequant_mfma_run(plan, dX, k, Y, m)
            torch.cuda.synchronize()
            assert B.msgemm_plan_get_info(plan)["workspace_bytes"] == before + m * (k // 2)
            check(torch_io.to_host(Y), oracle_y(codes, X, xd, None, 0), xd, "dense comparison on a d = 3 plan", bnd)
    finally:
        B.msgemm_destroy(plan)


def test_depth_three_in_lds_full_size_config2():
    """Config 2 asks for the sweep d in {2, 3}: d = 3 with the tables in LDS at full size, every row."""
    cfg, codes, X, _ = inputs.make_config("cfg2")
    for half in (0, 1):
        out, info = run_gpu(codes, X, "f16", None, 0, 3, B.VARIANT_FUSED_LDS, options={"half_tables_in_lds": half})
        assert info["d"] == 3 and info["variant"] == B.VARIANT_FUSED_LDS
        bnd = elem_bound(codes, X, "f16", None, 0)
        check(out, oracle_y(codes, X, "f16", None, 0), "f16", f"cfg2 d=3 in LDS half={half}", 2 * bnd if half else bnd)


def test_fused_repeated_calls_reuse_workspace():
    """Partial sums and arrival flags of one launch must not leak into the next."""
    m, k, b = 1000, 1024, 2
    codes = inputs.make_codes(m, k, seed=8)
    dC = torch_io.to_device(codes, "codes")
    plan = B.msgemm_plan(m, k, b, "i8", "i32", 2, 0, dC, None, B.VARIANT_FUSED_LDS)
    try:
        for rep in range(4):
            X = inputs.make_x(k, b, "i8", seed=20 + rep)
            dX = torch_io.to_device(X, "i8")
            Y = torch_io.empty_output(b, m, "i32")
            B.msgemm_run(plan, dX, k, Y, m)
            torch.cuda.synchronize()
            assert np.array_equal(torch_io.to_host(Y), oracle.gemm_i32(codes, X)), rep
    finally:
        B.msgemm_destroy(plan)


BACK_TO_BACK_CASES = [
    # m, k, b, xd, sg, variant, options: the reductions that hand partial sums over inside a launch
    (2049, 1024, 1, "f16", 128, B.VARIANT_FUSED_LDS, {"k_tiles_per_workgroup": 2, "reduce_mode": 3}),   # wide form, parity-tagged sums
    (1024, 1024, 1, "f32", 0, B.VARIANT_FUSED_LDS, None),                                                 # config 1's own choice
    (700, 1024, 1, "f16", 128, B.VARIANT_FUSED_LDS, {"k_tiles_per_workgroup": 3, "reduce_mode": 2}),      # long-k form, flags
    (4100, 1280, 2, "bf16", 128, B.VARIANT_FUSED_LDS, {"k_tiles_per_workgroup": 4, "reduce_mode": 3, "panels_per_workgroup": 16}),  # long-k form, parity-tagged sums
    (2300, 768, 2, "i8", 0, B.VARIANT_FUSED_LDS, {"k_tiles_per_workgroup": 1, "reduce_mode": 2}),         # plain form, flags, two column passes
    (2100, 512, 8, "bf16", 128, B.VARIANT_FUSED_LDS16, {"batched_form": 1, "reduce_mode": 3}),            # batched, sums added in the launch
]


@pytest.mark.parametrize("m,k,b,xd,sg,variant,options", BACK_TO_BACK_CASES)
def test_many_launches_back_to_back_on_one_plan(m, k, b, xd, sg, variant, options):
    """48 launches on one plan enqueued without a wait in between, each with activations and an output buffer of its
    own, all checked afterwards: a launch must never take a partial sum, a flag or a launch parity of its
    predecessor for its own (the benchmark's pattern: thousands of launches, one stream, no host in between)."""
    n = 48
    codes = inputs.make_codes(m, k, seed=5 * m + k)
    scales = inputs.make_scales(m, k, sg, seed=9) if sg else None
    dC = torch_io.to_device(codes, "codes")
    dS = torch_io.to_device(scales, "scales")
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS, variant, options=options)
    try:
        Xs = [inputs.make_x(k, b, xd, seed=1000 + i) for i in range(n)]
        dXs = [torch_io.to_device(X, xd) for X in Xs]
        Ys = [torch_io.empty_output(b, m, Y_OF_X[xd]) for _ in range(n)]
        for Y in Ys:
            Y.fill_(-3)
        torch.cuda.synchronize()
        for i in range(n):
            B.msgemm_run(plan, dXs[i], k, Ys[i], m)
        torch.cuda.synchronize()
        assert B.msgemm_plan_check(plan) == B.OK
        table16 = B.msgemm_plan_get_info(plan)["variant"] == B.VARIANT_FUSED_LDS16
        for i in range(n):
            check(torch_io.to_host(Ys[i]), oracle_y(codes, Xs[i], xd, scales, sg), xd, f"launch {i} of {n}",
                  elem_bound(codes, Xs[i], xd, scales, sg, table16=table16))
    finally:
        B.msgemm_destroy(plan)


COLUMN_PASS_CASES = [
    # m, k, b, xd, sg, options: several column passes through each form of the single-column kernels, with unit
    # counts (row blocks x k-slices) that are no multiple of the XCD count, so ids past the last unit exist
    (700, 768, 2, "f16", 128, {"k_tiles_per_workgroup": 1, "reduce_mode": 2}),                      # plain form, 3 units
    (2300, 1280, 3, "bf16", 256, {"k_tiles_per_workgroup": 1, "reduce_mode": 1, "panels_per_workgroup": 4}),  # 3 x 10 units, 3 passes
    (1030, 640, 3, "f16", 128, {"k_tiles_per_workgroup": 2, "reduce_mode": 3, "panels_per_workgroup": 3}),    # wide, two tables: 2 x 3 units
    (515, 1024, 2, "f32", 0, {"k_tiles_per_workgroup": 1, "reduce_mode": 3, "panels_per_workgroup": 8}),      # wide, one table: 8 units, resident
    (4100, 1280, 2, "i8", 0, {"k_tiles_per_workgroup": 4, "reduce_mode": 2, "panels_per_workgroup": 16}),     # long-k: 2 x 3 units
    (300, 8320, 5, "f16", 0, {"k_tiles_per_workgroup": 7, "reduce_mode": 1}),                                # long-k, 10 units, 5 passes
    (1500, 640, 10, "f32", 64, {}),                                                                          # four fp32 columns per entry: 3 passes
]


@pytest.mark.parametrize("m,k,b,xd,sg,options", COLUMN_PASS_CASES)
def test_column_passes_of_the_single_column_kernels(m, k, b, xd, sg, options):
    """Plans with several column passes (b = 2, full-width tables requested for wider batches, fp32 activations
    beyond four columns): the passes of one (row block, k-slice) unit get neighbouring workgroup ids on one XCD.
    Every form and reduction mode of the single-column kernels, twice on one plan."""
    codes = inputs.make_codes(m, k, seed=m + 3 * k + b)
    scales = inputs.make_scales(m, k, sg, seed=8) if sg else None
    dC = torch_io.to_device(codes, "codes")
    dS = torch_io.to_device(scales, "scales")
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS, B.VARIANT_FUSED_LDS, options=options or None)
    try:
        info = B.msgemm_plan_get_info(plan)
        assert info["variant"] == B.VARIANT_FUSED_LDS and -(-b // info["col_chunk"]) > 1
        for rep in range(2):
            X = inputs.make_x(k, b, xd, seed=57 + rep)
            dX = torch_io.to_device(X, xd)
            Y = torch_io.empty_output(b, m, Y_OF_X[xd], ldy=m + 5)
            Y.fill_(-3)
            B.msgemm_run(plan, dX, k, Y, m + 5)
            torch.cuda.synchronize()
            out = torch_io.to_host(Y)
            check(np.ascontiguousarray(out[:, :m]), oracle_y(codes, X, xd, scales, sg), xd,
                  f"column passes {options} call {rep}", elem_bound(codes, X, xd, scales, sg))
            minus3 = torch_io.to_host(torch.full((1,), -3, dtype=Y.dtype))[0]
            assert np.all(out[:, m:] == minus3), "output padding was written"
        assert B.msgemm_plan_check(plan) == B.OK
    finally:
        B.msgemm_destroy(plan)


def test_two_columns_at_full_size():
    """The paper's 12288 x 49152 GeMM (Section 5) with two activation vectors: two column passes through the long-k
    form, 234 units over 8 XCDs, every row against the oracle."""
    m, k, b, xd = 12288, 49152, 2, "f16"
    codes = inputs.make_codes(m, k, seed=41)
    X = inputs.make_x(k, b, xd, seed=42)
    out, info = run_gpu(codes, X, xd, None, 0, 2, B.VARIANT_AUTO)
    assert info["variant"] == B.VARIANT_FUSED_LDS and info["col_chunk"] == 1
    check(out, oracle_y(codes, X, xd, None, 0), xd, "mlp1 shape, b = 2", elem_bound(codes, X, xd, None, 0))


# ---------------------------------------------------------------------------
# the benchmark configurations at full size, library's own choice of variant

@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3a", "cfg3b", "cfg4", "cfg5", "mlp1", "mlp2", "mlp2_b16", "big1"])
def test_config_full_size(name):
    cfg, codes, X, scales = inputs.make_config(name)
    m, k, b, xd, sg = cfg["m"], cfg["k"], cfg["b"], cfg["x"], cfg["scale_group"]
    out, info = run_gpu(codes, X, xd, scales, sg, cfg["d"], B.VARIANT_AUTO)
    assert info["variant"] in (B.VARIANT_FUSED_LDS, B.VARIANT_FUSED_LDS16)
    # every row of every configuration goes through the oracle (the largest, cfg5, is 15e9 multiply-adds:
    # a few seconds on the host cores), and through it once more with magnitudes for the per-element bound
    rows = np.arange(m)
    ref = oracle_y(codes, X, xd, scales, sg)
    err = check(out, ref, xd, name, elem_bound(codes, X, xd, scales, sg, table16=info["variant"] == B.VARIANT_FUSED_LDS16))
    if xd != "i8":
        # against the oracle's own rounding to the output type as well
        widen = {"f32": lambda a: a.astype(np.float64), "f16": oracle.f16_bits_to_f64,
                 "bf16": oracle.bf16_bits_to_f64}[cfg["y"]]
        ref_rounded = widen(oracle.round_to(ref, cfg["y"]))
        err_r = oracle.rel_l2(torch_io.to_f64(np.ascontiguousarray(out[:, rows])), ref_rounded)
        assert err_r <= TOL[xd]
    print(f"{name}: rows checked {len(rows)}/{m}, rel L2 {err:.3e}")


@pytest.mark.parametrize("m,k,xd,sg", [
    ((1 << 20) + 3, 1024, "f16", 128),   # a million rows: 4097 panels, offsets of the partial buffer near their range
    (515, 1 << 18, "f16", 0),            # 2048 k-tiles: the long-k form at scale
    (259, 1 << 17, "i8", 0),             # the same with integer tables
])
def test_extreme_aspect_ratios(m, k, xd, sg):
    """Very tall and very wide problems (b = 1), every row against the oracle."""
    codes = inputs.make_codes(m, k, seed=17)
    X = inputs.make_x(k, 1, xd, seed=18)
    scales = inputs.make_scales(m, k, sg, seed=19) if sg else None
    out, info = run_gpu(codes, X, xd, scales, sg, 2, B.VARIANT_AUTO)
    assert info["variant"] == B.VARIANT_FUSED_LDS
    check(out, oracle_y(codes, X, xd, scales, sg), xd, f"{m}x{k}", elem_bound(codes, X, xd, scales, sg))


@pytest.mark.parametrize("pipelined", [0, 1])
@pytest.mark.parametrize("m,k,b,xd,sg", [
    (300001, 512, 8, "f16", 128),        # tall: 1172 panels of 256 rows (586 of 512)
    (515, 1 << 17, 8, "bf16", 0),        # wide: 2048 (4096) k-tiles, long segments
    (259, 1 << 16, 16, "i8", 0),         # the same with integer tables and two column passes
])
def test_extreme_aspect_ratios_batched(m, k, b, xd, sg, pipelined):
    """Very tall and very wide batched problems in both forms of the batched kernel, every row against the oracle."""
    codes = inputs.make_codes(m, k, seed=23)
    X = inputs.make_x(k, b, xd, seed=24)
    if xd != "i8" and k > 4096:
        X = (X.astype(np.float32) / 8).astype(X.dtype) if xd == "f16" else X  # keep fp16 outputs in range
    scales = inputs.make_scales(m, k, sg, seed=25) if sg else None
    out, info = run_gpu(codes, X, xd, scales, sg, 2, B.VARIANT_AUTO, options={"batched_form": 1 + pipelined})
    assert info["variant"] == B.VARIANT_FUSED_LDS16 and info["tile_groups"] == (16 if pipelined else 32)
    check(out, oracle_y(codes, X, xd, scales, sg), xd, f"{m}x{k}x{b}", elem_bound(codes, X, xd, scales, sg, table16=True))


@pytest.mark.parametrize("pipelined", [0, 1])
def test_int8_batched_sums_stay_exact_on_long_segments(pipelined):
    """The batched kernel adds int8 tables in fp32.  Worst case for that: the first half of k drives
    every sum to 2^25 (codes -8, activations -128), the second half adds ones, which fp32 could no longer
    hold if one segment ran through all of k.  A single segment is asked for; the library must cut it."""
    m, k, b = 300, 1 << 16, 8
    codes = np.empty((m, k // 2), dtype=np.uint8)
    codes[:, : k // 4] = 0x88           # two codes of -8
    codes[:, k // 4:] = 0x01            # codes +1 and 0
    X = np.empty((b, k), dtype=np.int8)
    X[:, : k // 2] = -128
    X[:, k // 2:] = 1
    X[3, k // 2:] = -1                  # one column counts down instead
    ref = oracle.gemm_i32(codes, X)
    assert ref[0, 0] == (1 << 25) + k // 4 and ref[3, 0] == (1 << 25) - k // 4
    out, info = run_gpu(codes, X, "i8", None, 0, 2, B.VARIANT_FUSED_LDS16,
                        options={"batched_form": 1 + pipelined, "batched_segments": 1})
    assert info["split_k"] >= (k // 2) // 8192  # at most 8192 groups per segment
    assert np.array_equal(out, ref)


def test_config2_d3_sweep_point():
    """Config 2 also asks for d = 3 (k = 4096 is not a multiple of 3: short last group)."""
    cfg, codes, X, _ = inputs.make_config("cfg2", m=2048)
    out, info = run_gpu(codes, X, "f16", None, 0, 3, B.VARIANT_AUTO)
    assert info["d"] == 3 and info["lut_groups"] == 1366
    check(out, oracle_y(codes, X, "f16", None, 0), "f16", "cfg2 d=3", elem_bound(codes, X, "f16", None, 0))


@pytest.mark.parametrize("d", [1, 2, 3, 4])
def test_config2_full_size_two_launch_variant(d):
    """The table in device memory, the launch configuration the d-sweep is timed in."""
    cfg, codes, X, scales = inputs.make_config("cfg2")
    out, info = run_gpu(codes, X, cfg["x"], scales, cfg["scale_group"], d, B.VARIANT_GLOBAL_LUT)
    assert info["variant"] == B.VARIANT_GLOBAL_LUT and info["d"] == d
    check(out, oracle_y(codes, X, cfg["x"], scales, cfg["scale_group"]), cfg["x"], f"cfg2 two-launch d={d}",
          elem_bound(codes, X, cfg["x"], scales, cfg["scale_group"]))


@pytest.mark.parametrize("m,k,b,xd,sg,d", [
    (700, 2048, 1, "f16", 128, 3),   # several segments, short last group per block
    (130, 1032, 3, "f32", 0, 3),     # one long block cut into chunks, ragged column pass
    (257, 768, 5, "bf16", 64, 4),
    (90, 512, 4, "i8", 0, 2),
    (64, 4096, 2, "f16", 0, 1),
])
def test_two_launch_consumers_agree_with_oracle(m, k, b, xd, sg, d):
    """The tiled consumer and the plain one-thread-per-output consumer against the oracle."""
    codes = inputs.make_codes(m, k, seed=m + d)
    X = inputs.make_x(k, b, xd, seed=k + d)
    scales = inputs.make_scales(m, k, sg, seed=8) if sg else None
    ref = oracle_y(codes, X, xd, scales, sg)
    chunks = {"global_chunk_kib": 64}  # several chunks per block where the block is long
    out_t, _ = run_gpu(codes, X, xd, scales, sg, d, B.VARIANT_GLOBAL_LUT, ldx_pad=2, ldy_pad=5, options=chunks)
    bnd = elem_bound(codes, X, xd, scales, sg)
    check(out_t, ref, xd, "tiled consumer", bnd)
    out_p, _ = run_gpu(codes, X, xd, scales, sg, d, B.VARIANT_GLOBAL_LUT, ldx_pad=2, ldy_pad=5,
                       options={"global_chunk_kib": 64, "global_plain_consumer": 1})
    check(out_p, ref, xd, "plain consumer", bnd)
    if xd == "i8":
        assert np.array_equal(out_t, out_p)


# ---------------------------------------------------------------------------
# half tables (Section 4.1): the two-launch variant storing only the combinations
# whose last code has its top bit clear

HALF_CASES = [
    # m, k, b, xd, sg, d
    (300, 520, 3, "f32", 0, 3),      # 520 = 173 * 3 + 1: a short last group; tiled consumer
    (257, 384, 5, "f16", 128, 3),    # short last group in every block
    (64, 256, 2, "bf16", 64, 2),
    (131, 130, 4, "i8", 0, 2),       # k not a multiple of 8: the plain consumer
    (90, 512, 4, "i8", 0, 1),        # 16-byte table reads
    (40, 64, 1, "f16", 16, 4),
    (2100, 1024, 1, "f16", 128, 3),  # several segments
    (50, 260, 20, "f16", 0, 3),      # tables built on the matrix cores, ragged column tile
]


@pytest.mark.parametrize("m,k,b,xd,sg,d", HALF_CASES)
def test_half_table_variant_against_oracle(m, k, b, xd, sg, d):
    codes = inputs.make_codes(m, k, seed=m + 3 * d)
    X = inputs.make_x(k, b, xd, seed=k + d)
    scales = inputs.make_scales(m, k, sg, seed=9) if sg else None
    ref = oracle_y(codes, X, xd, scales, sg)
    out, info = run_gpu(codes, X, xd, scales, sg, d, B.VARIANT_GLOBAL_LUT_HALF, ldx_pad=4, ldy_pad=2)
    assert info["variant"] == B.VARIANT_GLOBAL_LUT_HALF and info["d"] == d
    check(out, ref, xd, f"half tables d={d}", 2 * elem_bound(codes, X, xd, scales, sg) if xd != "i8" else None)
    out2, _ = run_gpu(codes, X, xd, scales, sg, d, B.VARIANT_GLOBAL_LUT_HALF, use_phases=True)
    assert np.array_equal(out2, out), "phases called separately differ from msgemm_run"


@pytest.mark.parametrize("b", [3, 24])
@pytest.mark.parametrize("xd,sg,d", [("f32", 0, 2), ("f16", 128, 3), ("i8", 0, 3), ("bf16", 0, 1)])
def test_half_table_contents_against_phase1_reference(xd, sg, d, b):
    """L_out = the first half of the oracle's table (last code 0..7), then S(j) =
    the oracle's entry for codes 0001..0001 (b = 1: the plain sum of the group)."""
    m, k = 8, 256
    codes = inputs.make_codes(m, k, seed=1)
    X = inputs.make_x(k, b, xd, seed=2)
    scales = inputs.make_scales(m, k, sg, seed=3) if sg else None
    dC, dS = torch_io.to_device(codes, "codes"), torch_io.to_device(scales, "scales")
    dX = torch_io.to_device(X, xd)
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], d, sg, dC, dS, B.VARIANT_GLOBAL_LUT_HALF)
    try:
        G, E = oracle.lut_groups(k, d, sg), 16 ** d
        assert B.msgemm_lut_bytes(plan) == G * (E // 2 + 1) * b * 4
        L = torch.empty(G * (E // 2 + 1) * b, dtype=torch.int32 if xd == "i8" else torch.float32, device="cuda:0")
        B.msgemm_build_lut(plan, dX, k, L)
        torch.cuda.synchronize()
        Lh = L.cpu().numpy()
    finally:
        B.msgemm_destroy(plan)
    table = Lh[: G * (E // 2) * b].reshape(G, E // 2, b)
    sums = Lh[G * (E // 2) * b:].reshape(G, b)
    ref = oracle.lut_build(X if xd == "i8" else x_to_f64(X, xd), d, sg)
    ones = sum(1 << (4 * r) for r in range(d))
    if xd == "i8":
        assert np.array_equal(table, ref[:, : E // 2, :]) and np.array_equal(sums, ref[:, ones, :])
    else:
        tol = d * 2.0 ** -23 * np.abs(ref).max()
        assert np.max(np.abs(table.astype(np.float64) - ref[:, : E // 2, :])) <= tol
        assert np.max(np.abs(sums.astype(np.float64) - ref[:, ones, :])) <= tol


def test_half_table_value_maps():
    """An unsigned map has value(~i) + value(i) = 15 and works with half tables; a map without such a constant is refused."""
    m, k, b, d = 200, 384, 2, 3
    codes = inputs.make_codes(m, k, seed=21)
    X = inputs.make_x(k, b, "f16", seed=22)
    dC, dX = torch_io.to_device(codes, "codes"), torch_io.to_device(X, "f16")
    plan = B.msgemm_plan(m, k, b, "f16", "f16", d, 0, dC, None, B.VARIANT_GLOBAL_LUT_HALF)
    try:
        assert B.msgemm_plan_set_codebook(plan, NONUNIFORM, check=False) == B.ERR_UNSUPPORTED
        B.msgemm_plan_set_codebook(plan, UINT4)
        Y = torch_io.empty_output(b, m, "f16")
        B.msgemm_run(plan, dX, k, Y, m)
        torch.cuda.synchronize()
        ref = oracle.gemm_f64(codes, x_to_f64(X, "f16"), codebook=UINT4)
        check(torch_io.to_host(Y), ref, "f16", "half tables, unsigned map", 2 * elem_bound(codes, X, "f16", None, 0, codebook=UINT4))
    finally:
        B.msgemm_destroy(plan)


# ---------------------------------------------------------------------------
# shared exponents (Section 3.3 names int4 mantissas with a shared 8-bit exponent):
# block scales that are powers of two

@pytest.mark.parametrize("m,k,b,variant", [(700, 1024, 1, B.VARIANT_FUSED_LDS), (300, 512, 2, B.VARIANT_GLOBAL_LUT),
                                           (520, 512, 8, B.VARIANT_FUSED_LDS16)])
def test_power_of_two_block_scales_are_exact(m, k, b, variant):
    """int4 mantissas times 2^e per block of 128, small integer activations: every
    partial sum is an integer times a power of two well inside fp32 (and fp16
    tables), so the fp32 result must equal the oracle's bit for bit."""
    sg = 128
    rng = np.random.default_rng(m + b)
    codes = inputs.make_codes(m, k, seed=41)
    X = rng.integers(-4, 5, size=(b, k)).astype(np.float32)
    scales = (2.0 ** rng.integers(-6, 3, size=(m, k // sg))).astype(np.float16)
    xd = "f32" if variant != B.VARIANT_FUSED_LDS16 else "f16"
    Xd = X if xd == "f32" else X.astype(np.float16)
    ref = oracle.gemm_f64(codes, X.astype(np.float64), scales, sg)
    out, info = run_gpu(codes, Xd, xd, scales, sg, 2, variant)
    assert info["variant"] == variant
    got = torch_io.to_f64(out)
    if xd == "f32":
        assert np.array_equal(got, ref)
    else:
        # fp16 output: the exact sum rounded once
        want = oracle.f16_bits_to_f64(oracle.round_to(ref, "f16"))
        assert np.array_equal(got, want)


@pytest.mark.parametrize("pipelined", [0, 1])
@pytest.mark.parametrize("xd", ["f16", "bf16"])
def test_16_bit_tables_report_activations_out_of_their_range(xd, pipelined):
    """A table entry of the batched kernels is b(c0) x0 + b(c1) x1 in fp16: |x| beyond 65504 / 16 = 4094 can push it
    to infinity.  The library's own choice for a large batch has such tables; it must say so (msgemm_plan_check), and
    the variant with full-width entries must give the right answer on the same inputs."""
    m, k, b = 600, 512, 8
    codes = inputs.make_codes(m, k, seed=1)
    X = inputs.make_x(k, b, "f32", seed=2)
    X[3, 100] = 30000.0          # times -8 and more: beyond fp16
    X[5, 7] = -5000.0
    Xh = X.astype(np.float16) if xd == "f16" else inputs.f32_to_bf16_bits(X)
    dC, dX = torch_io.to_device(codes, "codes"), torch_io.to_device(Xh, xd)
    Y = torch_io.empty_output(b, m, xd)
    plan = B.msgemm_plan(m, k, b, xd, xd, 2, 0, dC, None, B.VARIANT_FUSED_LDS16, options={"batched_form": 1 + pipelined})
    try:
        assert B.msgemm_plan_get_info(plan)["variant"] == B.VARIANT_FUSED_LDS16
        B.msgemm_run(plan, dX, k, Y, m)
        assert B.msgemm_plan_check(plan) == B.ERR_RANGE
        assert B.msgemm_plan_check(plan) == B.OK        # reported once
        # the same plan with activations inside the range is clean again
        Xok = np.clip(X, -4000.0, 4000.0)
        Xokh = Xok.astype(np.float16) if xd == "f16" else inputs.f32_to_bf16_bits(Xok)
        B.msgemm_run(plan, torch_io.to_device(Xokh, xd), k, Y, m)
        assert B.msgemm_plan_check(plan) == B.OK
        check(torch_io.to_host(Y), oracle_y(codes, Xokh, xd, None, 0), xd, "activations at the edge of the range",
              elem_bound(codes, Xokh, xd, None, 0, table16=True))
    finally:
        B.msgemm_destroy(plan)
    # full-width entries take the large activations (fp16 outputs of this size would overflow: bf16 only)
    if xd == "bf16":
        out, info = run_gpu(codes, Xh, xd, None, 0, 2, B.VARIANT_FUSED_LDS)
        assert info["variant"] == B.VARIANT_FUSED_LDS
        check(out, oracle_y(codes, Xh, xd, None, 0), xd, "full-width tables", elem_bound(codes, Xh, xd, None, 0))


def test_16_bit_tables_refuse_value_maps_out_of_their_range():
    dC = torch.zeros(128 * 64, dtype=torch.uint8, device="cuda:0")
    plan = B.msgemm_plan(128, 128, 8, "f16", "f16", 2, 0, dC, None, B.VARIANT_FUSED_LDS16)
    try:
        big = list(UINT4)
        big[9] = 1.0e5
        assert B.msgemm_plan_set_codebook(plan, big, check=False) == B.ERR_UNSUPPORTED
        assert B.msgemm_plan_set_codebook(plan, UINT4, check=False) == B.OK
    finally:
        B.msgemm_destroy(plan)
    plan = B.msgemm_plan(128, 128, 8, "f32", "f32", 2, 0, dC, None, B.VARIANT_FUSED_LDS)
    try:
        big = list(UINT4)
        big[9] = 1.0e5
        assert B.msgemm_plan_set_codebook(plan, big, check=False) == B.OK   # full-width entries hold it
    finally:
        B.msgemm_destroy(plan)
    v = e4m3_finite() * 1000.0    # up to 448000: beyond fp16
    dC8 = torch.zeros(128 * 128, dtype=torch.uint8, device="cuda:0")
    assert B.msgemm_plan_codes8(128, 128, 8, "f16", "f16", 0, dC8, None, v, check=False)[0] == B.ERR_UNSUPPORTED
    rc, plan = B.msgemm_plan_codes8(128, 128, 1, "f16", "f16", 0, dC8, None, v, check=False)  # one column: full-width tables
    assert rc == B.OK
    B.msgemm_destroy(plan)


# ---------------------------------------------------------------------------
# 8-bit weights with a 256-entry value map (Section 2: an 8-bit floating-point
# weight matrix is another datatype the method applies to)

def e4m3_finite():
    v = inputs.fp8_e4m3_values()
    v[np.isnan(v)] = 0.0  # the two NaN patterns never occur in the codes
    return v


CODES8_CASES = [
    # m, k, b, xd, sg, plan options
    (300, 520, 1, "f32", 0, {}),                       # ragged rows and a ragged last k-tile
    (2049, 512, 1, "f16", 128, {}),                    # 8 k-tiles, 9 panels, scales
    (700, 384, 2, "bf16", 64, {}),                     # two column passes, scale block = one k-tile
    (515, 4096, 1, "f16", 0, {"k_tiles_per_workgroup": 5}),   # the long-k form: runs of 5 k-tiles
    (4100, 640, 1, "f16", 128, {"k_tiles_per_workgroup": 3, "panels_per_workgroup": 16}),
    (64, 64, 1, "f32", 64, {}),                        # a single k-tile: straight to Y
    (520, 512, 8, "f16", 128, {}),                     # batches: fp16 tables of 8 columns
    (300, 384, 5, "bf16", 0, {}),                      # a ragged column pass
    (1000, 1024, 16, "f16", 32, {}),                   # two column passes, scale block = one k-tile of 32 columns
    (257, 256, 4, "f32", 0, {}),                       # fp32 activations: four fp32 columns per entry
    (130, 320, 7, "f32", 64, {}),
    (520, 512, 8, "f16", 128, {"batched_form": 2}),                        # the pipelined batched form
    (1000, 1024, 16, "f16", 32, {"batched_form": 2, "rows_per_lane": 4}),
    (300, 384, 5, "bf16", 0, {"batched_form": 2, "batched_segments": 3}),
    (12288, 1600, 16, "f16", 0, {"batched_form": 2, "batched_deal": 2}),    # k-tiles dealt evenly: shares of 3 cross row blocks
    (9000, 2048, 60, "bf16", 64, {"batched_form": 2, "batched_deal": 2}),   # ... with scale blocks of 4 k-tiles
]


@pytest.mark.parametrize("m,k,b,xd,sg,options", CODES8_CASES)
def test_codes8_against_oracle(m, k, b, xd, sg, options):
    codes = inputs.make_codes8(m, k, seed=m + k)
    X = inputs.make_x(k, b, xd, seed=k + 1)
    scales = inputs.make_scales(m, k, sg, seed=10) if sg else None
    values = e4m3_finite() / 16.0   # keeps fp16 outputs in range
    ref = oracle.gemm_f64_codes8(codes, x_to_f64(X, xd), values, scales, sg)
    dC, dS, dX = torch_io.to_device(codes, "codes"), torch_io.to_device(scales, "scales"), torch_io.to_device(X, xd)
    plan = B.msgemm_plan_codes8(m, k, b, xd, Y_OF_X[xd], sg, dC, dS, values, options=options or None)
    try:
        info = B.msgemm_plan_get_info(plan)
        assert (info["k"], info["d"], info["lut_groups"], info["scale_group"]) == (k, 1, k, sg)
        assert info["variant"] == (B.VARIANT_FUSED_LDS if b <= 2 or xd == "f32" else B.VARIANT_FUSED_LDS16)
        for rep in range(2):
            Y = torch_io.empty_output(b, m, Y_OF_X[xd], ldy=m + 1)
            Y.fill_(-3)
            B.msgemm_run(plan, dX, k, Y, m + 1)
            torch.cuda.synchronize()
            out = torch_io.to_host(Y)
            check(np.ascontiguousarray(out[:, :m]), ref, xd, f"8-bit weights call {rep}",
                  elem_bound(codes, X, xd, scales, sg, table16=info["variant"] == B.VARIANT_FUSED_LDS16, values256=values))
    finally:
        B.msgemm_destroy(plan)


def test_codes8_full_size_and_arbitrary_map():
    """cfg2's shape with 8-bit weights and a seeded 256-entry codebook, every row against the oracle."""
    m, k = 16384, 4096
    codes = inputs.make_codes8(m, k, seed=31)
    X = inputs.make_x(k, 1, "f16", seed=32)
    values = np.sort(np.random.default_rng(33).normal(size=256)).astype(np.float32).astype(np.float64) / 4
    dC, dX = torch_io.to_device(codes, "codes"), torch_io.to_device(X, "f16")
    plan = B.msgemm_plan_codes8(m, k, 1, "f16", "f16", 0, dC, None, values)
    try:
        Y = torch_io.empty_output(1, m, "f16")
        B.msgemm_run(plan, dX, k, Y, m)
        torch.cuda.synchronize()
        out = torch_io.to_host(Y)
    finally:
        B.msgemm_destroy(plan)
    ref = oracle.gemm_f64_codes8(codes, x_to_f64(X, "f16"), values)
    check(out, ref, "f16", "8-bit weights, cfg2 shape", elem_bound(codes, X, "f16", None, 0, values256=values))


def test_codes8_refusals():
    codes = inputs.make_codes8(64, 128, seed=1)
    dC = torch_io.to_device(codes, "codes")
    v = e4m3_finite()
    bad = v.copy(); bad[0x7f] = np.nan
    rc = lambda *a: B.msgemm_plan_codes8(*a, check=False)[0]
    assert rc(64, 128, 1, "f16", "f16", 0, dC, None, bad) == B.ERR_INVALID_ARG       # a NaN in the map
    assert rc(64, 128, 1, "i8", "i32", 0, dC, None, v) == B.ERR_UNSUPPORTED          # integer tables
    assert rc(64, 128, 1, "f16", "f16", 32, dC, dC, v) == B.ERR_UNSUPPORTED          # scale block below a k-tile
    plan = B.msgemm_plan_codes8(64, 128, 1, "f16", "f16", 0, dC, None, v)
    try:
        assert B.msgemm_lut_bytes(plan) == 0
        assert B.msgemm_plan_set_codebook(plan, UINT4, check=False) == B.ERR_UNSUPPORTED
        Y = torch_io.empty_output(1, 64, "f16")
        dX = torch_io.to_device(inputs.make_x(128, 1, "f16", seed=2), "f16")
        with pytest.raises(B.MsgemmError):
            B.msgemm_dequant_mfma_run(plan, dX, 128, Y, 64)
        with pytest.raises(B.MsgemmError):
            B.msgemm_build_lut(plan, dX, 128, Y)
    finally:
        B.msgemm_destroy(plan)


# ---------------------------------------------------------------------------
# the dense matrix-core comparison kernel (not msGeMM) computes the same Y

@pytest.mark.parametrize("m,k,b,xd,sg", [
    (300, 256, 5, "f16", 0),
    (257, 512, 64, "f16", 128),
    (513, 384, 70, "bf16", 128),     # two column tiles, ragged rows
    (64, 1024, 16, "bf16", 256),
])
def test_dequant_mfma_comparison_kernel(m, k, b, xd, sg):
    codes = inputs.make_codes(m, k, seed=m + k)
    X = inputs.make_x(k, b, xd, seed=b)
    scales = inputs.make_scales(m, k, sg, seed=4) if sg else None
    ref = oracle_y(codes, X, xd, scales, sg)
    dC, dS, dX = torch_io.to_device(codes, "codes"), torch_io.to_device(scales, "scales"), torch_io.to_device(X, xd)
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], 2, sg, dC, dS)
    try:
        Y = torch_io.empty_output(b, m, Y_OF_X[xd], ldy=m + 3)
        Y.fill_(-3)
        B.msgemm_dequant_mfma_run(plan, dX, k, Y, m + 3)
        torch.cuda.synchronize()
        out = torch_io.to_host(Y)
    finally:
        B.msgemm_destroy(plan)
    check(np.ascontiguousarray(out[:, :m]), ref, xd, "dequant+MFMA", elem_bound(codes, X, xd, scales, sg))


def test_dequant_mfma_unsupported_dtypes():
    dC = torch.zeros(64 * 32, dtype=torch.uint8, device="cuda:0")
    X = torch.zeros(64, dtype=torch.int8, device="cuda:0")
    Y = torch.zeros(64, dtype=torch.int32, device="cuda:0")
    plan = B.msgemm_plan(64, 64, 1, "i8", "i32", 2, 0, dC)
    try:
        with pytest.raises(B.MsgemmError) as e:
            B.msgemm_dequant_mfma_run(plan, X, 64, Y, 64)
        assert e.value.status == B.ERR_UNSUPPORTED
    finally:
        B.msgemm_destroy(plan)


def test_calibration_lds_read_entry_point():
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for width in (4, 8, 16):
        assert B.msgemm_calib_lds_read(width, 64, sink) == cus * 1024 * 64 * width
    torch.cuda.synchronize()
    assert int(sink[0]) == 0
    for width, reads in ((3, 64), (16, 0), (16, 12), (16, (1 << 20) + 8)):
        with pytest.raises(B.MsgemmError):
            B.msgemm_calib_lds_read(width, reads, sink)
    with pytest.raises(B.MsgemmError):
        B.msgemm_calib_lds_read(16, 64, None)


def test_calibration_lookup_add_entry_point():
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert B.msgemm_calib_lookup_add(3, sink) == cus * 8 * 64 * 128 * 3
    torch.cuda.synchronize()
    assert int(sink[0]) == 0
    for tiles in (0, -1, (1 << 16) + 1):
        with pytest.raises(B.MsgemmError):
            B.msgemm_calib_lookup_add(tiles, sink)
    with pytest.raises(B.MsgemmError):
        B.msgemm_calib_lookup_add(1, None)


def test_calibration_stream_read_entry_point():
    """The measurement aid accepts whole multiples of its launch footprint only and leaves the sink alone."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    unit = cus * 8 * 1024
    buf = torch.zeros(3 * unit, dtype=torch.uint8, device="cuda:0")
    sink = torch.full((4,), 7, dtype=torch.int32, device="cuda:0")
    B.msgemm_calib_stream_read(buf, 3 * unit, sink)
    B.msgemm_calib_stream_read(buf, unit, sink)
    torch.cuda.synchronize()
    assert sink.cpu().tolist() == [7, 7, 7, 7]
    for bad in (0, unit - 1024, unit + 16):
        with pytest.raises(B.MsgemmError):
            B.msgemm_calib_stream_read(buf, bad, sink)
    with pytest.raises(B.MsgemmError):
        B.msgemm_calib_stream_read(buf.data_ptr() + 4, unit, sink)


def test_calibration_stream_read_shape_entry_point():
    """The yardstick with its launch shape as parameters: whole loads per wavefront only, sink left alone."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    nbytes = cus * 16 * 1024 * 8            # 16 wavefronts per compute unit, 8 loads of 1 KiB each
    buf = torch.zeros(nbytes, dtype=torch.uint8, device="cuda:0")
    sink = torch.full((4,), 7, dtype=torch.int32, device="cuda:0")
    for waves, wgs, depth, nt in ((8, 2, 4, 0), (16, 1, 8, 1), (4, 4, 2, 0), (8, 1, 16, 0), (4, 1, 1, 1)):
        B.msgemm_calib_stream_read_shape(buf, nbytes, sink, waves, wgs, depth, nt)
    torch.cuda.synchronize()
    assert sink.cpu().tolist() == [7, 7, 7, 7]
    bad = [(0, 1, 4), (17, 1, 4), (8, 0, 4), (8, 17, 4), (8, 2, 3), (8, 2, 16), (12, 1, 4)]  # (8, 2, 16): 8 loads, depth 16
    for waves, wgs, depth in bad:
        assert B.msgemm_calib_stream_read_shape(buf, nbytes, sink, waves, wgs, depth, 0, check=False) == B.ERR_INVALID_ARG
    assert B.msgemm_calib_stream_read_shape(buf, nbytes - 1024, sink, 8, 2, 4, 0, check=False) == B.ERR_INVALID_ARG
    assert B.msgemm_calib_stream_read_shape(None, nbytes, sink, 8, 2, 4, 0, check=False) == B.ERR_INVALID_ARG


# ---------------------------------------------------------------------------
# other 16-value encodings of the codes (only b(.) changes)

UINT4 = [float(i) for i in range(16)]
NONUNIFORM = [0.0, 0.125, 0.25, 0.5, 1.0, 1.5, 2.5, 4.0, -6.0, -3.0, -2.0, -1.25, -0.75, -0.375, -0.1875, -0.0625]

CODEBOOK_CASES = [
    # m, k, b, xd, sg, d, variant
    (700, 768, 1, "f16", 128, 2, B.VARIANT_FUSED_LDS),     # single-column fused kernel, several k-tiles
    (300, 520, 2, "f32", 0, 2, B.VARIANT_FUSED_LDS),       # two column passes
    (515, 512, 9, "f16", 128, 2, B.VARIANT_FUSED_LDS16),   # batched kernel, fp16 table values
    (300, 260, 5, "bf16", 0, 2, B.VARIANT_FUSED_LDS16),
    (260, 256, 6, "f32", 0, 2, B.VARIANT_FUSED_LDS),       # 4-column fp32 kernel
    (64, 96, 3, "f16", 32, 1, B.VARIANT_GLOBAL_LUT),
    (64, 96, 3, "f32", 0, 3, B.VARIANT_GLOBAL_LUT),
    (64, 100, 18, "f16", 0, 3, B.VARIANT_GLOBAL_LUT),      # tables built on the matrix cores
]


@pytest.mark.parametrize("pipelined", [0, 1])
@pytest.mark.parametrize("table", [UINT4, NONUNIFORM])
@pytest.mark.parametrize("m,k,b,xd,sg,d,variant", CODEBOOK_CASES)
def test_codebook_against_oracle(m, k, b, xd, sg, d, variant, table, pipelined):
    if pipelined and variant != B.VARIANT_FUSED_LDS16:
        pytest.skip("only the batched kernel has a pipelined form")
    codes = inputs.make_codes(m, k, seed=m + k + 1)
    X = inputs.make_x(k, b, xd, seed=k + b + 3)
    scales = inputs.make_scales(m, k, sg, seed=13) if sg else None
    dC, dS, dX = torch_io.to_device(codes, "codes"), torch_io.to_device(scales, "scales"), torch_io.to_device(X, xd)
    plan = B.msgemm_plan(m, k, b, xd, Y_OF_X[xd], d, sg, dC, dS, variant, options={"batched_form": 1 + pipelined})
    try:
        assert B.msgemm_plan_get_info(plan)["variant"] == variant
        Y = torch_io.empty_output(b, m, Y_OF_X[xd])
        B.msgemm_plan_set_codebook(plan, table)
        B.msgemm_run(plan, dX, k, Y, m)
        torch.cuda.synchronize()
        ref = oracle.gemm_f64(codes, x_to_f64(X, xd), scales, sg, codebook=table)
        t16 = variant == B.VARIANT_FUSED_LDS16
        check(torch_io.to_host(Y), ref, xd, "codebook", elem_bound(codes, X, xd, scales, sg, table16=t16, codebook=table))
        # back to the paper's encoding
        B.msgemm_plan_set_codebook(plan, None)
        B.msgemm_run(plan, dX, k, Y, m)
        torch.cuda.synchronize()
        check(torch_io.to_host(Y), oracle_y(codes, X, xd, scales, sg), xd, "codebook restored",
              elem_bound(codes, X, xd, scales, sg, table16=t16))
    finally:
        B.msgemm_destroy(plan)


@pytest.mark.parametrize("b", [2, 32])
def test_codebook_table_build_against_phase1_reference(b):
    m, k, d = 8, 128, 2
    codes = inputs.make_codes(m, k, seed=1)
    X = inputs.make_x(k, b, "f16", seed=2)
    plan = B.msgemm_plan(m, k, b, "f16", "f16", d, 0, torch_io.to_device(codes, "codes"), None, B.VARIANT_GLOBAL_LUT)
    try:
        B.msgemm_plan_set_codebook(plan, NONUNIFORM)
        G = oracle.lut_groups(k, d, 0)
        L = torch.empty((G, 16 ** d, b), dtype=torch.float32, device="cuda:0")
        B.msgemm_build_lut(plan, torch_io.to_device(X, "f16"), k, L)
        torch.cuda.synchronize()
        ref = oracle.lut_build(X.astype(np.float64), d, 0, codebook=NONUNIFORM)
        # dyadic table values times fp16 activations: products exact, one rounding of the sum
        assert np.array_equal(L.cpu().numpy(), ref.astype(np.float32))
    finally:
        B.msgemm_destroy(plan)


def test_codebook_is_refused_where_it_cannot_apply():
    dC = torch.zeros(64 * 32, dtype=torch.uint8, device="cuda:0")
    plan = B.msgemm_plan(64, 64, 4, "i8", "i32", 2, 0, dC, None, B.VARIANT_AUTO)
    try:
        assert B.msgemm_plan_set_codebook(plan, UINT4, check=False) == B.ERR_UNSUPPORTED
        assert B.msgemm_plan_set_codebook(plan, None, check=False) == B.OK
    finally:
        B.msgemm_destroy(plan)
    plan = B.msgemm_plan(128, 128, 4, "f16", "f16", 2, 0, torch.zeros(128 * 64, dtype=torch.uint8, device="cuda:0"),
                         None, B.VARIANT_AUTO)
    try:
        bad = list(UINT4)
        bad[3] = float("nan")
        assert B.msgemm_plan_set_codebook(plan, bad, check=False) == B.ERR_INVALID_ARG
        B.msgemm_plan_set_codebook(plan, UINT4)
        X = torch.zeros((4, 128), dtype=torch.float16, device="cuda:0")
        Y = torch_io.empty_output(4, 128, "f16")
        with pytest.raises(B.MsgemmError):
            B.msgemm_dequant_mfma_run(plan, X, 128, Y, 128)
    finally:
        B.msgemm_destroy(plan)
    assert B.msgemm_plan_set_codebook(None, UINT4, check=False) == B.ERR_INVALID_ARG


# ---------------------------------------------------------------------------
# seeded random shapes: every variant, dtype, scale block and batch width mixed

def _random_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        xd = ["f32", "f16", "bf16", "i8"][rng.integers(4)]
        m = int(rng.integers(1, 1500))
        sg = 0 if xd == "i8" else int([0, 0, 32, 64, 128, 256][rng.integers(6)])
        k = 2 * int(rng.integers(1, 700))
        if sg:
            k = max(sg, (k // sg) * sg)  # scale blocks divide k
        b = int([1, 1, 2, 3, 5, 8, 9, 16, 17, 24][rng.integers(10)])
        variant = [B.VARIANT_AUTO, B.VARIANT_FUSED_LDS, B.VARIANT_FUSED_LDS16, B.VARIANT_GLOBAL_LUT,
                   B.VARIANT_GLOBAL_LUT_HALF][rng.integers(5)]
        d = 2
        if variant in (B.VARIANT_GLOBAL_LUT, B.VARIANT_GLOBAL_LUT_HALF):
            d = int(rng.integers(1, 4))
        if variant == B.VARIANT_FUSED_LDS16 and xd == "f32":
            continue  # no 16-bit tables for fp32 activations
        if variant == B.VARIANT_FUSED_LDS and sg % 128 or variant == B.VARIANT_FUSED_LDS16 and sg % 64:
            continue  # the fused kernels need scale blocks of whole k-tiles (128 resp. 64 columns)
        pipe = int(rng.integers(2))
        cases.append((m, k, b, xd, sg, d, variant, pipe))
    return cases


@pytest.mark.parametrize("m,k,b,xd,sg,d,variant,pipe", _random_cases(160, seed=20231006))
def test_random_shapes(m, k, b, xd, sg, d, variant, pipe):
    codes = inputs.make_codes(m, k, seed=m * 31 + k)
    X = inputs.make_x(k, b, xd, seed=k * 7 + b)
    scales = inputs.make_scales(m, k, sg, seed=m + b) if sg else None
    ref = oracle_y(codes, X, xd, scales, sg)
    out, info = run_gpu(codes, X, xd, scales, sg, 0 if variant == B.VARIANT_AUTO else d, variant, ldx_pad=2, ldy_pad=1,
                        options={"batched_form": 1 + pipe})
    if variant != B.VARIANT_AUTO:
        assert info["variant"] == variant
    bnd = elem_bound(codes, X, xd, scales, sg, table16=info["variant"] == B.VARIANT_FUSED_LDS16)
    if bnd is not None and info["variant"] == B.VARIANT_GLOBAL_LUT_HALF:
        bnd = 2 * bnd  # an entry of the missing half is c S(j) - L: one more rounding, of magnitude up to the group's sum
    check(out, ref, xd, f"random shape {m}x{k}x{b} {xd} sg={sg} d={d} variant={variant}", bnd)


def _random_batched_cases(count, seed):
    """Larger batched problems with the forms that place or deal their workgroups by the shape of the problem."""
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        xd = ["f16", "bf16", "i8"][rng.integers(3)]
        m = int(rng.integers(1500, 30000))
        sg = 0 if xd == "i8" else int([0, 32, 64, 128, 256][rng.integers(5)])
        k = 2 * int(rng.integers(300, 4000))
        if sg:
            k = max(sg, (k // sg) * sg)
        b = int(rng.integers(3, 70))
        if m * k * b > 3e9:
            continue  # (the oracle stays under a second)
        which = int(rng.integers(4))
        options = [{"batched_form": 2, "batched_deal": 2}, {"batched_deal": 2},
                   {"reduce_mode": 4, "batched_form": int(rng.integers(1, 3)), "panels_per_workgroup": int(rng.integers(1, 9)),
                    "batched_segments": int(rng.integers(2, 9))},
                   {"reduce_mode": 4}][which]
        if sg == 32 and options.get("batched_form") == 1:
            options["batched_form"] = 2  # (scale blocks of 32 columns: only the pipelined form has k-tiles that small)
        cases.append((m, k, b, xd, sg, options))
    return cases


@pytest.mark.parametrize("m,k,b,xd,sg,options", _random_batched_cases(24, seed=61782310))
def test_random_batched_shapes_dealt_and_xcd_local(m, k, b, xd, sg, options):
    """Seeded random batched problems through the pipelined form with its k-tiles dealt evenly and through the XCD-local
    reduction, where the shape allows them (elsewhere the request falls back to the library's choice): whatever the
    plan turns out to be, the result is the oracle's."""
    codes = inputs.make_codes(m, k, seed=m * 31 + k)
    X = inputs.make_x(k, b, xd, seed=k * 7 + b)
    scales = inputs.make_scales(m, k, sg, seed=m + b) if sg else None
    ref = oracle_y(codes, X, xd, scales, sg)
    out, info = run_gpu(codes, X, xd, scales, sg, 2, B.VARIANT_FUSED_LDS16, ldx_pad=2, ldy_pad=1, options=options)
    assert info["variant"] == B.VARIANT_FUSED_LDS16
    check(out, ref, xd, f"random batched shape {m}x{k}x{b} {xd} sg={sg} {options}", elem_bound(codes, X, xd, scales, sg, table16=True))
