"""msgemm_run_static, the entry point that allocates nothing (partial sums in a static device array), against
msgemm_run on the same plans and against the oracle: two calls in a row, the second on a smaller problem."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_06178_amd import binding as B
from paper_2310_06178_amd import inputs, torch_io

pytestmark = pytest.mark.gpu

TOL = {"f16": 2e-3, "i8": 0.0}


def _both_ways(m, k, b, xd, sg, seed):
    yd = {"f16": "f16", "i8": "i32"}[xd]
    codes = inputs.make_codes(m, k, seed=seed)
    X = inputs.make_x(k, b, xd, seed=seed + 1)
    scales = inputs.make_scales(m, k, sg, seed=seed + 2) if sg else None
    dC, dS, dX = torch_io.to_device(codes, "codes"), torch_io.to_device(scales, "scales"), torch_io.to_device(X, xd)
    plan = B.msgemm_plan(m, k, b, xd, yd, 2, sg, dC, dS)
    try:
        info = B.msgemm_plan_get_info(plan)
        assert info["variant"] in (B.VARIANT_FUSED_LDS, B.VARIANT_FUSED_LDS16) and info["split_k"] > 1
        Y1 = torch_io.empty_output(b, m, yd)
        Y2 = torch_io.empty_output(b, m, yd, ldy=m + 5)
        Y1.fill_(-3)
        Y2.fill_(-3)
        B.msgemm_run(plan, dX, k, Y1, m)
        B.msgemm_run_static(plan, dX, k, Y2, m + 5)
        torch.cuda.synchronize()
        y1, y2 = torch_io.to_host(Y1), torch_io.to_host(Y2)
    finally:
        B.msgemm_destroy(plan)
    minus3 = torch_io.to_host(torch.full((1,), -3, dtype=Y2.dtype))[0]
    assert np.all(y2[:, m:] == minus3), "output padding was written"
    y2 = np.ascontiguousarray(y2[:, :m])
    if xd == "i8":
        ref = oracle.gemm_i32(codes, X)
        assert np.array_equal(y1, ref) and np.array_equal(y2, ref)
        return
    ref = oracle.gemm_f64(codes, X.astype(np.float64), scales, sg)
    for y in (y1, y2):
        assert oracle.rel_l2(torch_io.to_f64(y), ref) <= TOL[xd]
    # the two entry points add the same partial sums, in another order at most: an output differs by the rounding
    # of the output type at most (one unit in the last place of fp16)
    a1, a2 = torch_io.to_f64(y1), torch_io.to_f64(y2)
    assert np.max(np.abs(a1 - a2) / np.maximum(np.abs(ref), 1e-3)) <= 2.0 ** -9


def test_static_scratch_entry_point_matches_msgemm_run_twice_in_a_row():
    _both_ways(4100, 2048, 1, "f16", 128, seed=50)     # single column, 16 k-tiles, 17 panels: 1.1 MB of partial sums
    _both_ways(700, 512, 1, "f16", 0, seed=60)         # then a smaller one over the same array
    _both_ways(1500, 1024, 9, "i8", 0, seed=70)        # a batched plan (two column passes), bit-exact
    _both_ways(300, 256, 1, "f16", 128, seed=80)


def test_static_scratch_entry_point_refusals():
    dC = torch.zeros(64 * 32, dtype=torch.uint8, device="cuda:0")
    X = torch.zeros(64, dtype=torch.float16, device="cuda:0")
    Y = torch.zeros(64, dtype=torch.float16, device="cuda:0")
    plan = B.msgemm_plan(64, 64, 1, "f16", "f16", 3, 0, dC, None, B.VARIANT_GLOBAL_LUT)
    try:
        assert B.msgemm_run_static(plan, X, 64, Y, 64, check=False) == B.ERR_UNSUPPORTED
    finally:
        B.msgemm_destroy(plan)
    plan = B.msgemm_plan(64, 64, 1, "f16", "f16", 2, 0, dC)
    try:
        assert B.msgemm_run_static(plan, X, 63, Y, 64, check=False) == B.ERR_INVALID_ARG
        assert B.msgemm_run_static(plan, None, 64, Y, 64, check=False) == B.ERR_INVALID_ARG
        assert B.msgemm_run_static(plan, X, 64, Y, 64, check=False) == B.OK   # a single k-tile: no partial sums at all
    finally:
        B.msgemm_destroy(plan)
    # more partial sums than the array holds: 64 k-tiles x 2 columns x 65536 rows x 4 bytes = 32 MiB
    m, k, b = 65536, 8192, 2
    big = torch.zeros(m * (k // 2), dtype=torch.uint8, device="cuda:0")
    plan = B.msgemm_plan(m, k, b, "f16", "f16", 2, 0, big, options={"k_tiles_per_workgroup": 1})
    try:
        info = B.msgemm_plan_get_info(plan)
        assert info["split_k"] * b * m * 4 > (16 << 20), "the case is meant to exceed the array"
        Xb = torch.zeros((b, k), dtype=torch.float16, device="cuda:0")
        Yb = torch.zeros((b, m), dtype=torch.float16, device="cuda:0")
        assert B.msgemm_run_static(plan, Xb, k, Yb, m, check=False) == B.ERR_UNSUPPORTED
        B.msgemm_run(plan, Xb, k, Yb, m)   # (the plan itself is fine)
    finally:
        B.msgemm_destroy(plan)
    torch.cuda.synchronize()
