#!/usr/bin/env python3
"""msGeMM benchmark: one JSON line on stdout.

A step is one pass of the whole hot path (table build, code stream, gather,
scale, k-tile reduction, output conversion = one ``msgemm_run``) over one batch
of synthetic activations.  The default workload is the b = 1 GEMV
(m = 16384, k = 4096, int4 weights, fp16 activations).  Inputs are resident in
HBM before the timed region.  To keep the code stream cold, successive steps
rotate through enough independent weight copies (> 1 GiB in total) to defeat
the 256 MB on-package cache, as a chain of layers would in a model.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg2] [--mode graph|eager]
                    [--hot] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

LDS_PEAK_GBS = 256 * 256 * 2.4  # 256 compute units x 256 B per clock (gfx950 LDS read width) x 2.4 GHz

# HBM bytes per launch of the dominant kernel of each configuration, reads + writes, from two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE), each scaled by what the same counter reads for a
# 64 MiB elementwise kernel in the same run: recorded in this table, one line per configuration.
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")


def measured_traffic(config: str):
    """(bytes per launch, kernel name) recorded for `config`, or (None, None)."""
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                w = line.split()
                if len(w) >= 5 and not line.startswith("#") and w[0] == config:
                    return int(w[2]) + int(w[3]), w[1]
    except OSError:
        pass
    return None, None


def parity_spot_check(cfg, codes, X, scales, Y_host, torch_io, max_macs=4e9):
    """The output of the seeded weight copy against the oracle: every row when that is quick, else the first
    and last rows and a seeded sample.  Bit-exact for int8, else the relative L2 error against the bound."""
    import oracle
    m, k, b = cfg["m"], cfg["k"], cfg["b"]
    if m * k * b <= max_macs:
        rows = np.arange(m)
    else:
        n = max(256, int(max_macs // (k * b)))
        rows = np.unique(np.concatenate([[0, m - 1], np.random.default_rng(7).choice(m, size=n, replace=False)]))
    c = codes[rows]
    s = None if scales is None else scales[rows]
    got = np.ascontiguousarray(Y_host[:, rows])
    if cfg["x"] == "i8":
        ok = bool(np.array_equal(got, oracle.gemm_i32(c, X)))
        return {"rows": int(len(rows)), "bit_exact": ok, "ok": ok}
    Xd = oracle.bf16_bits_to_f64(X) if cfg["x"] == "bf16" else X.astype(np.float64)
    err = oracle.rel_l2(torch_io.to_f64(got), oracle.gemm_f64(c, Xd, s, cfg["scale_group"]))
    bound = {"f32": 1e-5, "f16": 2e-3, "bf16": 1.6e-2}[cfg["y"]]
    return {"rows": int(len(rows)), "rel_l2": err, "bound": bound, "ok": bool(err <= bound)}


def algorithmic_bytes(cfg) -> int:
    """What the method itself must move per GeMM (Section 4.2: k*b + m*k element
    accesses, the same as a plain GeMM): the 4-bit codes once, the scales, X, Y."""
    m, k, b = cfg["m"], cfg["k"], cfg["b"]
    sx = {"f32": 4, "f16": 2, "bf16": 2, "i8": 1}[cfg["x"]]
    sy = {"f32": 4, "f16": 2, "bf16": 2, "i32": 4}[cfg["y"]]
    total = m * k // 2 + k * b * sx + m * b * sy
    if cfg["scale_group"]:
        total += m * (k // cfg["scale_group"]) * 2
    return total


def cpu_baseline(cfg, codes, X, scales, budget_s=12.0):
    """The oracle as it stands, on the host cores, on a bounded sample."""
    import oracle
    m, k, b = cfg["m"], cfg["k"], cfg["b"]
    # rows sampled so that one oracle pass is ~<= 2e9 multiply-adds
    rows = m if m * k * b <= 2e9 else max(256, int(2e9 // (k * b)))
    c = codes[:rows]
    s = None if scales is None else scales[:rows]
    if cfg["x"] == "i8":
        run = lambda: oracle.gemm_i32(c, X)
    else:
        Xd = oracle.bf16_bits_to_f64(X) if cfg["x"] == "bf16" else X.astype(np.float64)
        run = lambda: oracle.gemm_f64(c, Xd, s, cfg["scale_group"])
    run()  # warm-up
    reps, t_total = 0, 0.0
    best = float("inf")
    while t_total < budget_s and reps < 50:
        t0 = time.perf_counter()
        run()
        dt = time.perf_counter() - t0
        best = min(best, dt)
        t_total += dt
        reps += 1
    mean = t_total / reps
    cores = oracle.num_threads()
    # the same on one core (a few passes): what a single host thread does
    oracle.set_threads(1)
    try:
        run()
        t1, n1 = 0.0, 0
        while t1 < 3.0 and n1 < 5:
            t0 = time.perf_counter()
            run()
            t1 += time.perf_counter() - t0
            n1 += 1
    finally:
        oracle.set_threads(cores)
    return {
        "value": 2.0 * rows * k * b / mean / 1e12,
        "unit": "TOPS",
        "cores": cores,
        "kind": "oracle",
        "sample": f"{rows} of {m} rows x all k x all b, {reps} passes, mean {mean * 1e3:.2f} ms, best {best * 1e3:.2f} ms",
        "one_core": {"value": 2.0 * rows * k * b / (t1 / n1) / 1e12, "unit": "TOPS", "passes": n1},
    }


def stream_read_ceiling(B, torch, stream, nbytes, n_copies, steps):
    """The same timing protocol (HIP graph, rotating cold buffers, events on the
    launch stream) around a kernel that only reads `nbytes`: what this device
    gives a single launch that streams that many cold bytes and does nothing else."""
    unit = 256 * 8 * 1024  # bytes one load of every wavefront covers on a 256-CU device
    nbytes = max(unit, nbytes // unit * unit)
    bufs = [torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device="cuda:0") for _ in range(n_copies)]
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    for i in range(10):
        B.msgemm_calib_stream_read(bufs[i % n_copies], nbytes, sink)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        for i in range(steps):
            B.msgemm_calib_stream_read(bufs[i % n_copies], nbytes, sink)
    graph.replay()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        ev0.record(stream)
        graph.replay()
        ev1.record(stream)
    torch.cuda.synchronize()
    us = ev0.elapsed_time(ev1) * 1e3 / steps
    return {"bytes": nbytes, "us": us, "GB/s": nbytes / (us * 1e-6) / 1e9}


def stream_read_sweep(B, torch, stream, nbytes, n_copies, steps):
    """The read-only yardstick over launch shapes, loads in flight and cache policy, each timed like a step
    (HIP graph, rotating cold buffers, events on the launch stream); also an empty launch."""
    bufs = [torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device="cuda:0") for _ in range(n_copies)]
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")

    def timed(launch):
        for i in range(5):
            launch(i)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(steps):
                launch(i)
        graph.replay()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            with torch.cuda.stream(stream):
                ev0.record(stream)
                graph.replay()
                ev1.record(stream)
            torch.cuda.synchronize()
            best = min(best, ev0.elapsed_time(ev1) * 1e3 / steps)
        return best

    rows = []
    for waves, wgs, depth, nt in [(8, 1, 2, 0), (8, 1, 4, 0), (8, 1, 8, 0), (8, 1, 16, 0), (16, 1, 4, 0), (16, 1, 8, 0),
                                  (8, 2, 4, 0), (8, 2, 8, 0), (4, 2, 8, 0), (4, 2, 16, 0), (4, 4, 4, 0), (4, 4, 8, 0),
                                  (4, 8, 4, 0), (4, 8, 2, 0), (8, 1, 4, 1), (8, 1, 8, 1), (8, 1, 16, 1), (4, 8, 4, 1)]:
        us = timed(lambda i: B.msgemm_calib_stream_read_shape(bufs[i % n_copies], nbytes, sink, waves, wgs, depth, nt))
        rows.append({"waves_per_workgroup": waves, "workgroups_per_cu": wgs, "loads_in_flight": depth,
                     "non_temporal": nt, "us": round(us, 3), "GB/s": round(nbytes / (us * 1e-6) / 1e9, 1)})
    hot = timed(lambda i: B.msgemm_calib_stream_read_shape(bufs[0], nbytes, sink, 8, 1, 8, 0))
    empty = timed(lambda i: B.msgemm_calib_lds_read(4, 8, sink))  # a launch that touches no memory at all
    return {"bytes": nbytes, "rows": rows, "hot_same_buffer_us": round(hot, 3), "launch_without_memory_us": round(empty, 3)}


def lds_read_ceiling(B, torch, stream, width=16, reads=4096, launches=400):
    """Measured LDS read bandwidth of the device: conflict-free `width`-byte reads by 16 wavefronts on
    every compute unit (msgemm_calib_lds_read), HIP events on the launch stream; some 50 ms of launches, like a
    batched configuration's timed region (the clocks settle over the first 10 ms of sustained load)."""
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    nbytes = 0
    with torch.cuda.stream(stream):
        for _ in range(3):
            nbytes = B.msgemm_calib_lds_read(width, reads, sink, stream)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for _ in range(launches):
            B.msgemm_calib_lds_read(width, reads, sink, stream)
        ev1.record(stream)
    torch.cuda.synchronize()
    us = ev0.elapsed_time(ev1) * 1e3 / launches
    return {"width_bytes": width, "bytes": nbytes, "us": us, "GB/s": nbytes / (us * 1e-6) / 1e9}


def lookup_add_ceiling(B, torch, stream, tiles=64, launches=300):
    """Measured rate of the batched kernels' inner loop alone (msgemm_calib_lookup_add: a 16-byte look-up and its
    two matrix-core adds, 8 wavefronts per compute unit, no code stream, no table build): lane look-ups per second,
    over some 50 ms of launches like the timed region it is compared with."""
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    n = 0
    with torch.cuda.stream(stream):
        for _ in range(2):
            n = B.msgemm_calib_lookup_add(tiles, sink, stream)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for _ in range(launches):
            B.msgemm_calib_lookup_add(tiles, sink, stream)
        ev1.record(stream)
    torch.cuda.synchronize()
    us = ev0.elapsed_time(ev1) * 1e3 / launches
    return {"lane_lookups": n, "us": us, "Glookups/s": n / (us * 1e-6) / 1e9}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--shape", default=None, metavar="M,K,B,X,Y,SG",
                    help="an ad-hoc problem instead of a named configuration, e.g. 4096,4096,1,f16,f16,0 "
                         "(x / y: f32, f16, bf16, i8 / i32; SG: scale block or 0; same input recipe, seed 21)")
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph")
    ap.add_argument("--hot", action="store_true", help="one weight copy (cache-resident), labelled as such")
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--d", type=int, default=None)
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="a field of msgemm_plan_options_t (a particular kernel form), e.g. batched_segments=16")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle legs (cpu_baseline and the parity spot check)")
    ap.add_argument("--mfma", action="store_true",
                    help="time the dequantise + MFMA comparison kernel instead of the msGeMM path (labelled as such)")
    ap.add_argument("--no-ceiling", action="store_true",
                    help="skip the plain stream-read kernel that measures the practical HBM ceiling")
    ap.add_argument("--lib", default=None,
                    help="time another build of the library (a measurement build made with "
                         "`python -m paper_2310_06178_amd.build -D... --out PATH`); implies --no-cpu when it computes nothing")
    ap.add_argument("--ceiling-sweep", action="store_true",
                    help="also time the read-only yardstick over launch shapes, loads in flight and cache policy")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 64 MiB elementwise copy (untimed): gives hardware-counter runs a kernel of known traffic")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path has no multi-GPU part); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2310_06178_amd import binding as B
    from paper_2310_06178_amd import inputs, torch_io

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    if args.lib:
        B.LIB_PATH = os.path.abspath(args.lib)
    B.load()
    torch.cuda.set_device(0)

    if args.shape:
        sm, sk, sb, sx, sy, ssg = args.shape.split(",")
        args.config = "shape " + args.shape
        inputs.CONFIGS[args.config] = dict(m=int(sm), k=int(sk), b=int(sb), x=sx, y=sy, scale_group=int(ssg), d=2, seed=21)
    cfg, codes, X, scales = inputs.make_config(args.config)
    m, k, b = cfg["m"], cfg["k"], cfg["b"]
    steps_from_warmup = args.steps is None and b > 1
    if args.steps is None:
        args.steps = 2000  # (batches: replaced below by a count that makes the timed region about 60 ms)
    d = cfg["d"] if args.d is None else args.d
    code_bytes = m * k // 2
    n_copies = 1 if args.hot else (1 << 30) // code_bytes + 2
    n_copies = max(1, min(n_copies, 64))

    plan_options = {n: int(v) for n, v in (o.split("=", 1) for o in args.option)} or None
    dX = torch_io.to_device(X, cfg["x"])
    dS = torch_io.to_device(scales, "scales")
    plans = []
    rng = np.random.default_rng(1234)
    for i in range(n_copies):
        # independent weight bytes per copy (copy 0 is the seeded config itself)
        ci = codes if i == 0 else rng.integers(0, 256, size=codes.shape, dtype=np.uint8)
        dC = torch_io.to_device(ci, "codes")
        plans.append(B.msgemm_plan(m, k, b, cfg["x"], cfg["y"], d, cfg["scale_group"], dC, dS, args.variant,
                                   options=plan_options))
        torch.cuda.synchronize()
        del dC
    info = B.msgemm_plan_get_info(plans[0])
    Y = torch_io.empty_output(b, m, cfg["y"])

    run = B.msgemm_dequant_mfma_run if args.mfma else B.msgemm_run

    def step(i):
        run(plans[i % n_copies], dX, k, Y, m)

    torch.cuda.synchronize()
    t_warm = time.perf_counter()
    for i in range(max(args.warmup, 1)):
        step(i)
    torch.cuda.synchronize()
    if steps_from_warmup:
        # The device's clocks take some 10 ms of sustained load to settle after an idle gap (a step measures up to a
        # tenth slower inside that transient), so the timed region of a batched configuration is made about 60 ms
        # long: K from the warm-up's time per step, between 100 and 4000.  --steps overrides.
        per_step = (time.perf_counter() - t_warm) / max(args.warmup, 1)
        args.steps = int(min(4000, max(100, round(0.06 / max(per_step, 1e-6)))))
    if args.calib_copy:
        src = torch.ones(64 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)  # an elementwise kernel: reads 64 MiB, writes 64 MiB
        torch.cuda.synchronize()

    mode = args.mode
    graph = None
    stream = torch.cuda.Stream()
    if mode == "graph":
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(args.steps):
                    step(i)
            graph.replay()  # untimed replay: instantiation / upload costs stay outside
            torch.cuda.synchronize()
        except Exception as e:  # capture not possible: time the eager loop instead
            print(f"bench.py: graph capture failed ({e}); timing eager launches", file=sys.stderr)
            graph, mode = None, "eager"

    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        ev0.record(stream)
        if graph is not None:
            graph.replay()
        else:
            for i in range(args.steps):
                step(i)
        ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = ev0.elapsed_time(ev1)

    # the last step ran on plan (steps-1) % n_copies; copy 0 holds the seeded weights: run it once more,
    # eagerly, and compare that output with the oracle
    Y.zero_()
    step(0)
    torch.cuda.synchronize()
    spot = None if args.no_cpu else parity_spot_check(cfg, codes, X, scales, torch_io.to_host(Y), torch_io)

    ms_per_step = wall * 1e3 / args.steps
    kernel_us = gpu_ms * 1e3 / args.steps  # HIP events on the launch stream
    alg = algorithmic_bytes(cfg)
    achieved = alg / (kernel_us * 1e-6) / 1e9
    tops = 2.0 * m * k * b / (wall / args.steps) / 1e12

    out = {
        "metric": "effective TOPS (2mkb/t), int4-weight LUT GeMM (msGeMM)" if not args.mfma
                  else "effective TOPS (2mkb/t), int4 dequantise + MFMA comparison kernel (not msGeMM)",
        "value": tops,
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"f32": "f32", "f16": "f32", "bf16": "f32", "i8": "int32"}[cfg["x"]],
        "data": "synthetic",
        "library": os.path.relpath(B.LIB_PATH, ROOT),
        "config": {
            "workload": f"{args.config}: m={m} k={k} b={b} int4 W, {cfg['x']} X, {cfg['y']} Y, "
                        f"scale_group={cfg['scale_group']}, d={info['d']}",
            "variant": "dequant_mfma_comparison" if args.mfma else
                       {1: "global_lut", 2: "fused_lds", 3: "fused_lds16", 4: "global_lut_half"}[info["variant"]],
            "tile_rows": info["tile_rows"], "tile_groups": info["tile_groups"],
            "split_k": info["split_k"], "col_chunk": info["col_chunk"],
            "weight_copies_rotated": n_copies,
            "cache_state": "hot (single weight copy)" if args.hot else "cold (rotating copies > 1 GiB)",
            "launch": mode,
            "plan_options": plan_options,
            "paper_op_ratio": m * k / (16 ** info["d"] * k + (k / info["d"] - 1) * m),
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": None if args.mfma else measured_traffic(args.config)[0],
            "traffic_kernel": None if args.mfma else measured_traffic(args.config)[1],
            "algorithmic_bytes": alg,
            "kernel_us": kernel_us,
        },
    }
    if not args.mfma and info["variant"] == 3:
        # batches: the gather reads one 16-byte table entry (8 fp16 columns) per row, group and column pass from
        # LDS; peak = 256 compute units x 256 B per clock x 2.4 GHz (gfx950 LDS read width; SQ_LDS_IDX_ACTIVE
        # counts 4.3 cycles per 1 KiB ds_read_b128 in the profile of this kernel)
        lds_bytes = float(m) * (k // 2) * ((b + 7) // 8) * 16
        lds_peak = LDS_PEAK_GBS
        out["roofline"]["lds"] = {"bound": "lds", "achieved": lds_bytes / (kernel_us * 1e-6) / 1e9, "peak": lds_peak,
                                  "unit": "GB/s", "frac": lds_bytes / (kernel_us * 1e-6) / 1e9 / lds_peak,
                                  "table_bytes_gathered": lds_bytes}
        if not args.no_ceiling:
            # the same reads without anything else: what the LDS of this device delivers (measured in this run)
            measured = lds_read_ceiling(B, torch, stream)
            out["roofline"]["lds"]["measured_read_kernel"] = measured
            out["roofline"]["lds"]["frac_of_measured"] = out["roofline"]["lds"]["achieved"] / measured["GB/s"]
            # and the look-up + add instruction mix without anything else: the practical ceiling of the gather
            mix = lookup_add_ceiling(B, torch, stream)
            lookups = lds_bytes / 16.0
            out["roofline"]["lds"]["measured_lookup_add_kernel"] = mix
            out["roofline"]["lds"]["frac_of_lookup_add"] = lookups / (kernel_us * 1e-6) / 1e9 / mix["Glookups/s"]
    if graph is not None and not args.no_ceiling and not args.hot:
        try:
            out["roofline"]["stream_read_kernel"] = stream_read_ceiling(B, torch, stream, code_bytes, n_copies, args.steps)
        except Exception as e:  # a device with another CU count: the figure is optional
            print(f"bench.py: stream-read ceiling not measured ({e})", file=sys.stderr)
    if args.ceiling_sweep and graph is not None:
        out["roofline"]["stream_read_sweep"] = stream_read_sweep(B, torch, stream, code_bytes, n_copies, min(args.steps, 400))
    if not args.no_cpu:
        out["parity_spot_check"] = spot
        out["cpu_baseline"] = cpu_baseline(cfg, codes, X, scales)

    for p in plans:
        B.msgemm_destroy(p)
    print(json.dumps(out), flush=True)
    if spot is not None and not spot["ok"]:
        print(f"bench.py: the timed path does not match the oracle: {spot}", file=sys.stderr)
        return 4
    return 0


if __name__ == "__main__":
    sys.exit(main())
