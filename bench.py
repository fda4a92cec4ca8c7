#!/usr/bin/env python3
"""Benchmark of the CSR sparse matrix-vector product  y <- alpha*A*x + beta*y  on one MI355X.

One "step" is one spmv_csr_run() over one synthetic matrix (the whole hot path: every kernel of
the plan that spmv_csr_analyze() chose).  Timing follows the paper's protocol for its kernel
benchmark (section 3.3: warm-up runs, then the mean over the timed runs; defaults 3 and 50).

Inputs are resident in HBM before the timed region.  Matrices smaller than the 256 MB
last-level cache would be served from it when one copy is run back to back, so by default the
steps rotate over several disjoint copies of {rowptr, colidx, vals, x, y} (more than 512 MB in
total): `value` is that cold, HBM-bound rate; the cache-warm rate is reported beside it.

Prints ONE JSON line.  metric = effective GB/s over the algorithmic bytes
(vals + colidx + rowptr + x + y written, + y read when beta != 0); GFLOP/s = 2*nnz / time.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

import numpy as np

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
LLC_BYTES = 256 << 20           # last-level (memory-side) cache
ROTATE_TOTAL_BYTES = 640 << 20  # footprint the rotation must exceed


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="headline workload: one of the five configurations, 1..5")
    ap.add_argument("--plan", type=int, default=0, help="0 auto, 1 scalar, 2 vector, 3 binned, 4 adaptive, 5 merge, 6 windowed, 7 colblock, 8 twophase, 9 sell")
    ap.add_argument("--block-nnz", type=int, default=0)
    ap.add_argument("--rows-max", type=int, default=0)
    ap.add_argument("--items-per-chunk", type=int, default=0)
    ap.add_argument("--vector-lanes", type=int, default=0)
    ap.add_argument("--only", action="store_true", help="measure the headline workload only (skip the other configs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--spmm", type=int, default=0, metavar="LOG2ROWS",
                    help="run only the SpMM CSR product of the paper's shape with 2^LOG2ROWS rows and print its line")
    ap.add_argument("--two-pass-sweep", action="store_true",
                    help="run only the matrices that place the two-pass plan's thresholds (row-wise plan against plan 8) and print their lines")
    ap.add_argument("--formats", action="store_true", help="run only the COO / CSC / ELL products and print their lines")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the launch floor, the large uniform matrix and the paper-shaped sweep")
    ap.add_argument("--copies", type=int, default=0, help="override the number of rotating copies")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a kernel of known traffic, used to scale "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def kernels_sha256():
    import hashlib
    h = hashlib.sha256()
    # what the CSR matrix-vector product runs (the column-blocked plan multiplies with the coordinate kernel)
    for name in ("kernels.hip", "device_common.h", "row_phase.h", "kernels.h", "capi.cpp", "analysis.cpp", "analysis.h", "formats.hip",
                 "colblock.hip", "twophase.hip", "sell.hip"):
        h.update((ROOT / "paper_2603_07169_amd" / "csrc" / name).read_bytes())
    return h.hexdigest()


def recorded_traffic(workload):
    """HBM bytes one product really moves (FETCH_SIZE + WRITE_SIZE of every kernel of the plan, scaled by the copy
    calibration) from the committed counter summary, or None when there is none or the kernel sources have changed
    since it was taken."""
    f = ROOT / "profiles" / f"traffic_{workload}.txt"
    if not f.exists():
        return None
    kv = {}
    for line in f.read_text().splitlines():
        if ":" in line and not line.startswith("#"):
            k, v = line.split(":", 1)
            kv[k.strip()] = v.strip()
    if kv.get("csrc_sha256") != kernels_sha256():
        return None
    try:
        return float(kv["hbm_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def roofline_block(r):
    """The HBM roofline of one measured workload.  frac_effective = algorithmic CSR bytes / time / peak is the metric's
    ratio; a plan that moves fewer bytes than CSR's own arrays (16-bit window positions, row patterns) can push it past
    1, so it is no statement about the memory.  frac_real = bytes the counters saw / time / peak is that statement."""
    traffic = recorded_traffic(r["workload"])
    ms = r["ms_per_step"]
    return {"bound": "hbm", "peak": HBM_PEAK_GBPS, "unit": "GB/s", "kernel": r["kernel"],
            "algorithmic_bytes": r["algorithmic_bytes"], "achieved": r["GBps"], "frac_effective": r["GBps"] / HBM_PEAK_GBPS,
            "traffic": traffic, "real_GBps": None if traffic is None else traffic / ms / 1e6,
            "frac_real": None if traffic is None else traffic / ms / 1e6 / HBM_PEAK_GBPS,
            "traffic_over_algorithmic": None if traffic is None else traffic / r["algorithmic_bytes"]}


def dev(a):
    import torch
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()


class Resident:
    """`copies` disjoint device copies of one problem, each with its own handle."""

    def __init__(self, p, copies, params):
        import torch
        import paper_2603_07169_amd as s
        self.p = p
        self.sets = []
        self.analysis_ms = None
        for _ in range(copies):
            rowptr, colidx, vals, x = dev(p.rowptr), dev(p.colidx), dev(p.vals), dev(p.x)
            y = dev(p.y0) if p.y0 is not None else torch.zeros(p.m, dtype=torch.float32, device="cuda")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            A = s.CsrMatrix(p.m, p.n, rowptr, colidx, vals, s.SPMV_F32 if p.dtype == "f32" else s.SPMV_BF16, params)
            dt = (time.perf_counter() - t0) * 1e3       # create + analyze (synchronous), not part of the metric
            self.analysis_ms = dt if self.analysis_ms is None else min(self.analysis_ms, dt)
            self.sets.append((A, x, y))
        self.info = self.sets[0][0].info
        self.kernel = s.spmv_csr_main_kernel_name(self.sets[0][0].handle)

    def step(self, i, stream):
        A, x, y = self.sets[i % len(self.sets)]
        A.run(x, y, self.p.alpha, self.p.beta, stream)

    def close(self):
        for A, _, _ in self.sets:
            A.close()
        self.sets = []


def time_steps(res, steps, warmup, rotate=True):
    """Mean ms per step over `steps` steps, HIP events on the launch stream."""
    import torch
    stream = torch.cuda.current_stream()
    h = stream.cuda_stream
    idx = (lambda i: i) if rotate else (lambda i: 0)
    for i in range(warmup):
        res.step(idx(i), h)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for i in range(steps):
        res.step(idx(warmup + i), h)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def time_each(res, steps, rotate=True):
    """Per-step durations (ms) from one event pair per step: median and min."""
    import torch
    stream = torch.cuda.current_stream()
    h = stream.cuda_stream
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for i, (a, b) in enumerate(ev):
        a.record(stream)
        res.step(i if rotate else 0, h)
        b.record(stream)
    torch.cuda.synchronize()
    t = np.array([a.elapsed_time(b) for a, b in ev])
    return float(np.median(t)), float(t.min())


def measure(k, args, params):
    import workloads as w
    return measure_problem(w.config(k), args, params)


def measure_problem(p, args, params):
    bytes_alg = p.algorithmic_bytes()
    copies = args.copies or (max(2, -(-ROTATE_TOTAL_BYTES // bytes_alg)) if bytes_alg < 2 * LLC_BYTES else 2)
    copies = min(copies, 64)
    res = Resident(p, copies, params)
    ms, wall_ms = time_steps(res, args.steps, args.warmup, rotate=True)
    med, mn = time_each(res, min(args.steps, 50), rotate=True)
    ms_warm, _ = time_steps(res, args.steps, args.warmup, rotate=False)
    import paper_2603_07169_amd as s
    out = {
        "workload": p.name, "dtype": p.dtype, "m": p.m, "n": p.n, "nnz": p.nnz, "alpha": p.alpha, "beta": p.beta,
        "algorithmic_bytes": bytes_alg, "plan": s.PLAN_NAMES[res.info.plan], "kernel": res.kernel,
        "copies_rotated": copies, "ms_per_step": ms, "ms_median": med, "ms_min": mn, "ms_per_step_wall": wall_ms,
        "GBps": bytes_alg / ms / 1e6, "GFLOPs": p.flops() / ms / 1e6,
        "warm_ms_per_step": ms_warm, "warm_GBps": bytes_alg / ms_warm / 1e6, "analysis_ms": res.analysis_ms,
    }
    out["roofline"] = roofline_block(out)
    res.close()
    return p, out


def two_pass_sweep(args):
    """Matrices with scattered columns around the sizes where the two-pass plan starts to pay: the row-wise plan AUTO
    arrives at without it (merge for the power-law rows, adaptive for the uniform ones) against the two-pass plan."""
    import workloads as w
    import paper_2603_07169_amd as s
    out = []
    makers = [lambda: w.powerlaw(250_000), lambda: w.powerlaw(500_000), lambda: w.powerlaw(1_000_000), lambda: w.powerlaw(2_000_000),
              lambda: w.uniform_rows(1 << 18, 1 << 18, 16), lambda: w.uniform_rows(1 << 20, 1 << 20, 16),
              lambda: w.uniform_rows(1 << 21, 1 << 21, 16), lambda: w.uniform_rows(1 << 20, 1 << 20, 16, dtype="bf16"),
              lambda: w.uniform_rows(1 << 20, 1 << 18, 32), lambda: w.uniform_rows(1 << 16, 1 << 20, 64),
              lambda: w.powerlaw(8_000_000), lambda: w.uniform_rows(1 << 23, 1 << 23, 16)]
    for make in makers:
        p = make()
        row_wise = s.SPMV_PLAN_MERGE if int(np.diff(p.rowptr).max()) > 8192 else s.SPMV_PLAN_ADAPTIVE
        entry = {"workload": p.name, "dtype": p.dtype, "m": p.m, "n": p.n, "nnz": p.nnz}
        plans = [row_wise, s.SPMV_PLAN_TWOPHASE]
        if p.n > 2 * ((4 << 20) // (4 if p.dtype == "f32" else 2)):      # x beyond two 4 MiB stretches: the column-blocked plan as well
            plans.append(s.SPMV_PLAN_COLBLOCK)
        for plan in plans:
            _, r = measure_problem(p, args, dict(plan=plan))
            entry[r["plan"] + "_us"] = r["ms_per_step"] * 1e3
            entry[r["plan"] + "_analysis_ms"] = r["analysis_ms"]
        _, r = measure_problem(p, args, dict(plan=0))
        entry["auto_plan"] = r["plan"]
        out.append(entry)
    return out


def launch_floor_us(n=200):
    """Mean time of back-to-back launches of a one-wavefront kernel (the library's reduction
    self-check): what any kernel pays before it moves a byte."""
    import torch
    import paper_2603_07169_amd as s
    a = torch.zeros(64, dtype=torch.float32, device="cuda")
    b = torch.zeros(14 * 64, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    for _ in range(10):
        s.spmv_selftest_reduce(a.data_ptr(), b.data_ptr(), stream.cuda_stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(n):
        s.spmv_selftest_reduce(a.data_ptr(), b.data_ptr(), stream.cuda_stream)
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n * 1e3


def paper_sweep(args):
    """The workload the paper defines for this task (App. C task 12: rows 2^10..2^15, 2048 columns,
    density 0.01, random positions), FP32 and bf16: speed-up S_i of the planned path over the
    library's own one-lane-per-row kernel, and the paper's weighted score P (section 3.3, Eq. 2)
    with the task's complexity O(nnz) as weight: P = sum nnz_i S_i / sum nnz_i."""
    import workloads as w
    out = {"cases": []}
    for dtype in ("f32", "bf16"):
        num = den = 0.0
        for e in range(10, 16):
            p = w.density_random(1 << e, 2048, 0.01, dtype=dtype)
            _, planned = measure_problem(p, args, dict(plan=0))
            _, naive = measure_problem(p, args, dict(plan=1))
            S = naive["ms_per_step"] / planned["ms_per_step"]
            out["cases"].append({"rows": 1 << e, "dtype": dtype, "nnz": p.nnz, "plan": planned["plan"],
                                 "us": planned["ms_per_step"] * 1e3, "naive_us": naive["ms_per_step"] * 1e3, "S": S})
            num += p.nnz * S
            den += p.nnz
        out["P_" + dtype] = num / den
    return out


def spmm_sweep(args, cases=((10, "f32"), (12, "f32"), (14, "f32"), (16, "f32"), (18, "f32"), (16, "bf16"))):
    """The paper's SpMM CSR workload (App. C task 13: rows 2^10..2^18, cols 2048, K 4096, density 0.01): time of
    C <- A*B per size, GFLOP/s = 2*nnz*K / time, effective GB/s over the algorithmic bytes
    (A's three arrays + B once + C written once).  bf16: A's values and B stored as bf16, C as float."""
    import torch
    import paper_2603_07169_amd as s
    import workloads as w
    out = []
    K = 4096
    stream = torch.cuda.current_stream()
    for e, dtype in cases:
        p = w.density_random(1 << e, 2048, 0.01, dtype=dtype)
        esz = 4 if dtype == "f32" else 2
        rowptr, colidx, vals = dev(p.rowptr), dev(p.colidx), dev(p.vals)
        A = s.CsrMatrix(p.m, p.n, rowptr, colidx, vals, s.SPMV_F32 if dtype == "f32" else s.SPMV_BF16, dict(prepare_spmm=1))
        B = torch.rand(p.n, K, dtype=torch.float32, device="cuda")
        if dtype == "bf16":
            B = B.to(torch.bfloat16).view(torch.int16)
        C = torch.empty(p.m, K, dtype=torch.float32, device="cuda")
        steps = max(5, min(args.steps, int(2e9 // (p.m * K * 4)) or 5))
        for _ in range(2):
            A.spmm(B, C, 1.0, 0.0, stream.cuda_stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            A.spmm(B, C, 1.0, 0.0, stream.cuda_stream)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        bytes_alg = (4 + esz) * p.nnz + 4 * (p.m + 1) + esz * p.n * K + 4 * p.m * K
        out.append({"rows": p.m, "cols": p.n, "K": K, "nnz": p.nnz, "storage": dtype, "steps": steps, "ms": ms,
                    "GFLOPs": 2.0 * p.nnz * K / ms / 1e6, "algorithmic_bytes": bytes_alg,
                    "GBps": bytes_alg / ms / 1e6, "hbm_frac": bytes_alg / ms / 1e6 / HBM_PEAK_GBPS,
                    # bound by vector FMA issue: 256 CUs x 64 lanes x 2 flops x 2.4 GHz = 78.6 TFLOP/s without
                    # packed FP32 instructions (which this build keeps out), half of the published 157.3
                    "alu_frac": 2.0 * p.nnz * K / ms / 1e6 / 78600.0})
        if e <= 12 and not args_no_cpu(args):
            # the oracle beside it (one host thread), on the sizes it finishes in seconds
            import oracle
            Bh = B.cpu().numpy()
            Bh = Bh.view(np.uint16) if dtype == "bf16" else Bh
            t0 = time.perf_counter()
            oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, Bh)
            dt = time.perf_counter() - t0
            out[-1]["cpu_oracle"] = {"ms": dt * 1e3, "GFLOPs": 2.0 * p.nnz * K / dt / 1e9, "cores": 1, "kind": "oracle",
                                     "sample": "whole product, single thread, one run"}
        A.close()
        del B, C
    return out


def args_no_cpu(args):
    return bool(getattr(args, "no_cpu_baseline", False))


def formats_sweep(args):
    """SpMV in the benchmark's other layouts (App. C tasks 8, 10, 14): the largest paper shape of each
    task and config 3's stencil as a size where the kernels stream.  GB/s over each layout's own bytes."""
    import torch
    import paper_2603_07169_amd as s
    import workloads as w
    stream = torch.cuda.current_stream()
    out = []

    def timed(call, steps):
        for _ in range(3):
            call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            call()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    cases = [("coo", w.density_random(1 << 15, 2048, 0.01)), ("csc", w.density_random(2048, 1 << 15, 0.01)),
             ("ell", w.density_random(2048, 1 << 15, 0.01)), ("coo", w.config(3)), ("ell", w.config(3))]
    for layout, p in cases:
        e = 4 if p.dtype == "f32" else 2
        code = s.SPMV_F32 if p.dtype == "f32" else s.SPMV_BF16
        x = dev(p.x)
        y = torch.zeros(p.m, dtype=torch.float32, device="cuda")
        h = stream.cuda_stream
        if layout == "coo":
            row, col, vals = [dev(a) for a in w.to_coo(p)]
            nbytes = p.nnz * (e + 8) + e * p.n + 4 * p.m
            call = lambda: s.check(s.spmv_coo_run(p.m, p.n, p.nnz, row.data_ptr(), col.data_ptr(), vals.data_ptr(), code,
                                                  x.data_ptr(), y.data_ptr(), 1.0, 0.0, h))
        elif layout == "csc":
            co, row, vals = [dev(a) for a in w.to_csc(p)]
            nbytes = p.nnz * (e + 4) + 4 * (p.n + 1) + e * p.n + 4 * p.m
            call = lambda: s.check(s.spmv_csc_run(p.m, p.n, p.nnz, co.data_ptr(), row.data_ptr(), vals.data_ptr(), code,
                                                  x.data_ptr(), y.data_ptr(), 1.0, 0.0, h))
        else:
            width, ci, vals = w.to_ell(p)
            ci, vals = dev(ci), dev(vals)
            nbytes = p.m * width * (e + 4) + e * p.n + 4 * p.m
            call = lambda: s.check(s.spmv_ell_run(p.m, p.n, width, ci.data_ptr(), vals.data_ptr(), code, x.data_ptr(),
                                                  y.data_ptr(), 1.0, 0.0, h))
        ms = timed(call, min(args.steps, 50))
        out.append({"layout": layout, "workload": p.name, "dtype": p.dtype, "m": p.m, "n": p.n, "nnz": p.nnz,
                    "ms": ms, "algorithmic_bytes": nbytes, "GBps": nbytes / ms / 1e6,
                    "hbm_frac": nbytes / ms / 1e6 / HBM_PEAK_GBPS, "GFLOPs": 2.0 * p.nnz / ms / 1e6})
    return out


def graph_replay(args, configs=(1, 2)):
    """The same steps recorded once into a HIP graph and replayed (stream capture of spmv_csr_run):
    what the launch-bound configs cost when the host's launch path is taken out."""
    import torch
    import workloads as w
    out = []
    params = dict(plan=0)
    for k in configs:
        p = w.config(k)
        bytes_alg = p.algorithmic_bytes()
        copies = min(64, max(2, -(-ROTATE_TOTAL_BYTES // bytes_alg)))
        res = Resident(p, copies, params)
        side = torch.cuda.Stream()
        for i in range(copies):                       # eager pass first: nothing but launches may happen under capture
            res.step(i, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            h = torch.cuda.current_stream().cuda_stream
            for i in range(args.steps):
                res.step(i, h)
        for _ in range(2):
            g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        out.append({"workload": p.name, "steps_in_graph": args.steps, "copies_rotated": copies, "ms_per_step": ms,
                    "GBps": bytes_alg / ms / 1e6, "frac_effective": bytes_alg / ms / 1e6 / HBM_PEAK_GBPS})
        res.close()
    return out


def cpu_baseline(p, runs=3):
    """The oracle as it stands, one thread, on the whole workload: 1 warm-up + best of `runs`."""
    import oracle
    best = float("inf")
    for i in range(runs + 1):
        t0 = time.perf_counter()
        oracle.spmv_problem(p)
        dt = time.perf_counter() - t0
        if i > 0:
            best = min(best, dt)
    return {"value": p.algorithmic_bytes() / best / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"whole workload {p.name} ({p.nnz} nnz), single thread, best of {runs} after 1 warm-up",
            "ms": best * 1e3, "GFLOPs": p.flops() / best / 1e9, "host_cores_available": os.cpu_count()}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: the product has no multi-GPU path (run with --gpus 1).", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.formats:
        print(json.dumps({"formats": formats_sweep(args)}))
        return
    if args.two_pass_sweep:
        print(json.dumps({"two_pass_sweep": two_pass_sweep(args)}))
        return
    if args.spmm:
        print(json.dumps({"spmm_csr": spmm_sweep(args, cases=((args.spmm, "f32"), (args.spmm, "bf16")))}))
        return
    params = dict(plan=args.plan, block_nnz=args.block_nnz, rows_max=args.rows_max,
                  items_per_chunk=args.items_per_chunk, vector_lanes=args.vector_lanes, skip_validation=0)
    # every configuration in turn, each with the oracle timed on this host beside it; the headline is one of them
    per = {}
    for k in ([args.config] if args.only else range(1, 6)):
        p, r = measure(k, args, params)
        if not args.no_cpu_baseline:
            r["cpu_baseline"] = cpu_baseline(p)
        per[k] = r
        if k == args.config:
            head, shape = r, (p.m, p.n, p.nnz, p.alpha, p.beta, p.dtype)
        del p
    m, n, nnz, alpha, beta, storage = shape
    roof = dict(head["roofline"])
    roof["frac"] = roof["frac_effective"]   # algorithmic bytes / time / peak, as the metric defines it (see frac_real beside it)
    roof["algorithmic_bytes_per_launch"] = head["algorithmic_bytes"]
    roof["avg_launch_ms"] = head["ms_per_step"]
    line = {
        "metric": "CSR SpMV effective HBM bandwidth (algorithmic bytes / time)",
        "value": head["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": storage, "data": "synthetic",
        "config": {"workload": head["workload"], "m": m, "n": n, "nnz": nnz, "alpha": alpha, "beta": beta,
                   "storage": storage, "plan": head["plan"], "cache_state": f"cold: rotating over {head['copies_rotated']} disjoint copies",
                   "why_this_one": "the second of the five configurations (the 2-D Laplacian), the one the 70 % target names that is large "
                                   "enough to stream; all five are measured in per_config, each with its own roofline block"},
        "gflops": head["GFLOPs"], "warm_GBps": head["warm_GBps"],
        "roofline": roof,
    }
    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = head["cpu_baseline"]
    if not args.only:
        line["per_config"] = sorted(per.values(), key=lambda r: r["workload"])
    if not args.only and not args.no_extras:
        import workloads as w
        line["launch_floor_us"] = launch_floor_us()
        # not a config: config 1's generator at a size where the kernel streams instead of waiting for its launch
        big = w.uniform_rows(1 << 22, 1 << 22, 16)
        big.name = "supplementary_uniform16_4M_f32"
        _, r = measure_problem(big, args, params)
        del big
        line["supplementary"] = r
        # not a config either: config 4's generator with the power law read literally (type-I Pareto, mean row length 2.6)
        lit = w.powerlaw(4_000_000, literal=True)
        lit.name = "supplementary_powerlaw_literal_4M_f32"
        _, r = measure_problem(lit, args, params)
        del lit
        line["supplementary_literal"] = r
        line["paper_sweep"] = paper_sweep(args)
        line["spmm_csr"] = spmm_sweep(args)
        line["formats"] = formats_sweep(args)
        line["graph_replay"] = graph_replay(args)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
