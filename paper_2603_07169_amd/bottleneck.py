"""Bottleneck filter for rocprofv3 counter output (host-side tool, no GPU needed).

The paper's hardware analysis filter (section 3.2, Table 2; App. A "Bottleneck Classification Logic")
sorts a kernel into one of three classes from three utilisation figures, with one threshold of 30 %
for all of them, and then keeps only the four metrics that matter for that class:

    compute bound            Compute.Th > 30 %
    memory latency bound     Compute.Th < 30 %, DRAM.Th < 30 % and Memory.Th < 30 %
    memory bandwidth bound   Compute.Th < 30 %, DRAM.Th > 30 % or Memory.Th > 30 %

The paper reads its figures from Nsight Compute.  Here they are rebuilt from gfx950 counters that
rocprofv3 --pmc collects (several passes, one CSV directory each), per kernel, averaged over its
dispatches:

    cycles        GRBM_GUI_ACTIVE / 8            (the counter sums the 8 dies)
    Compute.Th    4 * SQ_ACTIVE_INST_VALU / (cycles * CUs * 4 SIMDs)     vector ALU issue, quad-cycle counter
    DRAM.Th       (2 * FETCH_SIZE + WRITE_SIZE) KiB / duration / peak    the factor 2 is the copy-kernel
                                                                          calibration of FETCH_SIZE on this chip
    Memory.Th     max(DRAM.Th, TA_TA_BUSY_sum / (cycles * CUs), SQ_LDS_IDX_ACTIVE / (cycles * CUs))
                                                                          the busiest stage of the memory path

A figure whose counters were not collected is None and takes no part in the rule (a missing figure
counts as "below threshold").  Usage:

    python -m paper_2603_07169_amd.bottleneck DIR [DIR ...] [--match spmv_] [--cus 256] [--peak-gbps 8000]
"""
from __future__ import annotations

import argparse
import csv
import glob
import os
from collections import defaultdict

THRESHOLD = 0.30
COMPUTE, LATENCY, BANDWIDTH = "compute bound", "memory latency bound", "memory bandwidth bound"

FILTERED = {
    COMPUTE: ("compute_throughput", "issue_slots_busy", "ipc_active", "cu_busy"),
    LATENCY: ("l2_hit_rate", "l1_hit_rate", "ipc_elapsed", "mem_busy"),
    BANDWIDTH: ("dram_throughput", "memory_throughput", "max_bandwidth_gbps", "mem_pipes_busy"),
}


def classify(compute_th, dram_th, memory_th, threshold=THRESHOLD):
    """Table 2's rule.  None (not measured) counts as below the threshold."""
    above = lambda v: v is not None and v > threshold
    if above(compute_th):
        return COMPUTE
    if above(dram_th) or above(memory_th):
        return BANDWIDTH
    return LATENCY


def derive(c, duration_ns, cus=256, peak_gbps=8000.0, fetch_scale=2.0):
    """All figures the three classes use, from a dict of counter means `c` (missing counters -> None)."""
    g = c.get
    cycles = g("GRBM_GUI_ACTIVE") / 8.0 if g("GRBM_GUI_ACTIVE") else None
    ratio = lambda num, den: (num / den) if (num is not None and den) else None
    out = {"duration_us": duration_ns / 1e3 if duration_ns else None, "max_bandwidth_gbps": peak_gbps}
    out["compute_throughput"] = ratio(4.0 * g("SQ_ACTIVE_INST_VALU") if g("SQ_ACTIVE_INST_VALU") is not None else None,
                                      cycles * cus * 4 if cycles else None)
    # wave-cycles spent issuing to any pipe per SIMD cycle (quad-cycle counter); the pipes of a SIMD work
    # side by side, so this can pass 100 %
    out["issue_slots_busy"] = ratio(4.0 * g("SQ_ACTIVE_INST_ANY") if g("SQ_ACTIVE_INST_ANY") is not None else None,
                                    cycles * cus * 4 if cycles else None)
    insts = sum(v for k, v in c.items() if k in ("SQ_INSTS_VALU", "SQ_INSTS_SALU", "SQ_INSTS_LDS", "SQ_INSTS_VMEM_RD")) or None
    out["ipc_elapsed"] = ratio(insts, cycles * cus if cycles else None)
    out["ipc_active"] = ratio(insts, g("SQ_BUSY_CYCLES") * cus / 32.0 if g("SQ_BUSY_CYCLES") else None)
    out["cu_busy"] = ratio(g("SQ_BUSY_CYCLES"), cycles * 32 if cycles else None)   # counted per shader engine (32 of them)
    if g("FETCH_SIZE") is not None or g("WRITE_SIZE") is not None:
        nbytes = 1024.0 * (fetch_scale * (g("FETCH_SIZE") or 0.0) + (g("WRITE_SIZE") or 0.0))
        out["dram_gbps"] = ratio(nbytes, duration_ns) if duration_ns else None
        out["dram_throughput"] = ratio(out["dram_gbps"], peak_gbps)
    else:
        out["dram_gbps"] = out["dram_throughput"] = None
    out["mem_pipes_busy"] = out["mem_busy"] = ratio(g("TA_TA_BUSY_sum"), cycles * cus if cycles else None)
    out["lds_busy"] = ratio(g("SQ_LDS_IDX_ACTIVE"), cycles * cus if cycles else None)
    stages = [v for v in (out["dram_throughput"], out["mem_pipes_busy"], out["lds_busy"]) if v is not None]
    out["memory_throughput"] = max(stages) if stages else None
    hit, miss = g("TCC_HIT_sum"), g("TCC_MISS_sum")
    out["l2_hit_rate"] = ratio(hit, hit + miss) if hit is not None and miss is not None else None
    out["l1_hit_rate"] = None
    if g("TCP_TCC_READ_REQ_sum") is not None and g("SQ_INSTS_VMEM_RD"):
        # requests that left L1 per wavefront load instruction; not a rate below 1, reported as is
        out["l1_requests_per_load"] = g("TCP_TCC_READ_REQ_sum") / g("SQ_INSTS_VMEM_RD")
    return out


def filter_report(name, counters, duration_ns, **kw):
    """{'kernel', 'class', 'basis': the three deciding figures, 'metrics': the class's four}."""
    d = derive(counters, duration_ns, **kw)
    cls = classify(d["compute_throughput"], d["dram_throughput"], d["memory_throughput"])
    return {"kernel": name, "class": cls, "duration_us": d["duration_us"],
            "basis": {k: d[k] for k in ("compute_throughput", "dram_throughput", "memory_throughput")},
            "metrics": {k: d.get(k) for k in FILTERED[cls]}}


def read_counter_dirs(dirs, match=""):
    """{kernel name: ({counter: mean over dispatches}, mean dispatch duration in ns)} from rocprofv3 CSV output."""
    values = defaultdict(lambda: defaultdict(list))
    durations = defaultdict(list)
    for d in dirs:
        for f in glob.glob(os.path.join(d, "*counter_collection.csv")):
            with open(f, newline="") as fh:
                for row in csv.DictReader(fh):
                    name = row["Kernel_Name"]
                    if match and match not in name:
                        continue
                    values[name][row["Counter_Name"]].append(float(row["Counter_Value"]))
                    durations[name].append(int(row["End_Timestamp"]) - int(row["Start_Timestamp"]))
    return {k: ({c: sum(v) / len(v) for c, v in cs.items()}, sum(durations[k]) / len(durations[k])) for k, cs in values.items()}


def short_name(name):
    return name.replace("spmv::(anonymous namespace)::", "").replace("void ", "").split("(")[0]


def to_markdown(reports):
    def fmt(v, key=""):
        if v is None:
            return "n/a"
        if key.startswith("ipc") or key == "max_bandwidth_gbps":
            return f"{v:.2f}" if v < 100 else f"{v:.0f}"
        return f"{100 * v:.1f} %"

    lines = ["| kernel | us | Compute.Th | DRAM.Th | Memory.Th | class | filtered metrics |", "|---|---|---|---|---|---|---|"]
    for r in reports:
        b = r["basis"]
        kept = ", ".join(f"{k} {fmt(v, k)}" for k, v in r["metrics"].items())
        lines.append(f"| {short_name(r['kernel'])} | {r['duration_us']:.1f} | {fmt(b['compute_throughput'])} | "
                     f"{fmt(b['dram_throughput'])} | {fmt(b['memory_throughput'])} | {r['class']} | {kept} |")
    return "\n".join(lines)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("dirs", nargs="+", help="rocprofv3 output directories holding *counter_collection.csv")
    ap.add_argument("--match", default="", help="only kernels whose name contains this")
    ap.add_argument("--cus", type=int, default=256)
    ap.add_argument("--peak-gbps", type=float, default=8000.0)
    a = ap.parse_args(argv)
    data = read_counter_dirs(a.dirs, a.match)
    reports = [filter_report(k, c, dur, cus=a.cus, peak_gbps=a.peak_gbps) for k, (c, dur) in sorted(data.items())]
    print(to_markdown(reports))
    return reports


if __name__ == "__main__":
    main()
