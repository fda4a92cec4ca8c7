"""The counter-based bottleneck filter (paper section 3.2, Table 2) is host logic: classification rule,
figure derivation and CSV reading are checked here without a GPU."""
import csv

import pytest

from paper_2603_07169_amd import bottleneck as b


@pytest.mark.parametrize("compute,dram,mem,want", [
    (0.31, 0.9, 0.9, b.COMPUTE),            # compute utilisation decides first
    (0.30, 0.9, 0.1, b.BANDWIDTH),          # exactly 30 % is not above the threshold
    (0.10, 0.31, 0.05, b.BANDWIDTH),
    (0.10, 0.05, 0.31, b.BANDWIDTH),        # "or": either memory figure suffices
    (0.10, 0.30, 0.30, b.LATENCY),
    (0.0, 0.0, 0.0, b.LATENCY),
    (None, None, 0.5, b.BANDWIDTH),         # figures that were not measured count as low
    (None, None, None, b.LATENCY),
])
def test_table_2_rule(compute, dram, mem, want):
    assert b.classify(compute, dram, mem) == want


def test_every_class_keeps_four_metrics():
    assert all(len(v) == 4 for v in b.FILTERED.values()) and set(b.FILTERED) == {b.COMPUTE, b.LATENCY, b.BANDWIDTH}


def test_derivation_from_counters():
    cus, cycles = 256, 1000.0
    c = {"GRBM_GUI_ACTIVE": 8 * cycles,
         "SQ_ACTIVE_INST_VALU": 0.5 * cycles * cus * 4 / 4,     # VALU issuing half of all SIMD cycles
         "FETCH_SIZE": 1000.0, "WRITE_SIZE": 500.0,              # KiB: 2*1000 + 500 = 2500 KiB
         "TA_TA_BUSY_sum": 0.25 * cycles * cus, "SQ_LDS_IDX_ACTIVE": 0.6 * cycles * cus,
         "TCC_HIT_sum": 30.0, "TCC_MISS_sum": 10.0}
    d = b.derive(c, duration_ns=1000.0, cus=cus, peak_gbps=8000.0)
    assert d["compute_throughput"] == pytest.approx(0.5)
    assert d["dram_gbps"] == pytest.approx(2500 * 1024 / 1000.0) and d["dram_throughput"] == pytest.approx(2560.0 / 8000)
    assert d["mem_pipes_busy"] == pytest.approx(0.25) and d["lds_busy"] == pytest.approx(0.6)
    assert d["memory_throughput"] == pytest.approx(0.6)          # the busiest stage
    assert d["l2_hit_rate"] == pytest.approx(0.75)
    r = b.filter_report("k", c, 1000.0, cus=cus)
    assert r["class"] == b.COMPUTE and tuple(r["metrics"]) == b.FILTERED[b.COMPUTE]
    c["SQ_ACTIVE_INST_VALU"] *= 0.2
    r = b.filter_report("k", c, 1000.0, cus=cus)
    assert r["class"] == b.BANDWIDTH and r["metrics"]["max_bandwidth_gbps"] == 8000.0
    missing = b.derive({"GRBM_GUI_ACTIVE": 8000.0}, 1000.0)
    assert missing["compute_throughput"] is None and missing["dram_throughput"] is None and missing["memory_throughput"] is None


def test_reads_rocprofv3_counter_csv(tmp_path):
    d = tmp_path / "pass1"
    d.mkdir()
    cols = ["Correlation_Id", "Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value", "Start_Timestamp", "End_Timestamp"]
    rows = [[1, 1, "spmv_x(int)", "GRBM_GUI_ACTIVE", 800.0, 100, 200], [2, 2, "spmv_x(int)", "GRBM_GUI_ACTIVE", 1200.0, 300, 500],
            [3, 3, "other(int)", "GRBM_GUI_ACTIVE", 5.0, 600, 601]]
    with open(d / "r_counter_collection.csv", "w", newline="") as fh:
        wr = csv.writer(fh, quoting=csv.QUOTE_NONNUMERIC)
        wr.writerow(cols)
        wr.writerows(rows)
    got = b.read_counter_dirs([str(d)], match="spmv_")
    assert list(got) == ["spmv_x(int)"]
    counters, dur = got["spmv_x(int)"]
    assert counters == {"GRBM_GUI_ACTIVE": 1000.0} and dur == 150.0
    assert "spmv_x" in b.to_markdown([b.filter_report(k, c, t) for k, (c, t) in got.items()])
