"""CPU-side checks of the C-ABI library: it loads, exports what the header declares, rejects bad
arguments before touching the device, and its host analysis equals the oracle bit for bit."""
import ctypes as C
import re
from pathlib import Path

import numpy as np
import pytest

import oracle
import paper_2603_07169_amd as s
import workloads as w

ROOT = Path(__file__).resolve().parents[1]
DEFAULT_ITEMS_PER_CHUNK = 2048   # as documented in the header


def rowptr_of(lens):
    return np.concatenate(([0], np.cumsum(np.asarray(lens, dtype=np.int64)))).astype(np.int32)


def test_library_exports_every_declared_symbol():
    header = (ROOT / "include" / "spmv_mi355.h").read_text()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(sp(?:mv|mm)_[a-z0-9_]+)\s*\(", header))
    assert {"spmv_csr_create", "spmv_csr_analyze", "spmv_csr_run", "spmm_csr_run", "spmv_destroy"} <= declared
    lib = C.CDLL(str(s.library_path()))
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(s.spmv.EXPORTS)           # the binding mirrors the header, name for name


def test_status_strings():
    assert s.spmv_status_string(0) == "ok"
    assert len({s.spmv_status_string(k) for k in range(8)}) == 8 and s.spmv_status_string(8) == "unknown status"


def test_create_argument_errors():
    A = 4096  # any aligned fake address: create never dereferences
    ok = lambda *a: s.spmv_csr_create(*a)[0]
    assert ok(4, 4, 8, A, A, A, s.SPMV_F32) == s.SPMV_OK
    assert ok(-1, 4, 8, A, A, A, 0) == s.SPMV_ERR_INVALID_ARG
    assert ok(4, -1, 8, A, A, A, 0) == s.SPMV_ERR_INVALID_ARG
    assert ok(4, 4, -8, A, A, A, 0) == s.SPMV_ERR_INVALID_ARG
    assert ok(4, 4, 8, None, A, A, 0) == s.SPMV_ERR_INVALID_ARG
    assert ok(4, 4, 8, A, None, A, 0) == s.SPMV_ERR_INVALID_ARG
    assert ok(4, 4, 8, A, A, None, 0) == s.SPMV_ERR_INVALID_ARG
    assert ok(4, 4, 0, A, None, None, 0) == s.SPMV_OK            # no entries: colidx/vals may be NULL
    assert ok(4, 0, 3, A, A, A, 0) == s.SPMV_ERR_INVALID_ARG     # entries but no columns
    assert ok(4, 4, 8, A, A, A, 7) == s.SPMV_ERR_INVALID_ARG     # unknown dtype
    assert ok(2 ** 31, 4, 8, A, A, A, 0) == s.SPMV_ERR_UNSUPPORTED
    assert ok(4, 4, 2 ** 31, A, A, A, 0) == s.SPMV_ERR_UNSUPPORTED
    big = s.SPMV_MAX_SIZE
    for sizes in ((big, 4, 8), (4, big, 8), (4, 4, big)):
        assert ok(*sizes, A, A, A, 0) == s.SPMV_OK
        assert ok(*(v + (v == big) for v in sizes), A, A, A, 0) == s.SPMV_ERR_UNSUPPORTED
    assert ok(4, 4, 8, A + 2, A, A, 0) == s.SPMV_ERR_UNSUPPORTED  # rowptr not int32-aligned
    assert ok(4, 4, 8, A, A, A + 2, s.SPMV_F32) == s.SPMV_ERR_UNSUPPORTED
    assert ok(4, 4, 8, A, A, A + 2, s.SPMV_BF16) == s.SPMV_OK
    st, h = s.spmv_csr_create(4, 4, 8, A, A, A, 0)
    assert s.spmv_csr_run(h, A, A, 1.0, 0.0) == s.SPMV_ERR_NOT_ANALYZED
    assert s.spmv_csr_refresh_values(h) == s.SPMV_ERR_NOT_ANALYZED
    assert s.spmv_csr_refresh_values(None) == s.SPMV_ERR_INVALID_ARG
    assert s.spmv_csr_get_analysis_info(h)[0] == s.SPMV_ERR_NOT_ANALYZED
    assert s.spmv_csr_main_kernel_name(h) == ""
    assert s.spmv_destroy(h) == s.SPMV_OK
    assert s.spmv_destroy(None) == s.SPMV_OK
    assert s.spmv_csr_analyze(None) == s.SPMV_ERR_INVALID_ARG


def test_size_limit_matches_the_header_and_binds_every_entry_point():
    header = (ROOT / "include" / "spmv_mi355.h").read_text()
    mm = re.search(r"#define SPMV_MAX_SIZE \(\(int64_t\)(\d+) - (\d+)\)", header)
    assert int(mm.group(1)) - int(mm.group(2)) == s.SPMV_MAX_SIZE == 2 ** 31 - 2 ** 22
    big, A = s.SPMV_MAX_SIZE, 4096
    # one row holding the largest entry count: the host analysis takes it, one more is refused
    st, info, _ = s.spmv_analyze_host(1, 8, big, np.array([0, big], np.int32), dict(plan=5))
    assert st == s.SPMV_OK and (info.nnz, info.max_len) == (big, big)
    assert info.num_chunks == -(-(big + 1) // DEFAULT_ITEMS_PER_CHUNK)
    assert s.spmv_analyze_host(1, 8, big + 1, np.array([0, 0], np.int32))[0] == s.SPMV_ERR_UNSUPPORTED
    # the stateless layouts check sizes before anything touches the device
    assert s.spmv_coo_run(4, 4, big + 1, A, A, A, 0, A, A, 1.0, 0.0) == s.SPMV_ERR_UNSUPPORTED
    assert s.spmv_coo_run(big + 1, 4, 8, A, A, A, 0, A, A, 1.0, 0.0) == s.SPMV_ERR_UNSUPPORTED
    assert s.spmv_csc_run(4, big + 1, 8, A, A, A, 0, A, A, 1.0, 0.0) == s.SPMV_ERR_UNSUPPORTED
    assert s.spmv_ell_run(4, 4, big + 1, A, A, 0, A, A, 1.0, 0.0) == s.SPMV_ERR_UNSUPPORTED
    assert s.spmv_ell_run(4, 4, -1, A, A, 0, A, A, 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    # the entry point with the fixed scratch array: its own, smaller limit on rows + entries, checked on the host first
    mm = re.search(r"#define SPMV_STATIC_MAX_ITEMS \(\(\(int64_t\)1 << (\d+)\) - (\d+)\)", header)
    lim = (1 << int(mm.group(1))) - int(mm.group(2))
    assert lim == s.SPMV_STATIC_MAX_ITEMS and lim % DEFAULT_ITEMS_PER_CHUNK == 0
    assert 16 * (lim // DEFAULT_ITEMS_PER_CHUNK) + 8 <= 2 << 20          # splits + carries of every chunk fit the 2 MiB array
    assert s.spmv_csr_run_static(lim // 2, 4, lim - lim // 2 + 1, A, A, A, 0, A, A, 1.0, 0.0) == s.SPMV_ERR_UNSUPPORTED
    assert s.spmv_csr_run_static(-1, 4, 8, A, A, A, 0, A, A, 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    assert s.spmv_csr_run_static(4, 4, 8, A, A, A, 2, A, A, 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    assert s.spmv_csr_run_static(0, 4, 0, None, None, None, 0, None, None, 1.0, 0.0) == s.SPMV_OK
    assert s.spmv_csr_run_static(4, 4, 8, A, A + 2, A, 0, A, A, 1.0, 0.0) == s.SPMV_ERR_UNSUPPORTED    # misaligned colidx


def test_analyze_parameter_ranges():
    rp = rowptr_of([1, 2, 3])
    def st(**kw):
        return s.spmv_analyze_host(3, 4, 6, rp, kw)[0]
    assert st() == s.SPMV_OK
    assert st(block_nnz=8192, rows_max=1024, items_per_chunk=8192, vector_lanes=64, plan=5) == s.SPMV_OK
    for bad in (dict(block_nnz=8193), dict(block_nnz=-1), dict(rows_max=1025), dict(rows_max=-3),
                dict(items_per_chunk=8193), dict(items_per_chunk=-1), dict(vector_lanes=3), dict(vector_lanes=1),
                dict(vector_lanes=128), dict(plan=6), dict(plan=7), dict(plan=8), dict(plan=9), dict(plan=10), dict(plan=-1)):  # 6 .. 9 need colidx: device only
        assert st(**bad) == s.SPMV_ERR_INVALID_ARG, bad


def test_spmm_row_order_matches_the_oracle():
    for lens in SHAPES + [list(np.random.default_rng(3).poisson(20.5, 13000)), [300, 252, 253, 0, 4, 5] * 7]:
        rp = rowptr_of(lens)
        m, nnz = rp.size - 1, int(rp[-1])
        st, info, got = s.spmv_analyze_host(m, 7, nnz, rp, dict(prepare_spmm=1))
        assert st == s.SPMV_OK
        rows = oracle.spmm_row_order(rp)
        assert np.array_equal(got["spmm_rows"], rows)
        desc, blocks = oracle.spmm_packed_layout(rp, rows)
        packed = oracle.spmm_packed_choice(nnz, blocks)
        assert info.spmm_prepared == (2 if packed else 1)
        assert (info.spmm_num_blocks, info.spmm_col_bytes) == ((blocks, 2) if packed else (0, 0))
        if packed:
            assert np.array_equal(got["spmm_desc"], desc)
        st, info, got = s.spmv_analyze_host(m, 7, nnz, rp)
        assert st == s.SPMV_OK and info.spmm_prepared == 0 and "spmm_rows" not in got
    rp = rowptr_of([20] * 100)                       # 32 slots a row for 20 entries: packed; column width by n
    assert [s.spmv_analyze_host(100, n, 2000, rp, dict(prepare_spmm=1))[1].spmm_col_bytes for n in (32768, 32769)] == [2, 4]
    assert s.spmv_analyze_host(400, 7, 2000, rowptr_of([5] * 400), dict(prepare_spmm=1))[1].spmm_prepared == 1
    rp = rowptr_of([1, 2, 3])
    assert s.spmv_analyze_host(3, 4, 6, rp, dict(prepare_spmm=2))[0] == s.SPMV_ERR_INVALID_ARG
    assert s.spmv_analyze_host(3, 4, 6, rp, dict(prepare_spmm=-1))[0] == s.SPMV_ERR_INVALID_ARG
    assert s.spmv_analyze_host(3, 4, 6, rp, dict(reserved=1))[0] == s.SPMV_ERR_INVALID_ARG


def test_large_row_counts_take_the_threaded_passes_and_still_match_the_oracle():
    """From 2^18 rows on the host analysis splits its passes over threads; results must not depend on that."""
    rng = np.random.default_rng(77)
    for m, params in ((300_000, {}), (1_100_000, dict(block_nnz=100, rows_max=7, items_per_chunk=64))):
        lens = np.where(rng.random(m) < 0.3, 0, rng.integers(0, 60, m))
        lens[rng.integers(0, m, 5)] = 9000
        compare_with_oracle(rowptr_of(lens), 10_000, params)
    bad = rowptr_of(np.full(400_000, 3))
    bad[350_000] -= 10                              # a decreasing offset deep inside a later thread's rows
    assert s.spmv_analyze_host(400_000, 10, int(bad[-1]), bad)[0] == s.SPMV_ERR_BAD_STRUCTURE


def test_analyze_rejects_malformed_rowptr():
    assert s.spmv_analyze_host(3, 4, 6, np.array([1, 2, 3, 6], np.int32))[0] == s.SPMV_ERR_BAD_STRUCTURE
    assert s.spmv_analyze_host(3, 4, 6, np.array([0, 4, 3, 6], np.int32))[0] == s.SPMV_ERR_BAD_STRUCTURE
    assert s.spmv_analyze_host(3, 4, 6, np.array([0, 2, 3, 5], np.int32))[0] == s.SPMV_ERR_BAD_STRUCTURE


def compare_with_oracle(rowptr, n, params):
    m, nnz = rowptr.size - 1, int(rowptr[-1])
    st, info, got = s.spmv_analyze_host(m, n, nnz, rowptr, params)
    assert st == s.SPMV_OK
    auto_bn, auto_rm = oracle.tile_shape(m, nnz)
    bn = params.get("block_nnz") or auto_bn
    rm = params.get("rows_max") or auto_rm
    ipc = params.get("items_per_chunk") or DEFAULT_ITEMS_PER_CHUNK
    stats = oracle.row_stats(rowptr)
    assert (info.m, info.n, info.nnz) == (m, n, nnz)
    assert (info.min_len, info.max_len, info.n_empty) == (stats["min_len"], stats["max_len"], stats["n_empty"])
    cnt, off, rows = oracle.row_bins(rowptr)
    assert np.array_equal(got["bin_count"], cnt) and np.array_equal(got["bin_offset"], off)
    assert np.array_equal(got["bin_rows"], rows)
    rb = oracle.row_blocks(rowptr, bn, rm)
    assert info.num_row_blocks == rb.size - 1 and np.array_equal(got["row_blocks"], rb)
    mr, mz = oracle.merge_path(rowptr, ipc)
    assert info.num_chunks == mr.size - 1
    assert np.array_equal(got["mp_row"], mr) and np.array_equal(got["mp_nz"], mz)
    want_plan = params.get("plan") or oracle.plan(m, nnz, stats["max_len"], bn)
    assert info.plan == want_plan
    assert info.vector_lanes == (params.get("vector_lanes") or oracle.vector_lanes(m, nnz))
    assert (info.block_nnz, info.rows_max, info.items_per_chunk) == (bn, rm, ipc)
    return info


SHAPES = [
    [], [0], [0, 0, 0], [5], [1, 0, 2, 0, 0, 7, 3], list(range(70)), [2049, 1, 2048, 0, 2047, 9000, 0, 0],
    [2] * 3000, np.random.default_rng(5).integers(0, 40, 5000), np.random.default_rng(6).integers(0, 3000, 700),
]
PARAMS = [
    {}, dict(block_nnz=1, rows_max=1, items_per_chunk=1), dict(block_nnz=6, rows_max=3, items_per_chunk=7),
    dict(block_nnz=8192, rows_max=1024, items_per_chunk=8192), dict(block_nnz=100, rows_max=1000, items_per_chunk=64),
    dict(plan=3, vector_lanes=16),
]


@pytest.mark.parametrize("lens", SHAPES)
@pytest.mark.parametrize("params", PARAMS)
def test_host_analysis_equals_oracle(lens, params):
    compare_with_oracle(rowptr_of(lens), 10000, params)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_host_analysis_equals_oracle_on_full_configs(k):
    """Only the row structure is needed, so the full-size configs are cheap here."""
    p = w.config(k, 1.0 if k in (1, 2) else 0.25)
    info = compare_with_oracle(p.rowptr, p.n, {})
    if k == 1:
        assert (info.block_nnz, info.rows_max) == (1024, 64)               # small matrix
        assert info.num_row_blocks == 64 and info.plan == s.SPMV_PLAN_ADAPTIVE
    if k == 2:
        assert (info.block_nnz, info.rows_max) == (2048, 256)              # mean 5 -> one lane per row
        assert info.num_row_blocks == 4096 and info.plan == s.SPMV_PLAN_ADAPTIVE
    if k == 4:
        assert info.plan == s.SPMV_PLAN_MERGE


def test_struct_layouts_of_the_binding_match_the_header(tmp_path):
    """The header compiled as plain C (it must be one) reports size and field offsets of every struct that crosses
    the boundary; the ctypes mirrors must agree field by field."""
    import subprocess
    structs = {"spmv_analyze_params_t": s.spmv.spmv_analyze_params_t, "spmv_analysis_info_t": s.spmv.spmv_analysis_info_t,
               "spmv_analysis_host_t": s.spmv.spmv_analysis_host_t}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "spmv_mi355.h"', 'int main(void) {']
    for name, cls in structs.items():
        lines.append(f'  printf("{name} size %zu\\n", sizeof({name}));')
        for field, _ in cls._fields_:
            lines.append(f'  printf("{name} {field} %zu\\n", offsetof({name}, {field}));')
    lines += ['  printf("SPMV_MAX_SIZE %lld\\n", (long long)SPMV_MAX_SIZE);', '  printf("SPMV_SPMM_WINDOW %d\\n", SPMV_SPMM_WINDOW);',
              '  printf("SPMV_TP_SNAP %d\\n", SPMV_TP_SNAP);', '  printf("SPMV_SELL_HEIGHT %d\\n", SPMV_SELL_HEIGHT);',
              '  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", f"-I{ROOT / 'include'}", str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, stdout=subprocess.PIPE, text=True).stdout.split("\n")
    seen = {}
    for line in filter(None, out):
        parts = line.split()
        seen[tuple(parts[:-1])] = int(parts[-1])
    for name, cls in structs.items():
        assert seen[(name, "size")] == C.sizeof(cls), name
        for field, _ in cls._fields_:
            assert seen[(name, field)] == getattr(cls, field).offset, (name, field)
        assert len([k for k in seen if k[0] == name]) == len(cls._fields_) + 1
    assert seen[("SPMV_MAX_SIZE",)] == s.SPMV_MAX_SIZE and seen[("SPMV_SPMM_WINDOW",)] == 4096
    assert seen[("SPMV_TP_SNAP",)] == s.SPMV_TP_SNAP == oracle.TP_SNAP and seen[("SPMV_SELL_HEIGHT",)] == s.SPMV_SELL_HEIGHT == oracle.SELL_HEIGHT
