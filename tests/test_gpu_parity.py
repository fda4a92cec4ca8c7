"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Floating point within the stated per-row bound (1e-5 * sum|a x| for FP32,
8e-3 * sum|a x| for bf16 storage); integer-valued inputs and analysis outputs bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_07169_amd as s
import workloads as w
from gpu_util import (check_patterns_equal_oracle, check_piece_rule, ALL_PLANS, DeviceProblem, assert_close, check_problem, expected_auto_plan, plan_params, reference,
                      to_dev)

pytestmark = pytest.mark.gpu

PLAN_IDS = {p: s.PLAN_NAMES[p] for p in ALL_PLANS}


def log(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ cross-lane reductions
def test_cross_lane_group_sums():
    rng = np.random.default_rng(11)
    v = rng.integers(-1000, 1000, 64).astype(np.float32)     # integers: sums are exact in any order
    d_in = to_dev(v)
    d_out = torch.zeros(14 * 64, dtype=torch.float32, device="cuda")
    s.check(s.spmv_selftest_reduce(d_in.data_ptr(), d_out.data_ptr(), None))
    torch.cuda.synchronize()
    out = d_out.cpu().numpy().reshape(14, 64)
    for gi in range(7):
        G = 1 << gi
        want = np.repeat(v.reshape(64 // G, G).sum(axis=1), G)
        assert np.array_equal(out[gi], want), f"compile-time G={G}"
        assert np.array_equal(out[7 + gi], want), f"run-time G={G}"


# ------------------------------------------------------------------ small adversarial shapes, every plan
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("plan", ALL_PLANS, ids=PLAN_IDS.get)
def test_tiny_adversarial(dtype, plan):
    for p in w.tiny_adversarial(dtype=dtype):
        log("case", p.name, dtype, s.PLAN_NAMES[plan])
        check_problem(p, plan_params(plan), what=s.PLAN_NAMES[plan])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("plan", ALL_PLANS, ids=PLAN_IDS.get)
def test_exact_integer_bit_for_bit(dtype, plan):
    """Integer-valued inputs: every partial sum is an integer below 2^24, so the float32 result
    does not depend on the summation order and must equal the oracle exactly."""
    lens = [0, 1, 2, 3, 4, 5, 7, 8, 9, 63, 64, 65, 255, 256, 257, 2047, 2048, 2049, 0, 0, 4096, 4097, 10000, 1, 1, 200000, 3]
    p = w.exact_integer(lens, 250000, dtype=dtype, alpha=3.0, beta=-2.0)
    log("case exact_integer", dtype, s.PLAN_NAMES[plan])
    d = DeviceProblem(p)
    A = d.matrix(plan_params(plan))
    y = d.run(A)
    y_ref, _ = reference(p)
    assert np.array_equal(y.astype(np.float64), y_ref)
    A.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_exact_integer_many_rows(dtype):
    rng = np.random.default_rng(21)
    lens = np.concatenate([rng.integers(0, 12, 20000), rng.integers(0, 400, 2000), [0] * 5000, rng.integers(0, 12, 3000)])
    p = w.exact_integer(lens, 5000, dtype=dtype, alpha=1.0, beta=1.0)
    y_ref, _ = reference(p)
    d = DeviceProblem(p)
    for plan in ALL_PLANS:
        log("case exact_integer_many_rows", dtype, s.PLAN_NAMES[plan])
        A = d.matrix(plan_params(plan))
        assert np.array_equal(d.run(A).astype(np.float64), y_ref), s.PLAN_NAMES[plan]
        A.close()


# ------------------------------------------------------------------ scaled configs, every plan
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("plan", ALL_PLANS, ids=PLAN_IDS.get)
def test_scaled_configs_every_plan(k, plan):
    p = w.config(k, 1.0 if k == 1 else 1 / 16)
    log("case", p.name, s.PLAN_NAMES[plan])
    check_problem(p, plan_params(plan), strict=True, what=s.PLAN_NAMES[plan])


# ------------------------------------------------------------------ tile-size parameters
@pytest.mark.parametrize("params", [
    dict(plan=4, block_nnz=1, rows_max=1), dict(plan=4, block_nnz=7, rows_max=3), dict(plan=4, block_nnz=8192, rows_max=1024),
    dict(plan=4, block_nnz=64, rows_max=1024), dict(plan=4, block_nnz=8192, rows_max=2),
    dict(plan=5, items_per_chunk=1), dict(plan=5, items_per_chunk=5), dict(plan=5, items_per_chunk=63),
    dict(plan=5, items_per_chunk=8192), dict(plan=2, vector_lanes=2), dict(plan=2, vector_lanes=64),
], ids=str)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_tile_parameters(params, dtype):
    rng = np.random.default_rng(31)
    lens = np.concatenate([rng.integers(0, 30, 700), [9000, 0, 0, 1, 8193, 8192, 8191], rng.integers(0, 300, 150)])
    p = w.from_row_lengths(lens, 20000, seed=77, dtype=dtype, alpha=1.5, beta=0.25)
    log("case tile_parameters", params, dtype)
    check_problem(p, params)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("plan", ALL_PLANS, ids=PLAN_IDS.get)
def test_misaligned_arrays(dtype, plan):
    """colidx / vals / x starting 1 element into an allocation: no 16-byte alignment, so the
    128-bit load paths must not be taken."""
    q = w.powerlaw(20000, dtype=dtype)
    log("case misaligned", dtype, s.PLAN_NAMES[plan])
    check_problem(q, plan_params(plan), offset_elems=1)


# ------------------------------------------------------------------ scalars, streams, reuse
def test_beta_zero_ignores_nan_in_y():
    p = w.config(2, 1 / 16)
    d = DeviceProblem(p)
    y_ref, S_ref = reference(p, 1.0, 0.0)
    nan_y = torch.full((p.m,), float("nan"), dtype=torch.float32, device="cuda")
    for plan in ALL_PLANS:
        A = d.matrix(plan_params(plan))
        y = d.run(A, 1.0, 0.0, y_init=nan_y)
        assert np.all(np.isfinite(y))
        assert_close(p, y, y_ref, S_ref, 1.0, 0.0, strict=True)
        A.close()


def test_alpha_beta_grid_and_reuse_on_side_stream():
    p = w.config(4, 1 / 100)
    d = DeviceProblem(p)
    A = d.matrix()
    st = torch.cuda.Stream()
    for alpha, beta in [(1.0, 0.0), (0.0, 1.0), (-2.5, 0.75), (1.0, 1.0), (0.0, 0.0)]:
        q = w.CsrProblem(p.name, p.dtype, p.m, p.n, p.rowptr, p.colidx, p.vals, p.x,
                         np.random.default_rng(1).uniform(-1, 1, p.m).astype(np.float32), alpha, beta)
        y0 = to_dev(q.y0)
        with torch.cuda.stream(st):
            y = y0.clone()
            A.run(d.x, y, alpha, beta, st.cuda_stream)
        st.synchronize()
        y_ref, S_ref = reference(q)
        assert_close(q, y.cpu().numpy(), y_ref, S_ref, alpha, beta)
    A.close()


def test_run_is_repeatable_bit_for_bit():
    """Every plan but COLBLOCK (float atomics) gives the same bits on every run."""
    for k in (2, 4):
        p = w.config(k, 1 / 16)
        d = DeviceProblem(p)
        A = d.matrix()
        assert A.info.plan != s.SPMV_PLAN_COLBLOCK
        y1 = d.run(A)
        y2 = d.run(A)
        assert np.array_equal(y1, y2)
        A.close()


# ------------------------------------------------------------------ analysis read back from the device
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_device_analysis_equals_oracle(k):
    p = w.config(k, 1.0 if k == 1 else 1 / 8)
    d = DeviceProblem(p)
    A = d.matrix()
    assert (A.info.block_nnz, A.info.rows_max) == oracle.tile_shape(p.m, p.nnz) and A.info.items_per_chunk == 2048
    got = A.analysis()
    cnt, off, rows = oracle.row_bins(p.rowptr)
    assert np.array_equal(got["bin_count"], cnt) and np.array_equal(got["bin_offset"], off)
    assert np.array_equal(got["bin_rows"], rows)
    assert np.array_equal(got["row_blocks"], oracle.row_blocks(p.rowptr, A.info.block_nnz, A.info.rows_max))
    mr, mz = oracle.merge_path(p.rowptr, A.info.items_per_chunk)
    assert np.array_equal(got["mp_row"], mr) and np.array_equal(got["mp_nz"], mz)
    st = oracle.row_stats(p.rowptr)
    assert A.info.plan == expected_auto_plan(p, A.info)
    assert (A.info.min_len, A.info.max_len, A.info.n_empty) == (st["min_len"], st["max_len"], st["n_empty"])
    A.close()


def check_windows_equal_oracle(p, A):
    got = A.analysis()
    ve = 8 if p.dtype == "bf16" else 4
    nv, xv_ptr, xv_start, lidx = oracle.x_windows(p.rowptr, p.colidx, got["row_blocks"], A.info.block_nnz, ve)
    assert A.info.num_x_vectors == xv_start.size and A.info.max_x_vectors == (nv.max() if nv.size else 0)
    assert np.array_equal(got["xv_ptr"], xv_ptr)
    assert np.array_equal(got["xv_start"], xv_start)
    assert np.array_equal(got["lidx"], lidx)
    grouped = oracle.lidx_grouped(p.rowptr, got["row_blocks"], lidx)
    assert A.info.lidx_grouped == int(grouped)
    check_patterns_equal_oracle(p, A, got, lidx, grouped)
    # the fixed-stride copy: block b's vectors at b*V, then -1
    V = max(1, int(A.info.max_x_vectors))
    pad = np.full((nv.size, V), -1, np.int32)
    for b in range(nv.size):
        pad[b, :nv[b]] = xv_start[xv_ptr[b]:xv_ptr[b + 1]]
    assert np.array_equal(got["xv_pad"].reshape(nv.size, V), pad)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", ["laplace", "stencil27", "broken", "unaligned", "wide_blocks", "reversed"])
def test_row_patterns_of_window_positions(dtype, shape):
    """Stencils: the window positions of a row are those of the row before plus a constant, so the kernel works from a
    few runs per block instead of the position stream and the row offsets.  Rows that break the pattern in the middle
    of a block (more than four runs: that block falls back to its positions; up to four: it stays patterned), arrays
    off their allocations, blocks of more rows than a workgroup has lanes, columns stored in descending order (a row's
    first entry no longer sits lowest: no pattern).  The runs and pattern lists bit for bit, and the product, each time."""
    params = None
    if shape == "stencil27":
        p = w.stencil27(24, dtype=dtype, alpha=0.75, beta=-0.5)
        p.y0 = np.linspace(-1, 1, p.m, dtype=np.float32)
        params = dict(rows_max=24, block_nnz=24 * 27)          # one grid line per block: three runs
    elif shape == "wide_blocks":
        p = w.laplace2d(640, dtype=dtype, alpha=-1.25, beta=0.5)
        params = dict(rows_max=640, block_nnz=3200)            # one grid line per block: 640 rows for 256 lanes
    else:
        p = w.laplace2d(160, dtype=dtype, alpha=-1.25, beta=0.5)
    colidx, vals = p.colidx.copy(), p.vals
    if shape == "broken":
        # default blocks hold 64 rows here; blocks 10 and 20 start a grid line.  Block 10: three rows apart lose their
        # pattern (eight runs: positions again).  Block 20: one row does (four runs: still patterned).  The right
        # neighbour's column moves two further.
        for r in (10 * 64 + 9, 10 * 64 + 30, 10 * 64 + 50, 20 * 64 + 33):
            k = p.rowptr[r] + int(np.flatnonzero(colidx[p.rowptr[r]:p.rowptr[r + 1]] == r + 1)[0])
            colidx[k] = r + 3
    if shape == "reversed":
        for r in range(p.m):
            colidx[p.rowptr[r]:p.rowptr[r + 1]] = colidx[p.rowptr[r]:p.rowptr[r + 1]][::-1]
        vals = p.vals.copy()
        for r in range(p.m):
            vals[p.rowptr[r]:p.rowptr[r + 1]] = vals[p.rowptr[r]:p.rowptr[r + 1]][::-1]
    q = w.CsrProblem(p.name + "_" + shape, p.dtype, p.m, p.n, p.rowptr, colidx, vals, p.x, p.y0, p.alpha, p.beta)
    log("case row patterns", dtype, shape, q.nnz)
    d = DeviceProblem(q, offset_elems=1 if shape == "unaligned" else 0)
    A = d.matrix(params)
    assert A.info.plan == s.SPMV_PLAN_WINDOWED
    assert A.info.lidx_patterned == (0 if shape == "reversed" else 1)
    assert s.spmv_csr_main_kernel_name(A.handle) == ("spmv_window_kernel" if shape == "reversed" else "spmv_pattern_kernel")
    got = A.analysis()
    ve = 8 if dtype == "bf16" else 4
    _, _, _, lidx = oracle.x_windows(q.rowptr, q.colidx, got["row_blocks"], A.info.block_nnz, ve)
    want = check_patterns_equal_oracle(q, A, got, lidx, False)
    if shape == "broken":
        assert want["n_runs"][10] == 0 and want["n_runs"][20] == 4 and (np.delete(want["n_runs"], 10) > 0).all()
    elif shape != "reversed":
        assert (want["n_runs"] > 0).all()
    check_windows_equal_oracle(q, A)
    y_ref, S_ref = reference(q)
    assert_close(q, d.run(A), y_ref, S_ref, q.alpha, q.beta)
    y1 = d.run(A)
    assert np.array_equal(y1, d.run(A))       # no atomics on the path: the same bits again
    A.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", ["whole", "unaligned", "tail", "one_off", "shifted"])
def test_grouped_window_positions(dtype, shape):
    """Rows made of aligned runs of eight columns: one window position per group of eight entries is read.  With a
    tail of fewer than eight entries it still is (the tail goes element by element); with one run broken by a
    skipped column, or every block start moved off the multiples of eight, it is not.  Product against the oracle each time."""
    p = w.block_clustered(m=5000, n=40_000, blocks_per_row=12, width=8, dtype=dtype, alpha=1.5, beta=0.25)
    rowptr, colidx, vals = p.rowptr.copy(), p.colidx.copy(), p.vals.copy()
    if shape == "tail":                       # the last row loses three entries
        rowptr[-1] -= 3
        colidx, vals = colidx[:-3], vals[:-3]
    elif shape == "one_off":                  # one run of eight skips a column: its last entry sits one further
        colidx[96 * 2500 + 8 + 7] += 1
    elif shape == "shifted":                  # the first row loses its first entry: every later row starts off the multiples of eight
        rowptr[1:] -= 1
        colidx, vals = colidx[1:], vals[1:]
    q = w.CsrProblem(p.name + "_" + shape, p.dtype, p.m, p.n, rowptr, colidx, vals, p.x, p.y0, p.alpha, p.beta)
    log("case grouped positions", dtype, shape, q.nnz)
    d = DeviceProblem(q, offset_elems=1 if shape == "unaligned" else 0)   # vals, colidx and x one element off their allocations
    A = d.matrix(plan_params(s.SPMV_PLAN_WINDOWED))
    assert A.info.plan == s.SPMV_PLAN_WINDOWED
    assert A.info.lidx_grouped == (1 if shape in ("whole", "unaligned", "tail") else 0)
    check_windows_equal_oracle(q, A)
    y_ref, S_ref = reference(q)
    assert_close(q, d.run(A), y_ref, S_ref, q.alpha, q.beta)
    A.close()


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_x_windows_equal_oracle(k):
    """The device-built x windows, bit for bit, on every config (forced, with blocks small enough
    for any column pattern) and under the automatic plan where it picks them."""
    p = w.config(k, 1.0 if k == 1 else 1 / 8)
    d = DeviceProblem(p)
    log("case x windows forced", p.name)
    A = d.matrix(plan_params(s.SPMV_PLAN_WINDOWED))
    assert A.info.plan == s.SPMV_PLAN_WINDOWED
    check_windows_equal_oracle(p, A)
    A.close()
    A = d.matrix()
    log("case x windows auto", p.name, s.PLAN_NAMES[A.info.plan])
    assert (A.info.plan == s.SPMV_PLAN_WINDOWED) == (k in (2, 3, 5))
    if A.info.plan == s.SPMV_PLAN_WINDOWED:
        check_windows_equal_oracle(p, A)
    A.close()


def test_x_windows_ragged_and_long_rows():
    rng = np.random.default_rng(41)
    lens = np.concatenate([rng.integers(0, 30, 700), [3000, 0, 0, 1, 1025, 1024, 1023], rng.integers(0, 300, 150)])
    for dtype in ("f32", "bf16"):
        p = w.from_row_lengths(lens, 20000, seed=78, dtype=dtype, allow_dup=True, sort_cols=False)
        d = DeviceProblem(p)
        for params in (dict(plan=6, block_nnz=1024, rows_max=64), dict(plan=6, block_nnz=300, rows_max=1024),
                       dict(plan=6, block_nnz=5, rows_max=2)):
            log("case x windows ragged", dtype, params)
            A = d.matrix(params)
            check_windows_equal_oracle(p, A)
            A.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("block_nnz", [2048, 4096, 8192])
def test_windowed_large_windows(dtype, block_nnz):
    """Random columns over a narrow x: blocks of thousands of entries touch 850..1000 distinct x
    vectors, so a lane fetches up to four of them and stages more than one round of entry groups."""
    n = 4000 if dtype == "f32" else 8000
    p = w.uniform_rows(6000, n, 24, dtype=dtype)
    d = DeviceProblem(p)
    log("case windowed large windows", dtype, block_nnz)
    A = d.matrix(dict(plan=6, block_nnz=block_nnz, rows_max=1024))
    assert 512 < A.info.max_x_vectors <= 1024
    y_ref, S_ref = reference(p)
    assert_close(p, d.run(A), y_ref, S_ref, p.alpha, p.beta, strict=True)
    check_windows_equal_oracle(p, A)
    A.close()


def test_forced_windowed_rejects_blocks_with_too_many_vectors():
    p = w.uniform_rows(4096, 1 << 20, 16)  # 8192-entry blocks of random columns: about 8000 distinct vectors
    d = DeviceProblem(p)
    st, h = s.spmv_csr_create(p.m, p.n, p.nnz, d.rowptr.data_ptr(), d.colidx.data_ptr(), d.vals.data_ptr(), 0)
    assert st == s.SPMV_OK
    assert s.spmv_csr_analyze(h, dict(plan=6, block_nnz=8192, rows_max=1024)) == s.SPMV_ERR_UNSUPPORTED
    assert s.spmv_csr_run(h, d.x.data_ptr(), d.y0.data_ptr(), 1.0, 0.0) == s.SPMV_ERR_NOT_ANALYZED
    assert s.spmv_csr_analyze(h) == s.SPMV_OK  # the automatic plan falls back to the tile kernel
    st, info = s.spmv_csr_get_analysis_info(h)
    assert info.plan == s.SPMV_PLAN_ADAPTIVE
    s.spmv_destroy(h)


@pytest.mark.parametrize("dtype,n", [("f32", 3_500_000), ("bf16", 5_000_000), ("f32", 4000)])
def test_column_blocks_equal_oracle_and_multiply(dtype, n):
    """Forced COLBLOCK plan on matrices wide enough for several column blocks (and one that has a single
    block): the regrouping read back bit for bit, and the product within tolerance."""
    rng = np.random.default_rng(77)
    lens = np.concatenate([rng.integers(0, 40, 20000), [3000, 0, 0, 1], rng.integers(0, 5, 5000)])
    p = w.from_row_lengths(lens, n, seed=5, dtype=dtype, alpha=1.5, beta=-0.5, sort_cols=(dtype == "f32"))
    d = DeviceProblem(p)
    log("case column blocks", dtype, n, p.nnz)
    A = d.matrix(dict(plan=s.SPMV_PLAN_COLBLOCK))
    width = oracle.column_block_width(dtype)
    assert A.info.plan == s.SPMV_PLAN_COLBLOCK and A.info.col_block_width == width
    assert A.info.num_col_blocks == -(-n // width)
    got = A.analysis()
    ptr, row, col, src = oracle.column_blocks(p.m, p.n, p.rowptr, p.colidx, width)
    assert np.array_equal(got["cb_ptr"], ptr) and np.array_equal(got["cb_src"], src)
    assert np.array_equal(got["cb_row"], row) and np.array_equal(got["cb_col"], col)
    y_ref, S_ref = reference(p)
    assert_close(p, d.run(A), y_ref, S_ref, p.alpha, p.beta)
    A.close()


TP_ARRAYS = ("tp_row", "tp_nz", "tp_piece_c", "tp_piece_g", "tp_chunk_g", "tp_col", "tp_src", "tp_from", "tp_pos")


@pytest.mark.parametrize("dtype,n", [("f32", 100_000), ("bf16", 70_001), ("f32", 4000)])
def test_two_phase_layout_equals_oracle_and_multiplies(dtype, n):
    """Forced TWOPHASE plan on matrices with several column blocks and chunks (and one with a single block):
    the regrouping read back bit for bit, the product within tolerance and the same bits on every run."""
    rng = np.random.default_rng(78)
    lens = np.minimum(np.concatenate([rng.integers(0, 40, 20000), [30000, 0, 0, 1], rng.integers(0, 5, 5000), [9000, 9000]]), n)
    p = w.from_row_lengths(lens, n, seed=6, dtype=dtype, alpha=1.5, beta=-0.5, sort_cols=(dtype == "f32"),
                           allow_dup=(dtype == "bf16"))
    d = DeviceProblem(p, offset_elems=1 if dtype == "f32" else 0)
    log("case two-phase layout", dtype, n, p.nnz)
    A = d.matrix(dict(plan=s.SPMV_PLAN_TWOPHASE))
    info = A.info
    assert info.plan == s.SPMV_PLAN_TWOPHASE and info.tp_col_shift == oracle.TP_SHIFT and info.tp_items == oracle.TP_ITEMS
    L = oracle.two_phase_layout(p.m, p.n, p.rowptr, p.colidx, piece_groups=info.tp_piece_groups)
    check_piece_rule(L, info)
    assert (info.tp_num_col_blocks, info.tp_num_chunks, info.tp_slots, info.tp_num_pieces) == (L["C"], L["P"], L["S"], L["Q"])
    got = A.analysis()
    for k in TP_ARRAYS:
        assert np.array_equal(got[k], L[k]), k
    y_ref, S_ref = reference(p)
    y = d.run(A)
    assert_close(p, y, y_ref, S_ref, p.alpha, p.beta)
    assert np.array_equal(d.run(A), y)
    A.close()


@pytest.mark.parametrize("which", ["wide_bf16", "powerlaw_1M_f32", "too_few_entries", "x_too_small", "x_just_enough", "banded", "banded_wide"])
def test_auto_and_the_two_pass_plan(which):
    """AUTO = TWOPHASE from x of 256 KiB and 1.5 * 2^22 entries on (tiles of eight entries or more), not below."""
    rng = np.random.default_rng(5)
    if which == "wide_bf16":            # 4.3 M bf16 columns, 5 M... entries: not enough; 7 M are
        p = w.from_row_lengths(rng.integers(4, 11, 1_000_000), 4_300_000, seed=9, dtype="bf16", alpha=-2.0, beta=1.0)
    elif which == "powerlaw_1M_f32":    # x of 4 MB, 8.2 M entries
        p = w.powerlaw(1_000_000)
    elif which == "too_few_entries":    # 6.0 M entries
        p = w.from_row_lengths(np.full(1_000_000, 6), 1_048_576, seed=3)
    elif which == "banded_wide":        # x beyond two 4 MiB stretches as well: neither regrouping plan takes clustered columns
        p = w.banded_random(2_200_000, 2048, 16)
    elif which == "banded":             # big enough, but the columns cluster (a band too wide for the x windows): row-wise gathers stay cheap
        p = w.banded_random(1 << 20, 2048, 16)
    elif which == "x_just_enough":      # x of exactly 256 KiB, 7 M entries
        p = w.from_row_lengths(np.full(1_000_000, 7), 65_536, seed=4)
    else:                               # one column short of 256 KiB
        p = w.from_row_lengths(np.full(1_000_000, 7), 65_535, seed=4)
    log("case auto two-pass", which, p.nnz)
    d = DeviceProblem(p)
    A = d.matrix()
    want = s.SPMV_PLAN_TWOPHASE if which in ("wide_bf16", "powerlaw_1M_f32", "x_just_enough") else s.SPMV_PLAN_ADAPTIVE
    assert A.info.plan == want == expected_auto_plan(p, A.info)
    y_ref, S_ref = reference(p)
    assert_close(p, d.run(A), y_ref, S_ref, p.alpha, p.beta)
    A.close()


@pytest.mark.parametrize("seed", range(8))
def test_two_phase_seeded_random_shapes(seed):
    """Several column blocks and chunks, row-length mixes with empty and very long rows, both storage types, x and the
    matrix arrays at odd offsets: layout bit for bit, product within tolerance."""
    rng = np.random.default_rng(2000 + seed)
    dtype = "f32" if seed % 2 == 0 else "bf16"
    m = int(rng.integers(1, 120_000))
    n = int(rng.integers(1, 200_000))
    kind = seed % 4
    if kind == 0:
        lens = rng.integers(0, min(n, 30) + 1, m)
    elif kind == 1:
        lens = np.minimum(w.powerlaw_lengths(rng, m, cap=60_000), n)
    elif kind == 2:
        lens = np.where(rng.random(m) < 0.8, 0, rng.integers(0, min(n, 300) + 1, m))
    else:
        lens = np.concatenate([[min(n, 40_000)], np.zeros(min(m, 20_000), np.int64), rng.integers(0, min(n, 12) + 1, max(m - 1, 0))])[:max(m, 1)]
    p = w.from_row_lengths(lens, n, seed=seed, dtype=dtype, alpha=float(rng.uniform(-2, 2)), beta=float(rng.choice([0.0, 1.0, -0.75])),
                           sort_cols=bool(seed & 4), allow_dup=(kind == 2))
    log("case two-phase seeded", seed, dtype, p.m, p.n, p.nnz)
    d = DeviceProblem(p, offset_elems=seed % 3)
    A = d.matrix(dict(plan=s.SPMV_PLAN_TWOPHASE))
    if p.nnz == 0:
        assert A.info.plan == s.SPMV_PLAN_SCALAR
    else:
        L = oracle.two_phase_layout(p.m, p.n, p.rowptr, p.colidx, piece_groups=A.info.tp_piece_groups)
        check_piece_rule(L, A.info)
        got = A.analysis()
        for k in TP_ARRAYS:
            assert np.array_equal(got[k], L[k]), k
    y_ref, S_ref = reference(p)
    assert_close(p, d.run(A), y_ref, S_ref, p.alpha, p.beta)
    A.close()


def test_two_phase_more_column_blocks_than_one_ranking_pass():
    """40 M columns = 2442 column blocks: the placement ranks 2048 blocks per pass over a chunk, so this takes two;
    rows of every length class, columns over the whole width.  Layout bit for bit, product within tolerance."""
    rng = np.random.default_rng(77)
    n = 40_000_000
    lens = np.concatenate([rng.integers(0, 9, 30_000), [25_000, 0, 3], rng.integers(0, 3, 4_000)])
    p = w.from_row_lengths(lens, n, seed=12, dtype="f32", alpha=0.5, beta=1.0)
    log("case two-phase wide", p.m, p.n, p.nnz)
    d = DeviceProblem(p)
    A = d.matrix(dict(plan=s.SPMV_PLAN_TWOPHASE))
    assert A.info.plan == s.SPMV_PLAN_TWOPHASE and A.info.tp_num_col_blocks == (n + (1 << oracle.TP_SHIFT) - 1) >> oracle.TP_SHIFT > 2048
    L = oracle.two_phase_layout(p.m, p.n, p.rowptr, p.colidx, piece_groups=A.info.tp_piece_groups)
    check_piece_rule(L, A.info)
    got = A.analysis()
    for k in TP_ARRAYS:
        assert np.array_equal(got[k], L[k]), k
    y_ref, S_ref = reference(p)
    assert_close(p, d.run(A), y_ref, S_ref, p.alpha, p.beta)
    A.close()


# ------------------------------------------------------------------ the sliced ELL plan
@pytest.mark.parametrize("which", ["mixed_f32", "mixed_bf16", "uniform", "one_row", "long_row", "stencil", "short_last_slice"])
def test_sell_layout_equals_oracle_and_multiplies(which):
    """Forced SELL plan: the sliced copy read back bit for bit (slice bounds, columns, source positions, -1 padding),
    the product within tolerance and the same bits on every run; the kernel name says which kernel ran."""
    rng = np.random.default_rng(91)
    if which.startswith("mixed"):
        lens = np.concatenate([rng.integers(0, 40, 3000), [0] * 130, [300, 0, 1], rng.integers(0, 5, 1000)])
        p = w.from_row_lengths(lens, 5000, seed=8, dtype=which[6:], alpha=1.5, beta=-0.5, allow_dup=True)
    elif which == "uniform":
        p = w.uniform_rows(4096, 4096, 16)
    elif which == "one_row":
        p = w.from_row_lengths(np.array([37]), 64, seed=2, beta=1.0)
    elif which == "long_row":
        p = w.from_row_lengths(np.concatenate([rng.integers(0, 6, 200), [50_000], rng.integers(0, 6, 200)]), 60_000, seed=3, dtype="bf16")
    elif which == "stencil":
        p = w.stencil27(20, dtype="bf16")
    else:
        p = w.from_row_lengths(rng.integers(1, 9, 64 * 5 + 1), 700, seed=5)
    log("case sell", which, p.m, p.nnz)
    d = DeviceProblem(p, offset_elems=1 if which == "mixed_f32" else 0)
    A = d.matrix(dict(plan=s.SPMV_PLAN_SELL))
    L = oracle.sell_layout(p.m, p.rowptr, p.colidx)
    assert A.info.plan == s.SPMV_PLAN_SELL and (A.info.sell_num_slices, A.info.sell_slots) == (L["ns"], L["S"])
    assert s.spmv_csr_main_kernel_name(A.handle) == "spmv_sell_kernel"
    got = A.analysis()
    for k in ("sell_ptr", "sell_col", "sell_src"):
        assert np.array_equal(got[k], L[k]), k
    y_ref, S_ref = reference(p)
    y = d.run(A)
    assert_close(p, y, y_ref, S_ref, p.alpha, p.beta, strict=(p.beta == 0.0))
    assert np.array_equal(d.run(A), y)
    A.close()


def test_sell_does_not_carry_nan_from_x0_into_padded_rows():
    """Padding slots point at no column: whatever x[0] holds (here NaN), a row shorter than its slice is not touched by it."""
    p = w.from_row_lengths(np.array([5, 1, 0, 3] * 40), 49, seed=11)
    x = np.concatenate([[np.float32("nan")], p.x]).astype(np.float32)      # column 0 is read by no entry
    q = w.CsrProblem("no_col0", "f32", p.m, 50, p.rowptr, (p.colidx + 1).astype(np.int32), p.vals, x, None, 1.0, 0.0)
    d = DeviceProblem(q)
    A = d.matrix(dict(plan=s.SPMV_PLAN_SELL))
    y = d.run(A)
    y_ref, S_ref = reference(q)
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(y_ref))
    assert_close(q, y, y_ref, S_ref, 1.0, 0.0, strict=True)
    A.close()


def group_layout(p, info):
    """The two-pass layout of the matrix of groups (what a group-aligned matrix is laid out as), pieces as the handle cut them."""
    rg, cg = oracle.group_matrix(p.m, p.rowptr, p.colidx)
    L = oracle.two_phase_layout(p.m, (p.n + 7) // 8, rg, cg, shift=oracle.TP_GROUP_SHIFT[p.dtype], piece_groups=info.tp_piece_groups)
    check_piece_rule(L, info)
    return L


@pytest.mark.parametrize("dtype,m,n,offset", [("bf16", 20_000, 300_000, 0), ("f32", 9_000, 70_000, 0), ("bf16", 3_000, 40_004, 1),
                                                ("f32", 700, 16_390, 1), ("bf16", 1, 64, 0)])
def test_two_phase_on_groups_layout_equals_oracle_and_multiplies(dtype, m, n, offset):
    """A forced TWOPHASE plan on a group-aligned matrix works on groups of eight entries: the layout read back is the
    oracle's two-pass layout of the matrix of groups, bit for bit; the product is within tolerance and the same on every
    run; x may start off a 16-byte boundary and n need not be a multiple of eight; values refreshed in place are picked up."""
    p = w.block_clustered(m=m, n=n, blocks_per_row=min(16, n // 8), dtype=dtype, alpha=-1.25, beta=0.5)
    p.y0 = np.random.default_rng(3).standard_normal(p.m).astype(np.float32)
    assert oracle.csr_groups(p.m, p.rowptr, p.colidx) == 1
    log("case two-phase on groups", dtype, m, n, p.nnz)
    d = DeviceProblem(p, offset_elems=offset)
    A = d.matrix(dict(plan=s.SPMV_PLAN_TWOPHASE))
    info = A.info
    assert info.plan == s.SPMV_PLAN_TWOPHASE and info.tp_group == 8 and info.tp_col_shift == oracle.TP_GROUP_SHIFT[dtype]
    assert s.spmv_csr_main_kernel_name(A.handle) == "tp_multiply_group_kernel"
    L = group_layout(p, A.info)
    assert (info.tp_num_col_blocks, info.tp_num_chunks, info.tp_slots, info.tp_num_pieces) == (L["C"], L["P"], L["S"], L["Q"])
    got = A.analysis()
    for k in TP_ARRAYS:
        assert np.array_equal(got[k], L[k]), k
    y_ref, S_ref = reference(p)
    y = d.run(A)
    assert_close(p, y, y_ref, S_ref, p.alpha, p.beta)
    assert np.array_equal(d.run(A), y)
    new_vals = np.random.default_rng(9).permutation(p.vals)
    d.vals.copy_(to_dev(new_vals))
    A.refresh_values()
    q = w.CsrProblem(p.name, p.dtype, p.m, p.n, p.rowptr, p.colidx, new_vals, p.x, p.y0, p.alpha, p.beta)
    y2_ref, S2_ref = reference(q)
    assert_close(q, d.run(A), y2_ref, S2_ref, p.alpha, p.beta, what="after refresh")
    A.close()


def test_two_phase_stays_on_entries_when_a_group_is_broken():
    """One column moved inside one group, or a row that starts inside a group: the matrix is no longer group-aligned and a
    forced TWOPHASE plan lays out entries as before."""
    p = w.block_clustered(m=2_000, n=100_000, dtype="bf16")
    for which in ("column", "row"):
        colidx, rowptr = p.colidx.copy(), p.rowptr.copy()
        if which == "column":
            colidx[8 * 777 + 3] += 8                                          # still ascending inside the row, no longer consecutive
        else:
            rowptr[5] += 4
        assert oracle.csr_groups(p.m, rowptr, colidx) == 0
        q = w.CsrProblem("broken_" + which, p.dtype, p.m, p.n, rowptr, colidx, p.vals, p.x, None, 1.0, 0.0)
        d = DeviceProblem(q)
        A = d.matrix(dict(plan=s.SPMV_PLAN_TWOPHASE))
        assert A.info.plan == s.SPMV_PLAN_TWOPHASE and A.info.tp_group == 1
        L = oracle.two_phase_layout(q.m, q.n, q.rowptr, q.colidx, piece_groups=A.info.tp_piece_groups)
        got = A.analysis()
        for k in TP_ARRAYS:
            assert np.array_equal(got[k], L[k]), k
        y_ref, S_ref = reference(q)
        assert_close(q, d.run(A), y_ref, S_ref, 1.0, 0.0, strict=True)
        A.close()


def test_forced_two_phase_rejects_too_many_column_blocks():
    n = 65536 * (1 << oracle.TP_SHIFT) + 1                              # 65537 column blocks
    rowptr, colidx, vals = to_dev(np.array([0, 2], np.int32)), to_dev(np.array([0, n - 1], np.int32)), to_dev(np.ones(2, np.float32))
    st, h = s.spmv_csr_create(1, n, 2, rowptr.data_ptr(), colidx.data_ptr(), vals.data_ptr(), 0)
    assert st == s.SPMV_OK
    assert s.spmv_csr_analyze(h, dict(plan=s.SPMV_PLAN_TWOPHASE)) == s.SPMV_ERR_UNSUPPORTED
    assert s.spmv_csr_analyze(h, dict(plan=s.SPMV_PLAN_SCALAR)) == s.SPMV_OK
    s.spmv_destroy(h)


def test_forced_column_blocks_reject_too_many_blocks():
    p = w.from_row_lengths([3, 0, 5], 17 * (1 << 20) + 1, seed=1)      # 18 blocks of binary32 columns
    d = DeviceProblem(p)
    st, h = s.spmv_csr_create(p.m, p.n, p.nnz, d.rowptr.data_ptr(), d.colidx.data_ptr(), d.vals.data_ptr(), 0)
    assert st == s.SPMV_OK
    assert s.spmv_csr_analyze(h, dict(plan=s.SPMV_PLAN_COLBLOCK)) == s.SPMV_ERR_UNSUPPORTED
    assert s.spmv_csr_analyze(h) == s.SPMV_OK
    s.spmv_destroy(h)


def test_analyze_rejects_bad_input_on_device():
    p = w.config(1)
    d = DeviceProblem(p)
    bad_col = p.colidx.copy()
    bad_col[1234] = p.n
    st, h = s.spmv_csr_create(p.m, p.n, p.nnz, d.rowptr.data_ptr(), to_dev(bad_col).data_ptr(), d.vals.data_ptr(), 0)
    assert st == s.SPMV_OK
    assert s.spmv_csr_analyze(h) == s.SPMV_ERR_BAD_STRUCTURE
    assert s.spmv_csr_run(h, d.x.data_ptr(), d.y0.data_ptr(), 1.0, 0.0) == s.SPMV_ERR_NOT_ANALYZED
    s.spmv_destroy(h)
    bad_rp = p.rowptr.copy()
    bad_rp[10] = bad_rp[11] + 1
    st, h = s.spmv_csr_create(p.m, p.n, p.nnz, to_dev(bad_rp).data_ptr(), d.colidx.data_ptr(), d.vals.data_ptr(), 0)
    assert s.spmv_csr_analyze(h) == s.SPMV_ERR_BAD_STRUCTURE
    s.spmv_destroy(h)


def test_degenerate_shapes():
    e32 = np.zeros(0, np.int32)
    # m == 0: nothing to do
    p = w.CsrProblem("m0", "f32", 0, 5, np.zeros(1, np.int32), e32, np.zeros(0, np.float32), np.ones(5, np.float32), None)
    d = DeviceProblem(p)
    A = d.matrix()
    A.run(d.x, d.y0, 1.0, 0.0)
    A.close()
    # nnz == 0: y <- beta*y for every plan
    y0 = np.arange(7, dtype=np.float32)
    p = w.CsrProblem("nnz0", "f32", 7, 5, np.zeros(8, np.int32), e32, np.zeros(0, np.float32), np.ones(5, np.float32), y0, 1.0, 3.0)
    d = DeviceProblem(p)
    for plan in [0] + ALL_PLANS:
        A = d.matrix(plan_params(plan))
        assert np.array_equal(d.run(A), 3.0 * y0)
        assert np.array_equal(d.run(A, 1.0, 0.0), np.zeros(7, np.float32))
        A.close()


# ------------------------------------------------------------------ HIP graph capture
@pytest.mark.parametrize("k,plan", [(2, 0), (4, 0), (1, 0), (5, 3), (4, 8)])
def test_run_can_be_captured_in_a_graph_and_replayed(k, plan):
    """spmv_csr_run only enqueues kernels (no allocation, copy, memset or synchronisation), so a stream
    capture records it as it is.  Every replay is checked against the eager result, with eager work and
    synchronisations of the program's own in between."""
    p = w.config(k, 1.0 if k == 1 else 1 / 16)
    d = DeviceProblem(p)
    A = d.matrix(dict(plan=plan))
    y_eager = d.run(A)                                   # also sets any per-kernel attribute before the capture
    y = d.y0.clone()
    y_in = d.y0.clone()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        y.copy_(y_in)                                    # beta != 0 reads y: restore it inside the graph
        A.run(d.x, y, p.alpha, p.beta, torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), y_eager), (p.name, rep)
        assert np.array_equal(d.run(A), y_eager)         # eager work between replays
    A.close()


# ------------------------------------------------------------------ seeded random shapes, every plan, random tile parameters
@pytest.mark.parametrize("seed", range(12))
def test_seeded_random_shapes_and_parameters(seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = "f32" if seed % 2 == 0 else "bf16"
    m = int(rng.integers(1, 6000))
    n = int(rng.integers(1, 9000))
    kind = seed % 4
    if kind == 0:
        lens = rng.integers(0, min(n, 40) + 1, m)
    elif kind == 1:
        lens = np.minimum(w.powerlaw_lengths(rng, m), n)
    elif kind == 2:
        lens = np.where(rng.random(m) < 0.7, 0, rng.integers(0, min(n, 700) + 1, m))     # mostly empty rows
    else:
        lens = np.full(m, min(n, int(rng.integers(1, 130))))
    p = w.from_row_lengths(lens, n, seed=seed, dtype=dtype, alpha=float(rng.choice([1.0, -2.0, 0.5])),
                           beta=float(rng.choice([0.0, 1.0, -0.75])), sort_cols=bool(seed % 3), allow_dup=bool(seed % 5 == 0))
    y_ref, S_ref = reference(p)
    d = DeviceProblem(p)
    trials = [dict(plan=pl) for pl in (0, 1, 2, 3, 5, 7)]
    for _ in range(3):
        trials.append(dict(plan=4, block_nnz=int(rng.integers(1, 8193)), rows_max=int(rng.integers(1, 1025))))
        trials.append(dict(plan=6, block_nnz=int(rng.integers(1, 1025)), rows_max=int(rng.integers(1, 1025))))
        trials.append(dict(plan=5, items_per_chunk=int(rng.integers(1, 8193))))
    for params in trials:
        log("case random", seed, p.name, dtype, m, n, params)
        A = d.matrix(params)
        assert_close(p, d.run(A), y_ref, S_ref, p.alpha, p.beta, what=str(params))
        A.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_values_changed_in_place_are_picked_up_after_refresh(dtype):
    """Same structure, new numbers: every plan must give the new product once spmv_csr_refresh_values() has run
    (the plans that read vals directly give it anyway; COLBLOCK holds a regrouped copy)."""
    p = w.powerlaw(30000, dtype=dtype, beta=0.5)
    d = DeviceProblem(p)
    rng = np.random.default_rng(3)
    new_vals = rng.permutation(p.vals)                                       # same bit patterns, shuffled
    p2 = w.CsrProblem(p.name, p.dtype, p.m, p.n, p.rowptr, p.colidx, new_vals, p.x, p.y0, p.alpha, p.beta)
    y_old, S_old = reference(p)
    y_new, S_new = reference(p2)
    for plan in ALL_PLANS:
        log("case refresh", s.PLAN_NAMES[plan], dtype)
        d.vals.copy_(to_dev(p.vals))
        A = d.matrix(plan_params(plan))
        assert_close(p, d.run(A), y_old, S_old, p.alpha, p.beta, what="before")
        d.vals.copy_(to_dev(new_vals))
        A.refresh_values()
        assert_close(p2, d.run(A), y_new, S_new, p.alpha, p.beta, what="after " + s.PLAN_NAMES[plan])
        A.close()



def test_two_handles_on_two_streams_and_one_handle_refusing_a_second_stream():
    """Two handles, each on a stream of its own, overlap freely and both give the oracle's result.  One handle whose plan
    keeps scratch (MERGE, TWOPHASE) refuses a run on a second stream while its last run is still in flight, enqueues
    nothing, and takes the run once the first has finished; a plan without scratch takes both at once."""
    p = w.powerlaw(1_000_000, beta=0.5)
    p.y0 = np.linspace(-1, 1, p.m, dtype=np.float32)
    y_ref, S_ref = reference(p)
    d1, d2 = DeviceProblem(p), DeviceProblem(p)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for plan in (s.SPMV_PLAN_MERGE, s.SPMV_PLAN_TWOPHASE, s.SPMV_PLAN_ADAPTIVE):
        log("case two streams", s.PLAN_NAMES[plan])
        A1, A2 = d1.matrix(dict(plan=plan)), d2.matrix(dict(plan=plan))
        ya, yb = d1.y0.clone(), d2.y0.clone()
        torch.cuda.synchronize()
        for _ in range(3):            # re-runs on a handle's own stream are always in order
            ya.copy_(d1.y0), yb.copy_(d2.y0)
            torch.cuda.synchronize()
            assert s.spmv_csr_run(A1.handle, d1.x.data_ptr(), ya.data_ptr(), p.alpha, p.beta, s1.cuda_stream) == s.SPMV_OK
            assert s.spmv_csr_run(A2.handle, d2.x.data_ptr(), yb.data_ptr(), p.alpha, p.beta, s2.cuda_stream) == s.SPMV_OK
            torch.cuda.synchronize()
            assert_close(p, ya.cpu().numpy(), y_ref, S_ref, p.alpha, p.beta, what="stream 1")
            assert_close(p, yb.cpu().numpy(), y_ref, S_ref, p.alpha, p.beta, what="stream 2")
        # one handle, two streams, no ordering between them
        ya.copy_(d1.y0), yb.copy_(d1.y0)
        torch.cuda.synchronize()
        first = [s.spmv_csr_run(A1.handle, d1.x.data_ptr(), ya.data_ptr(), p.alpha, p.beta, s1.cuda_stream) for _ in range(4)]
        second = s.spmv_csr_run(A1.handle, d1.x.data_ptr(), yb.data_ptr(), p.alpha, p.beta, s2.cuda_stream)
        assert first[0] == s.SPMV_OK
        if plan == s.SPMV_PLAN_ADAPTIVE:
            assert second == s.SPMV_OK
        else:
            assert second == s.SPMV_ERR_BUSY            # four products of 8 M entries cannot have finished yet
            torch.cuda.synchronize()
            assert np.array_equal(yb.cpu().numpy(), d1.y0.cpu().numpy())     # nothing was enqueued
            assert s.spmv_csr_run(A1.handle, d1.x.data_ptr(), yb.data_ptr(), p.alpha, p.beta, s2.cuda_stream) == s.SPMV_OK
        torch.cuda.synchronize()
        assert_close(p, yb.cpu().numpy(), y_ref, S_ref, p.alpha, p.beta, what="second stream")
        A1.close(), A2.close()


def test_analyses_running_at_the_same_time_in_threads():
    """Four threads analyse four different matrices at once, several times over (the host copy of rowptr goes through one
    pinned staging buffer that only one analysis can hold; the others take pageable memory of their own): every handle's
    analysis equals the one made alone, and every product the oracle's."""
    import threading
    probs = [w.powerlaw(300_000 + 1000 * i, seed=50 + i) for i in range(4)]
    devs = [DeviceProblem(p) for p in probs]
    alone = []
    for d in devs:
        A = d.matrix()
        alone.append((A.info.as_dict(), A.analysis()))
        A.close()
    for rep in range(3):
        log("case analyses in threads", rep)
        made, errors = [None] * 4, []

        def work(i):
            try:
                made[i] = devs[i].matrix()
            except Exception as e:                   # noqa: BLE001 - reported below, in the main thread
                errors.append((i, repr(e)))

        threads = [threading.Thread(target=work, args=(i,)) for i in range(4)]
        [t.start() for t in threads]
        [t.join() for t in threads]
        assert not errors, errors
        for i, A in enumerate(made):
            info, got = alone[i]
            assert A.info.as_dict() == info
            now = A.analysis()
            assert now.keys() == got.keys() and all(np.array_equal(now[k], got[k]) for k in got), i
            y_ref, S_ref = reference(probs[i])
            assert_close(probs[i], devs[i].run(A), y_ref, S_ref, probs[i].alpha, probs[i].beta, what="threads")
            A.close()


def test_column_block_refresh_with_columns_the_caller_did_not_check():
    """skip_validation with a column outside the matrix: the regrouping drops that entry, and refreshing the value copy
    must not read through the slot it left unfilled."""
    p = w.uniform_rows(3000, 5000, 9)
    colidx = p.colidx.copy()
    colidx[123] = 1 << 30                                   # far outside every column block
    d = DeviceProblem(p)
    d.colidx.copy_(to_dev(colidx))
    A = d.matrix(dict(plan=s.SPMV_PLAN_COLBLOCK, skip_validation=1))
    A.refresh_values()
    torch.cuda.synchronize()
    got = A.analysis()
    assert got["cb_ptr"][-1] == p.nnz - 1 and got["cb_src"][-1] == -1
    vals = p.vals.copy()
    vals[123] = 0.0                                         # the product without the dropped entry
    q = w.CsrProblem(p.name, p.dtype, p.m, p.n, p.rowptr, p.colidx, vals, p.x, p.y0, p.alpha, p.beta)
    y_ref, S_ref = reference(q)
    assert_close(q, d.run(A), y_ref, S_ref, q.alpha, q.beta, what="dropped entry")
    A.close()
