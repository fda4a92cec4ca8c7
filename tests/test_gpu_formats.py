"""GPU parity of spmv_coo_run / spmv_csc_run / spmv_ell_run (paper App. C tasks 8, 10, 14) against their oracles."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_07169_amd as s
import workloads as w
from gpu_util import DTYPE_CODE, TOL, to_dev

pytestmark = pytest.mark.gpu


def log(*a):
    print(*a, flush=True)


def bound(p, S, alpha, beta, y0):
    return TOL[p.dtype] * (abs(alpha) * S + (np.abs(np.float64(np.float32(beta)) * y0) if beta != 0 else 0.0))


def y_init(p):
    return p.y0 if p.y0 is not None else np.linspace(-1, 1, p.m, dtype=np.float32)


def problems(dtype):
    return w.tiny_adversarial(dtype=dtype) + [w.uniform_rows(3000, 2500, 11, dtype=dtype, beta=0.5), w.powerlaw(20000, dtype=dtype),
                                              w.laplace2d(64, dtype=dtype), w.block_clustered(3000, dtype=dtype),
                                              w.density_random(4096, 2048, 0.01, dtype=dtype, alpha=-1.5, beta=2.0)]


def check(p, y, y_ref, S, what):
    err = np.abs(y.astype(np.float64) - y_ref)
    bad = np.flatnonzero(~(err <= bound(p, S, p.alpha, p.beta, y_init(p))))
    assert bad.size == 0, (what, p.name, int(bad[0]), float(err[bad[0]]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_coo(dtype):
    for p in problems(dtype):
        y0 = y_init(p)
        for seed in (None, 5):      # CSR order (runs of equal rows), and scrambled (hardly any run)
            log("case coo", p.name, dtype, seed)
            row, col, vals = w.to_coo(p, seed)
            y_ref, S = oracle.spmv_coo(dtype, p.m, p.n, row, col, vals, p.x, y0, p.alpha, p.beta)
            d = [to_dev(a) for a in (row, col, vals, p.x)]
            y = to_dev(y0.copy())
            st = s.spmv_coo_run(p.m, p.n, p.nnz, *[t.data_ptr() if t.numel() else None for t in d[:3]], DTYPE_CODE[dtype],
                                d[3].data_ptr(), y.data_ptr(), p.alpha, p.beta)
            assert st == s.SPMV_OK
            torch.cuda.synchronize()
            check(p, y.cpu().numpy(), y_ref, S, "coo")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_csc(dtype):
    # the last three: few rows and long columns, which two workgroups per stretch of columns share by halves of the rows
    few_rows = [w.from_row_lengths([50, 0, 60, 33, 1, 0, 47], 20, seed=3, dtype=dtype, beta=-0.5, allow_dup=True),
                w.from_row_lengths([400, 300], 37, seed=4, dtype=dtype, allow_dup=True),
                w.density_random(2048, 1 << 13, 0.01, dtype=dtype)]
    for p in problems(dtype) + few_rows:
        log("case csc", p.name, dtype)
        y0 = y_init(p)
        co, row, vals = w.to_csc(p)
        y_ref, S = oracle.spmv_csc(dtype, p.m, p.n, co, row, vals, p.x, y0, p.alpha, p.beta)
        d = [to_dev(a) for a in (co, row, vals, p.x)]
        y = to_dev(y0.copy())
        st = s.spmv_csc_run(p.m, p.n, p.nnz, d[0].data_ptr(), *[t.data_ptr() if t.numel() else None for t in d[1:3]],
                            DTYPE_CODE[dtype], d[3].data_ptr(), y.data_ptr(), p.alpha, p.beta)
        assert st == s.SPMV_OK
        torch.cuda.synchronize()
        check(p, y.cpu().numpy(), y_ref, S, "csc")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ell(dtype):
    for p in problems(dtype):
        if np.diff(p.rowptr).max(initial=0) * p.m > 40_000_000:
            continue      # a single very long row would pad every row to its length
        y0 = y_init(p)
        for extra in (0, 5):
            log("case ell", p.name, dtype, extra)
            width, ci, vals = w.to_ell(p, int(np.diff(p.rowptr).max(initial=0)) + extra)
            y_ref, S = oracle.spmv_ell(dtype, p.m, p.n, width, ci, vals, p.x, y0, p.alpha, p.beta)
            d = [to_dev(a) for a in (ci, vals, p.x)]
            y = to_dev(y0.copy())
            st = s.spmv_ell_run(p.m, p.n, width, *[t.data_ptr() if t.numel() else None for t in d[:2]], DTYPE_CODE[dtype],
                                d[2].data_ptr(), y.data_ptr(), p.alpha, p.beta)
            assert st == s.SPMV_OK
            torch.cuda.synchronize()
            check(p, y.cpu().numpy(), y_ref, S, "ell")


def test_exact_integer_inputs_agree_bit_for_bit_in_every_layout():
    """Integer-valued inputs: no rounding in any order, so atomics and reductions must hit the oracle exactly."""
    lens = [0, 1, 2, 3, 17, 64, 255, 256, 257, 0, 0, 1000, 5, 31, 33]
    p = w.exact_integer(lens, 1500, alpha=3.0, beta=-2.0)
    y_ref, _ = oracle.spmv_csr("f32", p.m, p.n, p.rowptr, p.colidx, p.vals, p.x, p.y0, p.alpha, p.beta)
    x = to_dev(p.x)
    row, col, vals = w.to_coo(p, 9)
    y = to_dev(p.y0.copy())
    assert s.spmv_coo_run(p.m, p.n, p.nnz, to_dev(row).data_ptr(), to_dev(col).data_ptr(), to_dev(vals).data_ptr(), 0,
                          x.data_ptr(), y.data_ptr(), p.alpha, p.beta) == s.SPMV_OK
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().astype(np.float64), y_ref)
    co, row, vals = w.to_csc(p)
    y = to_dev(p.y0.copy())
    assert s.spmv_csc_run(p.m, p.n, p.nnz, to_dev(co).data_ptr(), to_dev(row).data_ptr(), to_dev(vals).data_ptr(), 0,
                          x.data_ptr(), y.data_ptr(), p.alpha, p.beta) == s.SPMV_OK
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().astype(np.float64), y_ref)
    width, ci, vals = w.to_ell(p)
    y = to_dev(p.y0.copy())
    assert s.spmv_ell_run(p.m, p.n, width, to_dev(ci).data_ptr(), to_dev(vals).data_ptr(), 0, x.data_ptr(), y.data_ptr(),
                          p.alpha, p.beta) == s.SPMV_OK
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().astype(np.float64), y_ref)


def test_beta_zero_ignores_nan_and_argument_errors():
    p = w.uniform_rows(500, 400, 7)
    row, col, vals = w.to_coo(p)
    d = [to_dev(a) for a in (row, col, vals, p.x)]
    y = torch.full((p.m,), float("nan"), dtype=torch.float32, device="cuda")
    assert s.spmv_coo_run(p.m, p.n, p.nnz, d[0].data_ptr(), d[1].data_ptr(), d[2].data_ptr(), 0, d[3].data_ptr(), y.data_ptr(), 1.0, 0.0) == s.SPMV_OK
    torch.cuda.synchronize()
    y_ref, S = oracle.spmv_coo("f32", p.m, p.n, row, col, vals, p.x)
    assert np.all(np.abs(y.cpu().numpy() - y_ref) <= 1e-5 * S)
    assert s.spmv_coo_run(p.m, p.n, p.nnz, None, d[1].data_ptr(), d[2].data_ptr(), 0, d[3].data_ptr(), y.data_ptr(), 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    assert s.spmv_coo_run(-1, p.n, p.nnz, d[0].data_ptr(), d[1].data_ptr(), d[2].data_ptr(), 0, d[3].data_ptr(), y.data_ptr(), 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    assert s.spmv_coo_run(p.m, p.n, p.nnz, d[0].data_ptr(), d[1].data_ptr(), d[2].data_ptr(), 7, d[3].data_ptr(), y.data_ptr(), 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    assert s.spmv_csc_run(p.m, p.n, p.nnz, None, d[0].data_ptr(), d[2].data_ptr(), 0, d[3].data_ptr(), y.data_ptr(), 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    assert s.spmv_ell_run(p.m, p.n, -2, d[1].data_ptr(), d[2].data_ptr(), 0, d[3].data_ptr(), y.data_ptr(), 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    # nothing stored: y <- beta*y
    y = to_dev(np.arange(5, dtype=np.float32))
    assert s.spmv_coo_run(5, 3, 0, None, None, None, 0, d[3].data_ptr(), y.data_ptr(), 1.0, 2.0) == s.SPMV_OK
    assert s.spmv_ell_run(5, 3, 0, None, None, 0, d[3].data_ptr(), y.data_ptr(), 1.0, 0.5) == s.SPMV_OK
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy(), np.arange(5, dtype=np.float32))
    # no columns at all: every slot is padding, x may point at nothing
    ci = to_dev(np.full(5 * 4, -1, np.int32))
    assert s.spmv_ell_run(5, 0, 4, ci.data_ptr(), d[2].data_ptr(), 0, None, y.data_ptr(), 1.0, 3.0) == s.SPMV_OK
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy(), 3 * np.arange(5, dtype=np.float32))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ell_widths_around_the_tile_limits_with_garbage_in_the_padding(dtype):
    """Widths 1..513 (rows of up to 64 slots are staged through LDS, wider ones are not), row counts that are
    no multiple of a tile, misaligned arrays, and NaN / Inf in the padding slots' values, which must be ignored."""
    rng = np.random.default_rng(17)
    for width, m, off in [(1, 1000, 0), (3, 777, 0), (7, 2049, 1), (8, 300, 0), (27, 5001, 0), (27, 5001, 3), (63, 900, 0), (64, 901, 1), (65, 902, 0), (100, 333, 0),
                          (511, 70, 0), (512, 41, 0), (513, 40, 0), (16, 256, 0), (16, 257, 2)]:
        lens = rng.integers(0, width + 1, m)
        lens[rng.integers(0, m, 3)] = width
        p = w.from_row_lengths(lens, max(width, 600), seed=width, dtype=dtype, beta=0.5, alpha=-2.0, allow_dup=True)
        log("case ell width", width, m, off, dtype)
        got_width, ci, vals = w.to_ell(p, width)
        assert got_width == width
        vals = vals.copy()
        pad = ci < 0
        junk = np.array([np.nan, np.inf, -np.inf, 3e38], np.float32)[rng.integers(0, 4, int(pad.sum()))]
        vals[pad] = junk if dtype == "f32" else w.f32_to_bf16_bits(np.nan_to_num(junk, nan=3e38, posinf=3e38, neginf=-3e38)) | np.uint16(0x7F80)
        y0 = y_init(p)
        y_ref, S = oracle.spmv_ell(dtype, p.m, p.n, width, ci, vals, p.x, y0, p.alpha, p.beta)
        assert np.all(np.isfinite(y_ref))
        d = [to_dev(ci, off), to_dev(vals, off), to_dev(p.x)]
        y = to_dev(y0.copy())
        assert s.spmv_ell_run(p.m, p.n, width, d[0].data_ptr(), d[1].data_ptr(), DTYPE_CODE[dtype], d[2].data_ptr(),
                              y.data_ptr(), p.alpha, p.beta) == s.SPMV_OK
        torch.cuda.synchronize()
        check(p, y.cpu().numpy(), y_ref, S, "ell widths")
    # no columns at all: every slot is padding and x points at nothing
    ci = np.full((50, 4), -1, np.int32).reshape(-1)
    y = to_dev(np.ones(50, np.float32))
    assert s.spmv_ell_run(50, 0, 4, to_dev(ci).data_ptr(), to_dev(np.zeros(200, np.float32)).data_ptr(), 0,
                          to_dev(np.zeros(1, np.float32)).data_ptr(), y.data_ptr(), 1.0, 3.0) == s.SPMV_OK
    torch.cuda.synchronize()
    assert np.all(y.cpu().numpy() == 3.0)
