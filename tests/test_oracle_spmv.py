"""Pins for the CPU oracle of y = alpha*A*x + beta*y (App. C task 12 + BLAS scalars).

Every check here compares the oracle with something that is not the oracle: a dense
numpy matvec, a closed form, an independent library product, exact integer arithmetic
in Python ints, or hand-worked values stored under tests/golden/.
"""
import json

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import workloads as w


def dense_from_csr(p, widen):
    A = np.zeros((p.m, p.n), dtype=np.float64)
    rows = np.repeat(np.arange(p.m), np.diff(p.rowptr))
    np.add.at(A, (rows, p.colidx), widen(p.vals).astype(np.float64))
    return A


def widen_for(dtype):
    return (lambda a: a) if dtype == "f32" else w.bf16_bits_to_f32


# ------------------------------------------------------------------ hand-worked fixture
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_handworked_fixture(golden_dir, dtype):
    g = json.loads((golden_dir / "spmv_3x4_handworked.json").read_text())
    rowptr = np.array(g["rowptr"], dtype=np.int32)
    colidx = np.array(g["colidx"], dtype=np.int32)
    y0 = np.array(g["y0"], dtype=np.float32)
    if dtype == "f32":
        vals = np.array(g["vals"], dtype=np.float32)
        x = np.array(g["x"], dtype=np.float32)
    else:
        vals = np.array([int(s, 16) for s in g["vals_bf16_bits"]], dtype=np.uint16)
        x = np.array([int(s, 16) for s in g["x_bf16_bits"]], dtype=np.uint16)
    y, S = oracle.spmv_csr(dtype, g["m"], g["n"], rowptr, colidx, vals, x, y0, g["alpha"], g["beta"])
    assert y.tolist() == g["y"]
    assert S.tolist() == g["S"]
    y, S = oracle.spmv_csr(dtype, g["m"], g["n"], rowptr, colidx, vals, x, None, 1.0, 0.0)
    assert y.tolist() == g["y_alpha1_beta0"]


# ------------------------------------------------------------------ dense matvec, tiny
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("seed", range(12))
def test_dense_matvec_tiny(dtype, seed):
    rng = np.random.default_rng(seed)
    m = int(rng.integers(1, 65))
    n = int(rng.integers(1, 65))
    lens = rng.integers(0, n + 1, size=m)
    lens[rng.integers(0, m)] = 0          # at least one empty row
    lens[rng.integers(0, m)] = n          # at least one full row
    dup = seed % 3 == 0
    p = w.from_row_lengths(lens, n, seed=100 + seed, dtype=dtype, allow_dup=dup, sort_cols=not (seed % 2),
                           alpha=float(rng.uniform(-2, 2)), beta=float(rng.uniform(-2, 2)), normal=bool(seed % 2))
    A = dense_from_csr(p, widen_for(dtype))
    xw = widen_for(dtype)(p.x).astype(np.float64)
    # alpha/beta are passed to the oracle as C floats
    a32, b32 = float(np.float32(p.alpha)), float(np.float32(p.beta))
    expect = a32 * (A @ xw) + b32 * p.y0.astype(np.float64)
    S_expect = np.abs(A) @ np.abs(xw) if not dup else None
    y, S = oracle.spmv_problem(p)
    scale = np.abs(A) @ np.abs(xw) * abs(a32) + np.abs(b32 * p.y0) + 1e-300
    assert np.all(np.abs(y - expect) <= 1e-13 * scale)
    if S_expect is not None:
        assert np.allclose(S, S_expect, rtol=1e-13, atol=0)


def test_transposed_operand_would_fail():
    """A is not symmetric here; A^T x differs, so an oracle that swapped the roles of
    row and column would not pass the dense pin."""
    p = w.from_row_lengths([2, 0, 3, 1], 4, seed=5)
    A = dense_from_csr(p, lambda a: a)
    y, _ = oracle.spmv_csr("f32", p.m, p.n, p.rowptr, p.colidx, p.vals, p.x)
    assert np.allclose(y, A @ p.x.astype(np.float64), rtol=1e-14)
    assert not np.allclose(y, A.T @ p.x.astype(np.float64), rtol=1e-3)


# ------------------------------------------------------------------ identity / diagonal
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_identity_and_diagonal(dtype):
    rng = np.random.default_rng(3)
    n = 257
    rowptr = np.arange(n + 1, dtype=np.int32)
    colidx = np.arange(n, dtype=np.int32)
    x32 = rng.uniform(-1, 1, n).astype(np.float32)
    d32 = rng.uniform(-3, 3, n).astype(np.float32)
    y0 = rng.uniform(-1, 1, n).astype(np.float32)
    if dtype == "bf16":
        xs, ds, one = w.f32_to_bf16_bits(x32), w.f32_to_bf16_bits(d32), np.full(n, 0x3F80, dtype=np.uint16)
        x64, d64 = w.bf16_bits_to_f32(xs).astype(np.float64), w.bf16_bits_to_f32(ds).astype(np.float64)
    else:
        xs, ds, one = x32, d32, np.ones(n, dtype=np.float32)
        x64, d64 = x32.astype(np.float64), d32.astype(np.float64)
    alpha, beta = 1.5, -0.25   # exact in float32
    y, S = oracle.spmv_csr(dtype, n, n, rowptr, colidx, one, xs, y0, alpha, beta)
    assert np.array_equal(y, alpha * x64 + beta * y0.astype(np.float64))
    assert np.array_equal(S, np.abs(x64))
    y, S = oracle.spmv_csr(dtype, n, n, rowptr, colidx, ds, xs, y0, alpha, beta)
    assert np.array_equal(y, alpha * (d64 * x64) + beta * y0.astype(np.float64))
    # anti-diagonal: picks x in reverse, catches an ignored column index
    y, _ = oracle.spmv_csr(dtype, n, n, rowptr, colidx[::-1].copy(), one, xs, None, 1.0, 0.0)
    assert np.array_equal(y, x64[::-1])


# ------------------------------------------------------------------ A * 1 = row sums
def test_laplacian_times_ones_closed_form():
    g = 37
    p = w.laplace2d(g, beta=0.0)
    ones = np.ones(p.n, dtype=np.float32)
    y, S = oracle.spmv_csr("f32", p.m, p.n, p.rowptr, p.colidx, p.vals, ones)
    ix, iy = np.arange(p.m) % g, np.arange(p.m) // g
    on_edge = (ix == 0).astype(int) + (ix == g - 1) + (iy == 0) + (iy == g - 1)   # 0 interior, 1 edge, 2 corner
    assert np.array_equal(y, on_edge.astype(np.float64))
    assert np.array_equal(S, 8.0 - on_edge)


@pytest.mark.parametrize("k", [1, 3, 4, 5])
def test_row_sums_of_scaled_configs(k):
    p = w.config(k, scale=1 / 64 if k != 1 else 1.0)
    wid = widen_for(p.dtype)
    ones = np.ones(p.n, dtype=np.float32)
    ones = ones if p.dtype == "f32" else w.f32_to_bf16_bits(ones)
    y, S = oracle.spmv_csr(p.dtype, p.m, p.n, p.rowptr, p.colidx, p.vals, ones)
    v = wid(p.vals).astype(np.float64)
    # np.add.reduceat cannot express empty rows; use a cumulative sum in extended precision instead
    cs = np.concatenate(([0.0], np.cumsum(v.astype(np.longdouble))))
    rs = (cs[p.rowptr[1:]] - cs[p.rowptr[:-1]]).astype(np.float64)
    absum = np.concatenate(([0.0], np.cumsum(np.abs(v).astype(np.longdouble))))
    rsa = (absum[p.rowptr[1:]] - absum[p.rowptr[:-1]]).astype(np.float64)
    assert np.all(np.abs(y - rs) <= 1e-9 * (rsa + 1e-300))
    assert np.all(np.abs(S - rsa) <= 1e-9 * (rsa + 1e-300))


# ------------------------------------------------------------------ independent library product
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_against_scipy_csr(k):
    p = w.config(k, scale=1 / 32 if k != 1 else 1.0)
    wid = widen_for(p.dtype)
    A = sp.csr_matrix((wid(p.vals).astype(np.float64), p.colidx, p.rowptr), shape=(p.m, p.n))
    x64 = wid(p.x).astype(np.float64)
    expect = p.alpha * (A @ x64)
    if p.beta != 0.0:
        expect = expect + p.beta * p.y0.astype(np.float64)
    y, S = oracle.spmv_problem(p)
    Sx = abs(A) @ np.abs(x64)
    assert np.all(np.abs(y - expect) <= 1e-13 * (Sx + np.abs(expect) + 1e-300))
    assert np.all(np.abs(S - Sx) <= 1e-13 * (Sx + 1e-300))


# ------------------------------------------------------------------ exact integers, brute force in Python ints
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_exact_integer_bruteforce(dtype):
    lens = [0, 1, 2, 3, 64, 65, 700, 0, 5]
    p = w.exact_integer(lens, 800, dtype=dtype, alpha=3.0, beta=-2.0)
    wid = widen_for(dtype)
    v, x = wid(p.vals), wid(p.x)
    y, S = oracle.spmv_problem(p)
    for i in range(p.m):
        acc, s = 0, 0
        for k in range(p.rowptr[i], p.rowptr[i + 1]):
            t = int(v[k]) * int(x[p.colidx[k]])
            acc += t
            s += abs(t)
        assert y[i] == 3 * acc - 2 * int(p.y0[i])
        assert S[i] == s


# ------------------------------------------------------------------ invariants
def test_linearity_and_row_permutation():
    p = w.config(4, scale=1 / 400)
    rng = np.random.default_rng(0)
    x2 = rng.uniform(-1, 1, p.n).astype(np.float32)
    y1, S1 = oracle.spmv_csr("f32", p.m, p.n, p.rowptr, p.colidx, p.vals, p.x)
    y2, S2 = oracle.spmv_csr("f32", p.m, p.n, p.rowptr, p.colidx, p.vals, x2)
    xs = (p.x.astype(np.float64) + x2.astype(np.float64)).astype(np.float32)   # rounded sum: compare with its own widening
    y12, _ = oracle.spmv_csr("f32", p.m, p.n, p.rowptr, p.colidx, p.vals, xs)
    resid = np.abs(y12 - (y1 + y2))
    assert np.all(resid <= 1.3e-7 * (S1 + S2) + 1e-300)     # float32 rounding of x1+x2 only
    y4, _ = oracle.spmv_csr("f32", p.m, p.n, p.rowptr, p.colidx, p.vals, (4 * p.x).astype(np.float32))
    assert np.array_equal(y4, 4 * y1)                        # scaling by a power of two is exact
    # permuting rows permutes y
    perm = rng.permutation(p.m)
    lens = np.diff(p.rowptr)
    rp = np.concatenate(([0], np.cumsum(lens[perm]))).astype(np.int32)
    idx = np.concatenate([np.arange(p.rowptr[r], p.rowptr[r + 1]) for r in perm]) if p.nnz else np.zeros(0, int)
    yp, Sp = oracle.spmv_csr("f32", p.m, p.n, rp, p.colidx[idx].copy(), p.vals[idx].copy(), p.x)
    assert np.array_equal(yp, y1[perm]) and np.array_equal(Sp, S1[perm])


def test_beta_zero_never_reads_y0():
    p = w.from_row_lengths([3, 0, 2], 6, seed=9)
    y0 = np.full(p.m, np.nan, dtype=np.float32)
    y, _ = oracle.spmv_csr("f32", p.m, p.n, p.rowptr, p.colidx, p.vals, p.x, y0, 1.0, 0.0)
    assert np.all(np.isfinite(y))
    y, _ = oracle.spmv_csr("f32", p.m, p.n, p.rowptr, p.colidx, p.vals, p.x, y0, 1.0, 1.0)
    assert np.all(np.isnan(y))


def test_empty_shapes():
    rp = np.zeros(1, dtype=np.int32)
    e = np.zeros(0, dtype=np.int32)
    y, S = oracle.spmv_csr("f32", 0, 4, rp, e, np.zeros(0, np.float32), np.ones(4, np.float32))
    assert y.size == 0 and S.size == 0
    rp = np.zeros(5, dtype=np.int32)
    y0 = np.arange(4, dtype=np.float32)
    y, S = oracle.spmv_csr("f32", 4, 4, rp, e, np.zeros(0, np.float32), np.ones(4, np.float32), y0, 1.0, 2.0)
    assert np.array_equal(y, 2.0 * y0) and not S.any()


def test_rejects_bad_column():
    rp = np.array([0, 1], dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.spmv_csr("f32", 1, 3, rp, np.array([3], np.int32), np.ones(1, np.float32), np.ones(3, np.float32))
