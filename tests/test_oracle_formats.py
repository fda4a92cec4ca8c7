"""Pins of the COO / CSC / ELL oracles (oracle/formats_oracle.cpp): a hand-worked fixture, and the
pinned CSR oracle on the same matrix after scipy's own format conversions (an independent routine)."""
import json

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import workloads as w


@pytest.fixture(scope="module")
def hand(golden_dir):
    return json.loads((golden_dir / "spmv_formats_3x4_handworked.json").read_text())


def test_handworked(hand):
    h = hand
    x, y0 = np.array(h["x"], np.float32), np.array(h["y0"], np.float32)
    a32 = lambda v: np.array(v, np.float32)
    i32 = lambda v: np.array(v, np.int32)
    for alpha, beta, want in ((1.0, 0.0, h["row_dot"]), (h["alpha"], h["beta"], h["y"])):
        y, S = oracle.spmv_coo("f32", 3, 4, i32(h["coo"]["row"]), i32(h["coo"]["col"]), a32(h["coo"]["vals"]), x, y0, alpha, beta)
        assert y.tolist() == want and S.tolist() == h["S"]
        y, S = oracle.spmv_csc("f32", 3, 4, i32(h["csc"]["col_offsets"]), i32(h["csc"]["row"]), a32(h["csc"]["vals"]), x, y0, alpha, beta)
        assert y.tolist() == want and S.tolist() == h["S"]
        y, S = oracle.spmv_ell("f32", 3, 4, h["ell"]["width"], i32(h["ell"]["col_ids"]), a32(h["ell"]["vals"]), x, y0, alpha, beta)
        assert y.tolist() == want and S.tolist() == h["S"]


def problems(dtype):
    return [w.uniform_rows(60, 45, 6, dtype=dtype), w.powerlaw(400, dtype=dtype), w.laplace2d(9, dtype=dtype),
            w.density_random(128, 256, 0.02, dtype=dtype)] + w.tiny_adversarial(dtype=dtype)[:5]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scipy_conversions_reproduce_the_csr_oracle(dtype):
    """The entries keep their values through a conversion; only their order changes.  With values of
    mixed sign the double sums may differ in the last bits between orders, so compare to 1e-12 * S."""
    for p in problems(dtype):
        if p.nnz == 0 or np.any(np.diff(p.colidx)[np.diff(np.repeat(np.arange(p.m), np.diff(p.rowptr))) == 0] <= 0):
            continue  # scipy merges repeated coordinates; those matrices are covered by the workloads' own re-layouts
        y0 = p.y0 if p.y0 is not None else np.zeros(p.m, np.float32)
        y_ref, S_ref = oracle.spmv_csr(dtype, p.m, p.n, p.rowptr, p.colidx, p.vals, p.x, y0, 1.25, -0.5)
        tag = np.arange(1, p.nnz + 1, dtype=np.float64)            # scipy carries entry ids, not values
        A = sp.csr_matrix((tag, p.colidx, p.rowptr), shape=(p.m, p.n))
        coo = A.tocoo()
        ids = coo.data.astype(np.int64) - 1
        y, S = oracle.spmv_coo(dtype, p.m, p.n, coo.row.astype(np.int32), coo.col.astype(np.int32), p.vals[ids].copy(), p.x, y0, 1.25, -0.5)
        assert np.all(np.abs(y - y_ref) <= 1e-12 * (S_ref + 1)) and np.allclose(S, S_ref, rtol=1e-12, atol=0)
        csc = A.tocsc()
        ids = csc.data.astype(np.int64) - 1
        y, S = oracle.spmv_csc(dtype, p.m, p.n, csc.indptr.astype(np.int32), csc.indices.astype(np.int32), p.vals[ids].copy(), p.x, y0, 1.25, -0.5)
        assert np.all(np.abs(y - y_ref) <= 1e-12 * (S_ref + 1)) and np.allclose(S, S_ref, rtol=1e-12, atol=0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_own_relayouts_agree_with_scipy_and_with_the_csr_oracle(dtype):
    for p in problems(dtype) + [w.from_row_lengths([6] * 40, 11, dtype=dtype, allow_dup=True, sort_cols=False)]:
        y0 = p.y0 if p.y0 is not None else np.zeros(p.m, np.float32)
        y_ref, S_ref = oracle.spmv_csr(dtype, p.m, p.n, p.rowptr, p.colidx, p.vals, p.x, y0, p.alpha, p.beta)
        tol = 1e-12 * (S_ref + 1)
        for seed in (None, 3):
            row, col, vals = w.to_coo(p, seed)
            y, S = oracle.spmv_coo(dtype, p.m, p.n, row, col, vals, p.x, y0, p.alpha, p.beta)
            assert np.all(np.abs(y - y_ref) <= tol)
        co, row, vals = w.to_csc(p)
        assert co[0] == 0 and co[-1] == p.nnz and np.all(np.diff(co) >= 0)
        y, S = oracle.spmv_csc(dtype, p.m, p.n, co, row, vals, p.x, y0, p.alpha, p.beta)
        assert np.all(np.abs(y - y_ref) <= tol)
        for extra in (0, 3):
            width, ci, vals = w.to_ell(p, int(np.diff(p.rowptr).max(initial=0)) + extra)
            assert (ci != -1).sum() == p.nnz
            y, S = oracle.spmv_ell(dtype, p.m, p.n, width, ci, vals, p.x, y0, p.alpha, p.beta)
            assert np.array_equal(y, y_ref) and np.array_equal(S, S_ref)     # ELL keeps the CSR order: bit for bit


def test_rejects_indices_out_of_range():
    x = np.ones(4, np.float32)
    with pytest.raises(ValueError):
        oracle.spmv_coo("f32", 3, 4, np.array([3], np.int32), np.array([0], np.int32), np.ones(1, np.float32), x)
    with pytest.raises(ValueError):
        oracle.spmv_csc("f32", 3, 4, np.array([0, 1, 1, 1, 1], np.int32), np.array([-1], np.int32), np.ones(1, np.float32), x)
    with pytest.raises(ValueError):
        oracle.spmv_ell("f32", 1, 4, 2, np.array([0, 4], np.int32), np.ones(2, np.float32), x)
    y, S = oracle.spmv_ell("f32", 1, 4, 2, np.array([-1, -1], np.int32), np.full(2, np.nan, np.float32), x)
    assert y[0] == 0.0 and S[0] == 0.0     # padding values are never read into the sum
