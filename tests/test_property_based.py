"""Randomised cross-checks (hypothesis): the library's host analysis against the oracle's literal
definitions on arbitrary row-length profiles and parameters, and the SpMV / SpMM oracles against a
dense product on arbitrary small matrices.  CPU only."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
import workloads as w
from test_capi_host import compare_with_oracle, rowptr_of

lens_strategy = st.lists(st.one_of(st.integers(0, 12), st.integers(0, 300), st.just(0), st.integers(2000, 9000)),
                         min_size=0, max_size=120)
params_strategy = st.fixed_dictionaries({}, optional={
    "block_nnz": st.integers(1, 8192), "rows_max": st.integers(1, 1024), "items_per_chunk": st.integers(1, 8192)})


@settings(max_examples=120, deadline=None)
@given(lens=lens_strategy, params=params_strategy)
def test_host_analysis_equals_oracle_everywhere(lens, params):
    compare_with_oracle(rowptr_of(lens), 10000, params)


@settings(max_examples=60, deadline=None)
@given(lens=st.lists(st.integers(0, 9), min_size=1, max_size=12), n=st.integers(1, 14), seed=st.integers(0, 10 ** 6),
       alpha=st.sampled_from([1.0, -0.5, 2.0]), beta=st.sampled_from([0.0, 1.0, -1.5]), K=st.integers(1, 5))
def test_oracles_against_dense_products(lens, n, seed, alpha, beta, K):
    p = w.from_row_lengths(lens, n, seed=seed, alpha=alpha, beta=beta, allow_dup=True, sort_cols=False)
    A = np.zeros((p.m, p.n))
    for i in range(p.m):
        for e in range(p.rowptr[i], p.rowptr[i + 1]):
            A[i, p.colidx[e]] += np.float64(p.vals[e])
    y, S = oracle.spmv_problem(p)
    want = alpha * (A @ p.x.astype(np.float64)) + (beta * p.y0.astype(np.float64) if beta != 0 else 0.0)
    assert np.allclose(y, want, rtol=0, atol=1e-12 * (1 + np.abs(A).sum()))
    B = np.random.default_rng(seed).uniform(-1, 1, (p.n, K)).astype(np.float32)
    C, _ = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, B, None, alpha, 0.0)
    assert np.allclose(C, alpha * (A @ B.astype(np.float64)), rtol=0, atol=1e-12 * (1 + np.abs(A).sum()))
    # the other layouts of the same matrix
    row, col, vals = w.to_coo(p, seed)
    y2, _ = oracle.spmv_coo("f32", p.m, p.n, row, col, vals, p.x, p.y0, alpha, beta)
    co, row, vals = w.to_csc(p)
    y3, _ = oracle.spmv_csc("f32", p.m, p.n, co, row, vals, p.x, p.y0, alpha, beta)
    width, ci, vals = w.to_ell(p)
    y4, _ = oracle.spmv_ell("f32", p.m, p.n, width, ci, vals, p.x, p.y0, alpha, beta)
    for other in (y2, y3, y4):
        assert np.allclose(other, want, rtol=0, atol=1e-12 * (1 + np.abs(A).sum()))


@settings(max_examples=60, deadline=None)
@given(lens=st.lists(st.integers(0, 40), min_size=1, max_size=60), n=st.integers(41, 400), seed=st.integers(0, 10 ** 6),
       block_nnz=st.integers(1, 200), rows_max=st.integers(1, 20), ve=st.sampled_from([4, 8]))
def test_x_windows_reconstruct_the_columns(lens, n, seed, block_nnz, rows_max, ve):
    p = w.from_row_lengths(lens, n, seed=seed)
    rb = oracle.row_blocks(p.rowptr, block_nnz, rows_max)
    nv, xv_ptr, xv_start, lidx = oracle.x_windows(p.rowptr, p.colidx, rb, block_nnz, ve)
    for b in range(rb.size - 1):
        k0, k1 = p.rowptr[rb[b]], p.rowptr[rb[b + 1]]
        if k1 - k0 > block_nnz:
            assert nv[b] == 0
            continue
        starts = xv_start[xv_ptr[b]:xv_ptr[b + 1]]
        li = lidx[k0:k1].astype(np.int64)
        assert np.array_equal(starts[li // ve] + li % ve, p.colidx[k0:k1])
        assert np.all(np.diff(starts) > 0) and np.all(starts % ve == 0)
