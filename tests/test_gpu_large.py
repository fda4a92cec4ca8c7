"""Entry counts beyond 2^30: every plan on a matrix of 1.14 * 10^9 stored entries, compared with
the oracle row by row, every row.  The kernels index entries with 32-bit integers; this is the
case that shows an index, or a byte offset formed from one, leaving the 31-bit range."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_07169_amd as s
import workloads as w
from gpu_util import DeviceProblem, assert_close, check_piece_rule, reference

pytestmark = pytest.mark.gpu


def test_more_than_2_to_30_entries_every_plan():
    p = w.clustered_arithmetic()
    assert 2 ** 30 < p.nnz <= s.SPMV_MAX_SIZE and p.nnz == 1_140_850_688
    print("case", p.name, p.nnz, flush=True)
    y_ref, S_ref = reference(p)
    d = DeviceProblem(p)

    # group-aligned, the runs of a block of rows all at different places: AUTO takes the two passes on the 142 M groups
    A = d.matrix()
    print("  analyzed: plan", s.PLAN_NAMES[A.info.plan], flush=True)
    assert s.PLAN_NAMES[A.info.plan] == "twophase" and A.info.tp_group == 8 and A.info.tp_slots >= p.nnz // 8
    y = d.run(A)
    worst = assert_close(p, y, y_ref, S_ref, p.alpha, p.beta, strict=True, what="auto")
    print(f"  two-pass on groups: max |err| / sum|a x| = {worst:.3e}", flush=True)
    assert np.array_equal(d.run(A), y)
    A.close()

    A = d.matrix(dict(plan=s.SPMV_PLAN_WINDOWED))
    assert A.info.plan == s.SPMV_PLAN_WINDOWED and A.info.lidx_grouped == 1
    y = d.run(A)
    worst = assert_close(p, y, y_ref, S_ref, p.alpha, p.beta, strict=True, what="windowed")
    print(f"  windowed: max |err| / sum|a x| = {worst:.3e}", flush=True)
    assert np.array_equal(d.run(A), y)

    # analysis outputs, bit for bit where the oracle's literal definitions finish in seconds
    got = A.analysis()
    rb = oracle.row_blocks(p.rowptr, A.info.block_nnz, A.info.rows_max)
    assert np.array_equal(got["row_blocks"], rb)
    mr, mz = oracle.merge_path(p.rowptr, A.info.items_per_chunk)
    assert np.array_equal(got["mp_row"], mr) and np.array_equal(got["mp_nz"], mz)
    cnt, off, rows = oracle.row_bins(p.rowptr)
    assert np.array_equal(got["bin_count"], cnt) and np.array_equal(got["bin_rows"], rows)
    # x windows: sampled row blocks (first, last, around entry 2^30, random), each against the
    # oracle run on that block alone
    nb = rb.size - 1
    xv_ptr = got["xv_ptr"]
    V = int(A.info.max_x_vectors)
    across = int(np.searchsorted(p.rowptr[rb], 2 ** 30))
    pick = np.unique(np.concatenate([[0, 1, nb - 2, nb - 1], np.arange(across - 3, across + 3),
                                     np.random.default_rng(31).integers(0, nb, 200)]))
    for b in pick:
        nv, _, xs, li = oracle.x_windows(p.rowptr, p.colidx, rb[b:b + 2].copy(), A.info.block_nnz, 8)
        k0, k1 = p.rowptr[rb[b]], p.rowptr[rb[b + 1]]
        assert xv_ptr[b + 1] - xv_ptr[b] == nv[0], b
        assert np.array_equal(got["xv_start"][xv_ptr[b]:xv_ptr[b + 1]], xs), b
        assert np.array_equal(got["lidx"][k0:k1], li[k0:k1]), b
        assert np.array_equal(got["xv_pad"][b * V:b * V + nv[0]], xs) and np.all(got["xv_pad"][b * V + nv[0]:(b + 1) * V] == -1), b
    del got
    A.close()

    for plan in (s.SPMV_PLAN_ADAPTIVE, s.SPMV_PLAN_MERGE, s.SPMV_PLAN_BINNED, s.SPMV_PLAN_VECTOR, s.SPMV_PLAN_SCALAR,
                 s.SPMV_PLAN_COLBLOCK):
        print("  plan", s.PLAN_NAMES[plan], flush=True)
        A = d.matrix(dict(plan=plan))
        assert A.info.plan == plan
        worst = assert_close(p, d.run(A), y_ref, S_ref, p.alpha, p.beta, strict=True, what=s.PLAN_NAMES[plan])
        print(f"    max |err| / sum|a x| = {worst:.3e}", flush=True)
        A.close()


@pytest.mark.parametrize("log2_rows", [22, 23])
def test_two_pass_plan_on_many_scattered_entries(log2_rows):
    """16 entries a row at random columns, 4 M x 4 M (67 M entries: the largest matrix the benchmark line reports for the
    two-pass plan, 256 column blocks x 8704 chunks) and 8 M x 8 M (134 M entries, 8.9 M tiles of 15 entries): the regrouping
    bit for bit, every row against the oracle, same bits on a second run, and values changed in place picked up after a
    refresh."""
    p = w.uniform_rows(1 << log2_rows, 1 << log2_rows, 16, alpha=1.25, beta=-0.5)
    print("case", p.name, p.nnz, flush=True)
    d = DeviceProblem(p)
    A = d.matrix()
    assert A.info.plan == s.SPMV_PLAN_TWOPHASE
    L = oracle.two_phase_layout(p.m, p.n, p.rowptr, p.colidx, piece_groups=A.info.tp_piece_groups)
    check_piece_rule(L, A.info)
    assert (A.info.tp_num_col_blocks, A.info.tp_num_chunks, A.info.tp_slots, A.info.tp_num_pieces) == (L["C"], L["P"], L["S"], L["Q"])
    got = A.analysis()
    for name in ("tp_row", "tp_nz", "tp_piece_c", "tp_piece_g", "tp_chunk_g", "tp_col", "tp_src", "tp_from", "tp_pos"):
        assert np.array_equal(got[name], L[name]), name
    del got, L
    y_ref, S_ref = reference(p)
    y = d.run(A)
    worst = assert_close(p, y, y_ref, S_ref, p.alpha, p.beta, strict=False, what="two-pass")
    print(f"  two-pass: max |err| / sum|a x| = {worst:.3e}", flush=True)
    assert np.array_equal(d.run(A), y)
    new_vals = np.roll(p.vals, 12345)
    d.vals.copy_(torch.from_numpy(new_vals).cuda())
    A.refresh_values()
    q = w.CsrProblem(p.name, p.dtype, p.m, p.n, p.rowptr, p.colidx, new_vals, p.x, p.y0, p.alpha, p.beta)
    y_ref, S_ref = reference(q)
    assert_close(q, d.run(A), y_ref, S_ref, q.alpha, q.beta, what="two-pass after refresh")
    A.close()
