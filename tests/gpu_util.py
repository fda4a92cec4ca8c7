"""Helpers of the GPU parity tests: move a workloads.CsrProblem to the device with torch
(memory and streams only), run it through the C ABI, and compare with the oracle."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2603_07169_amd as s

TOL = {"f32": 1e-5, "bf16": 8e-3}
DTYPE_CODE = {"f32": s.SPMV_F32, "bf16": s.SPMV_BF16}
ALL_PLANS = [s.SPMV_PLAN_SCALAR, s.SPMV_PLAN_VECTOR, s.SPMV_PLAN_BINNED, s.SPMV_PLAN_ADAPTIVE, s.SPMV_PLAN_MERGE,
             s.SPMV_PLAN_WINDOWED, s.SPMV_PLAN_COLBLOCK, s.SPMV_PLAN_TWOPHASE, s.SPMV_PLAN_SELL]


def plan_params(plan):
    """Parameters that force `plan`.  A forced WINDOWED plan needs every row block to touch at
    most 1024 x vectors; blocks of at most 1024 entries guarantee that for any matrix."""
    if plan == s.SPMV_PLAN_WINDOWED:
        return dict(plan=plan, block_nnz=1024, rows_max=64)
    return dict(plan=plan)


def expected_auto_plan(p, info):
    """The plan AUTO must arrive at, from the oracle's rules."""
    st = oracle.row_stats(p.rowptr)
    plan = oracle.plan(p.m, p.nnz, st["max_len"], info.block_nnz)
    if plan in (s.SPMV_PLAN_ADAPTIVE, s.SPMV_PLAN_MERGE) and p.nnz >= 3 << 24:     # fewer than 3 * 2^21 groups: the rule says no anyway
        rb = oracle.row_blocks(p.rowptr, info.block_nnz, info.rows_max)
        nv, _, _, _ = oracle.x_windows(p.rowptr, p.colidx, rb, info.block_nnz, 8 if p.dtype == "bf16" else 4)
        vectors, entries = oracle.scatter_counts(p.rowptr, rb, info.block_nnz, nv)
        if oracle.grouped_two_phase_choice(p.m, p.n, p.nnz, p.dtype, plan, oracle.csr_groups(p.m, p.rowptr, p.colidx), vectors, entries):
            return s.SPMV_PLAN_TWOPHASE                                            # on groups of eight: looked at before the windows
    if plan == s.SPMV_PLAN_ADAPTIVE:
        rb = oracle.row_blocks(p.rowptr, info.block_nnz, info.rows_max)
        nv, _, _, _ = oracle.x_windows(p.rowptr, p.colidx, rb, info.block_nnz, 8 if p.dtype == "bf16" else 4)
        if oracle.window_choice(nv, p.nnz):
            plan = s.SPMV_PLAN_WINDOWED
    if plan in (s.SPMV_PLAN_ADAPTIVE, s.SPMV_PLAN_MERGE) and p.nnz >= 1 << 22:     # below that many entries both rules say no anyway
        rb = oracle.row_blocks(p.rowptr, info.block_nnz, info.rows_max)
        nv, _, _, _ = oracle.x_windows(p.rowptr, p.colidx, rb, info.block_nnz, 8 if p.dtype == "bf16" else 4)
        vectors, entries = oracle.scatter_counts(p.rowptr, rb, info.block_nnz, nv)
        if oracle.two_phase_choice(p.m, p.n, p.nnz, p.dtype, plan, vectors, entries):
            plan = s.SPMV_PLAN_TWOPHASE
        elif oracle.column_block_choice(p.n, p.nnz, p.dtype, plan, vectors, entries):
            plan = s.SPMV_PLAN_COLBLOCK
    return plan


def check_piece_rule(L, info):
    """The size of the multiply pass's pieces that the handle reports is the one the oracle's rule gives for the device's
    count of resident workgroups; L = the oracle's layout made with that size."""
    groups = np.bincount(L["tp_piece_c"], weights=np.diff(L["tp_piece_g"]), minlength=L["C"]).astype(np.int64)
    assert info.tp_resident > 0 and info.tp_piece_groups == oracle.two_phase_piece_groups(groups, info.tp_resident)


def to_dev(a: np.ndarray, offset_elems: int = 0) -> torch.Tensor:
    """numpy -> cuda tensor with the same bits (uint16 travels as int16).  offset_elems > 0
    places the data that many elements into a larger allocation (a misaligned view)."""
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    t = torch.from_numpy(np.ascontiguousarray(a))
    if offset_elems:
        buf = torch.empty(t.numel() + offset_elems, dtype=t.dtype, device="cuda")
        view = buf[offset_elems:]
        view.copy_(t)
        return view
    return t.cuda()


class DeviceProblem:
    def __init__(self, p, offset_elems=0):
        self.p = p
        self.rowptr = to_dev(p.rowptr)
        self.colidx = to_dev(p.colidx, offset_elems)
        self.vals = to_dev(p.vals, offset_elems)
        self.x = to_dev(p.x, offset_elems)
        self.y0 = to_dev(p.y0) if p.y0 is not None else torch.zeros(p.m, dtype=torch.float32, device="cuda")

    def matrix(self, params=None) -> s.CsrMatrix:
        p = self.p
        return s.CsrMatrix(p.m, p.n, self.rowptr, self.colidx, self.vals, DTYPE_CODE[p.dtype], params)

    def run(self, A, alpha=None, beta=None, y_init=None, stream=None) -> np.ndarray:
        p = self.p
        alpha = p.alpha if alpha is None else alpha
        beta = p.beta if beta is None else beta
        y = (self.y0 if y_init is None else y_init).clone()
        A.run(self.x, y, alpha, beta, stream)
        torch.cuda.synchronize()
        return y.cpu().numpy()


def reference(p, alpha=None, beta=None):
    alpha = p.alpha if alpha is None else alpha
    beta = p.beta if beta is None else beta
    y0 = p.y0 if p.y0 is not None else np.zeros(p.m, dtype=np.float32)
    return oracle.spmv_csr(p.dtype, p.m, p.n, p.rowptr, p.colidx, p.vals, p.x, y0, alpha, beta)


def assert_close(p, y, y_ref, S_ref, alpha, beta, strict=False, what=""):
    """|y - y_ref| <= tol * sum_j |a_ij x_j| per row (strict: exactly that bound).  Otherwise the
    bound also carries |alpha| and the float32 rounding of beta*y0, which the stated bound
    leaves out (it is zero for empty rows)."""
    tol = TOL[p.dtype]
    err = np.abs(y.astype(np.float64) - y_ref)
    if strict:
        bound = tol * S_ref
    else:
        y0 = p.y0 if (p.y0 is not None and beta != 0.0) else np.zeros(p.m, dtype=np.float32)
        bound = tol * (abs(alpha) * S_ref + np.abs(np.float64(np.float32(beta)) * y0))
    bad = np.flatnonzero(~(err <= bound))
    if bad.size:
        i = int(bad[0])
        raise AssertionError(f"{what} {p.name}: {bad.size} rows off; first row {i}: y={y[i]!r} ref={y_ref[i]!r} "
                             f"err={err[i]:.3e} bound={bound[i]:.3e} len={p.rowptr[i+1]-p.rowptr[i]}")
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(S_ref > 0, err / S_ref, 0.0)
    return float(ratio.max(initial=0.0))


def check_problem(p, params=None, strict=False, offset_elems=0, what=""):
    d = DeviceProblem(p, offset_elems)
    A = d.matrix(params)
    y = d.run(A)
    y_ref, S_ref = reference(p)
    r = assert_close(p, y, y_ref, S_ref, p.alpha, p.beta, strict, what)
    A.close()
    return r


def unpack_run_desc(words):
    """The packed runs of the row patterns (eight words per block, see include/spmv_mi355.h) as the oracle's arrays:
    n_runs[nb] and run_rows / run_len / run_base / run_stride [nb, 4]."""
    w8 = words.reshape(-1, 8).astype(np.int64) & 0xFFFFFFFF
    halves = lambda lo, hi: np.stack([w8[:, lo] & 0xFFFF, w8[:, lo] >> 16, w8[:, hi] & 0xFFFF, w8[:, hi] >> 16], axis=1)
    stride = halves(5, 6)
    stride = np.where(stride >= 1 << 15, stride - (1 << 16), stride)
    length = np.stack([(w8[:, 2] >> (8 * r)) & 0xFF for r in range(4)], axis=1)
    return dict(n_runs=w8[:, 7], run_rows=halves(0, 1), run_len=length, run_base=halves(3, 4), run_stride=stride)


def check_patterns_equal_oracle(p, A, got, lidx, grouped):
    """The row patterns the library kept (or its decision to keep none) against the oracle's, bit for bit."""
    rb = got["row_blocks"]
    nb = rb.size - 1
    want = oracle.row_patterns(p.rowptr, rb, lidx, A.info.block_nnz)
    patterned = (not grouped) and oracle.pattern_choice(p.nnz, want["covered"])
    assert A.info.lidx_patterned == int(patterned), (A.info.lidx_patterned, want["covered"], p.nnz)
    if not patterned:
        assert A.info.pat_cap == 0 and A.info.pat_entries == 0
        return want
    sizes = np.diff(want["pat_ptr"])
    cap = max(8, -(-int(sizes.max()) // 8) * 8)
    assert (A.info.pat_cap, A.info.pat_entries) == (cap, want["covered"])
    have = unpack_run_desc(got["run_desc"])
    for name in ("n_runs", "run_rows", "run_len", "run_base", "run_stride"):
        assert np.array_equal(have[name], want[name]), name
    pad = np.zeros((nb, cap), np.uint16)
    for b in range(nb):
        pad[b, :sizes[b]] = want["pat"][want["pat_ptr"][b]:want["pat_ptr"][b + 1]]
    assert np.array_equal(got["pat_pad"].reshape(nb, cap), pad)
    return want
