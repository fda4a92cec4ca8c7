"""GPU parity of spmm_csr_run (C <- alpha*A*B + beta*C, paper App. C task 13) against the oracle,
element by element: |C - C_ref| <= tol * sum_e |a_ie b_ek| (plus the rounding of beta*C0 when beta != 0), tol = 1e-5 with
FP32 storage of A and B and 8e-3 with bf16 storage (the bounds stated for the matrix-vector product)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_07169_amd as s
import workloads as w
from gpu_util import DeviceProblem, to_dev

pytestmark = pytest.mark.gpu
TOL = 1e-5
TOLS = {"f32": 1e-5, "bf16": 8e-3}


def log(*a):
    print(*a, flush=True)


def rand(shape, seed):
    return np.random.default_rng(seed).uniform(-1, 1, shape).astype(np.float32)


def rand_b(p, K, seed):
    """A dense B in the storage type of p: float32, or bf16 bit patterns (rounded once, here)."""
    B = rand((p.n, K), seed)
    return w.f32_to_bf16_bits(B) if p.dtype == "bf16" else B


def b_tensor(B):
    return torch.from_numpy(B.view(np.int16) if B.dtype == np.uint16 else B)


def run_spmm(p, B, C0, alpha, beta, lead_pad=0, offset=0, matrix_params=None):
    """Runs the product on the device; B and C live in wider allocations (leading dimension K + lead_pad)
    starting `offset` elements in, so that strided and misaligned layouts are exercised."""
    d = DeviceProblem(p)
    A = d.matrix(matrix_params)
    K = B.shape[1]
    ld = K + lead_pad
    Bbuf = torch.zeros(p.n * ld + offset + 8, dtype=torch.int16 if B.dtype == np.uint16 else torch.float32, device="cuda")
    Cbuf = torch.full((p.m * ld + offset + 8,), 7.0, dtype=torch.float32, device="cuda")
    Bv = Bbuf[offset:offset + p.n * ld].view(p.n, ld)[:, :K]
    Cv = Cbuf[offset:offset + p.m * ld].view(p.m, ld)[:, :K]
    Bv.copy_(b_tensor(B))
    Cv.copy_(torch.from_numpy(C0))
    A.spmm(Bv, Cv, alpha, beta)
    torch.cuda.synchronize()
    out = Cv.cpu().numpy()
    if lead_pad:  # the padding columns of C are not touched
        pad = Cbuf[offset:offset + p.m * ld].view(p.m, ld)[:, K:].cpu().numpy()
        assert np.all(pad == 7.0)
    A.close()
    return out


def check(p, K, alpha=1.0, beta=0.0, seed=0, **kw):
    """Both row orders: rows as they come, and the length-sorted order built at analysis time."""
    B, C0 = rand_b(p, K, seed), rand((p.m, K), seed + 1)
    C_ref, S = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, B, C0, alpha, beta)
    bound = TOLS[p.dtype] * (abs(alpha) * S + (np.abs(np.float64(np.float32(beta)) * C0) if beta != 0 else 0.0))
    for prepare in (0, 1):
        C = run_spmm(p, B, C0, alpha, beta, matrix_params=dict(prepare_spmm=prepare), **kw)
        err = np.abs(C.astype(np.float64) - C_ref)
        bad = np.argwhere(~(err <= bound))
        assert bad.size == 0, (p.name, K, prepare, bad[:3].tolist(), err[tuple(bad[0])], bound[tuple(bad[0])])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("K", [1, 3, 4, 15, 16, 17, 40, 64, 100])
def test_small_shapes_every_k(K, dtype):
    for p in w.tiny_adversarial(dtype=dtype) + [w.uniform_rows(300, 200, 9, dtype=dtype), w.powerlaw(2000, dtype=dtype),
                                                w.laplace2d(20, dtype=dtype)]:
        log("case spmm", p.name, K, dtype)
        check(p, K, alpha=p.alpha, beta=p.beta, seed=K)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("lead_pad,offset", [(0, 0), (4, 0), (3, 0), (0, 1), (5, 3), (0, 4)])
def test_strided_and_misaligned_layouts(lead_pad, offset, dtype):
    p = w.powerlaw(1500, dtype=dtype)
    for K in (16, 33):
        log("case spmm layout", lead_pad, offset, K)
        check(p, K, alpha=-1.5, beta=0.75, seed=3, lead_pad=lead_pad, offset=offset)


def test_more_columns_than_one_lds_block():
    """n > 2048: B is taken in several passes that accumulate into C."""
    for p in (w.uniform_rows(700, 5000, 12), w.powerlaw(3000, n=7001), w.from_row_lengths([0, 5000, 3, 0, 9000], 9000, seed=4),
              w.powerlaw(3000, n=7001, dtype="bf16")):
        for beta in (0.0, 0.5):
            log("case spmm wide", p.name, beta)
            check(p, 24, alpha=2.0, beta=beta, seed=5)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_exact_integer_bit_for_bit(dtype):
    lens = [0, 1, 2, 3, 17, 64, 255, 256, 257, 0, 0, 1000, 5]
    p = w.exact_integer(lens, 1500, alpha=3.0, beta=-2.0, dtype=dtype)
    rng = np.random.default_rng(8)
    B = rng.integers(-3, 4, (p.n, 20)).astype(np.float32)
    if dtype == "bf16":
        B = w.f32_to_bf16_bits(B)               # small integers: exact
    C0 = rng.integers(-5, 6, (p.m, 20)).astype(np.float32)
    C_ref, _ = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, B, C0, p.alpha, p.beta)
    for prepare in (0, 1):
        C = run_spmm(p, B, C0, p.alpha, p.beta, matrix_params=dict(prepare_spmm=prepare))
        assert np.array_equal(C.astype(np.float64), C_ref)


def test_beta_zero_ignores_nan_in_c_and_errors():
    p = w.uniform_rows(100, 80, 6)
    B = rand((p.n, 16), 1)
    C = run_spmm(p, B, np.full((p.m, 16), np.nan, np.float32), 1.0, 0.0)
    C_ref, S = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, B)
    assert np.all(np.abs(C - C_ref) <= TOL * S)
    d = DeviceProblem(p)
    A = d.matrix()
    Bt, Ct = torch.zeros(p.n, 16, device="cuda"), torch.zeros(p.m, 16, device="cuda")
    assert s.spmm_csr_run(A.handle, Bt.data_ptr(), 8, Ct.data_ptr(), 16, 16, 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    assert s.spmm_csr_run(A.handle, Bt.data_ptr(), 16, Ct.data_ptr(), 15, 16, 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    assert s.spmm_csr_run(A.handle, None, 16, Ct.data_ptr(), 16, 16, 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    assert s.spmm_csr_run(A.handle, Bt.data_ptr(), 16, Ct.data_ptr(), 16, -1, 1.0, 0.0) == s.SPMV_ERR_INVALID_ARG
    assert s.spmm_csr_run(A.handle, Bt.data_ptr(), 16, Ct.data_ptr(), 16, 0, 1.0, 0.0) == s.SPMV_OK
    A.close()
    q = w.uniform_rows(100, 80, 6, dtype="bf16")       # a bf16 handle takes a bf16 B: an odd address is refused
    d = DeviceProblem(q)
    A = d.matrix(dict(prepare_spmm=1))
    Bh = torch.zeros(q.n * 16 + 8, dtype=torch.int16, device="cuda")
    assert s.spmm_csr_run(A.handle, Bh.data_ptr() + 1, 16, Ct.data_ptr(), 16, 16, 1.0, 0.0) == s.SPMV_ERR_UNSUPPORTED
    assert s.spmm_csr_run(A.handle, Bh.data_ptr() + 2, 16, Ct.data_ptr(), 16, 16, 1.0, 0.0) == s.SPMV_OK
    torch.cuda.synchronize()
    assert not Ct.cpu().numpy().any()
    A.close()


def test_row_order_and_packed_copy_read_back_match_the_oracle():
    cases = [(w.density_random(1 << 14, 2048, 0.01), 2, 2), (w.powerlaw(5000), 1, 0),
             (w.from_row_lengths([0, 300, 3, 0, 252, 253, 9], 400, seed=4), 1, 0),
             (w.uniform_rows(3000, 5000, 24), 2, 2), (w.uniform_rows(700, 40000, 24), 2, 4),
             (w.from_row_lengths(np.random.default_rng(1).poisson(30, 1000), 100, seed=2, allow_dup=True), 2, 2),
             (w.density_random(1 << 12, 2048, 0.01, dtype="bf16"), 2, 2), (w.uniform_rows(700, 40000, 24, dtype="bf16"), 2, 4)]
    for p, prepared, col_bytes in cases:
        log("case spmm packed", p.name)
        d = DeviceProblem(p)
        A = d.matrix(dict(prepare_spmm=1))
        assert (A.info.spmm_prepared, A.info.spmm_col_bytes) == (prepared, col_bytes)
        got = A.analysis()
        rows = oracle.spmm_row_order(p.rowptr)
        assert np.array_equal(got["spmm_rows"], rows)
        if prepared == 2:
            desc, blocks = oracle.spmm_packed_layout(p.rowptr, rows)
            assert oracle.spmm_packed_choice(p.nnz, blocks) and A.info.spmm_num_blocks == blocks
            assert np.array_equal(got["spmm_desc"], desc)
            # the copy holds binary32 values: bf16 ones widened (exactly, by the generator module's bit shift)
            pcol, pval = oracle.spmm_pack(p.rowptr, p.colidx, p.vals if p.dtype == "f32" else w.bf16_bits_to_f32(p.vals), rows, desc)
            pad = 2048 if p.n <= 2048 else (65535 if col_bytes == 2 else -1)   # what the library writes for "no entry"
            lib_col = got["spmm_col"].astype(np.int64)
            assert np.array_equal(np.where(lib_col == pad, -1, lib_col), pcol) and np.array_equal(got["spmm_val"], pval)
        A.analyze()                                # re-planned without it: the order is dropped
        assert A.info.spmm_prepared == 0 and "spmm_rows" not in A.analysis()
        A.close()


@pytest.mark.parametrize("rows_log2,dtype", [(10, "f32"), (12, "f32"), (14, "f32"), (10, "bf16"), (13, "bf16")])
def test_paper_shapes_full_compare(rows_log2, dtype):
    """Task 13's shapes: cols 2048, K 4096, density 0.01; every element of C."""
    p = w.density_random(1 << rows_log2, 2048, 0.01, dtype=dtype)
    log("case spmm paper shape", p.m, p.nnz, dtype)
    check(p, 4096, seed=rows_log2)


@pytest.mark.parametrize("rows_log2,dtype", [(16, "f32"), (18, "f32"), (16, "bf16")])
def test_paper_shapes_2_16_and_2_18_sampled_rows(rows_log2, dtype):
    """rows = 2^16 (C = 1 GiB) and 2^18 (C = 4 GiB, the task's largest): 300 sampled rows of C against the oracle run on
    just those rows."""
    p = w.density_random(1 << rows_log2, 2048, 0.01, dtype=dtype)
    log("case spmm sampled", p.m, p.nnz, dtype)
    K = 4096
    B = rand_b(p, K, 21)
    d = DeviceProblem(p)
    A = d.matrix(dict(prepare_spmm=1))             # as bench.py times it
    Bt = b_tensor(B).cuda()
    Ct = torch.empty(p.m, K, dtype=torch.float32, device="cuda")
    A.spmm(Bt, Ct)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, p.m - 1], np.random.default_rng(2).integers(0, p.m, 300)]))
    lens = (p.rowptr[rows + 1] - p.rowptr[rows]).astype(np.int64)
    sub_rp = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    take = np.concatenate([np.arange(p.rowptr[r], p.rowptr[r + 1]) for r in rows])
    C_ref, S = oracle.spmm_csr(rows.size, p.n, sub_rp, p.colidx[take].copy(), p.vals[take].copy(), B)
    got = Ct[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - C_ref) <= TOLS[dtype] * S)
    A.close()
    del Ct


def test_packed_copy_follows_values_after_refresh():
    p = w.density_random(1 << 12, 2048, 0.01)
    K = 32
    B = rand((p.n, K), 5)
    d = DeviceProblem(p)
    A = d.matrix(dict(prepare_spmm=1))
    assert A.info.spmm_prepared == 2
    Bt = torch.from_numpy(B).cuda()
    Ct = torch.empty(p.m, K, dtype=torch.float32, device="cuda")
    new_vals = np.random.default_rng(4).permutation(p.vals)
    for vals, refresh in ((p.vals, False), (new_vals, True)):
        d.vals.copy_(to_dev(vals))
        if refresh:
            A.refresh_values()
        A.spmm(Bt, Ct)
        torch.cuda.synchronize()
        C_ref, S = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, vals, B)
        assert np.all(np.abs(Ct.cpu().numpy() - C_ref) <= TOL * S), refresh
    A.close()

