"""spmv_csr_run_static (the entry point for callers that cannot allocate) against spmv_csr_run on a handle with the
MERGE plan: the same kernels on the same merge-path chunks, so the two must agree bit for bit; and against the oracle."""
import numpy as np
import pytest
import torch

import paper_2603_07169_amd as s
import workloads as w
from gpu_util import DTYPE_CODE, DeviceProblem, assert_close, reference

pytestmark = pytest.mark.gpu


def run_static(d, alpha, beta, y_init, stream=None):
    p = d.p
    y = y_init.clone()
    st = s.spmv_csr_run_static(p.m, p.n, p.nnz, d.rowptr.data_ptr(), d.colidx.data_ptr() if p.nnz else None,
                               d.vals.data_ptr() if p.nnz else None, DTYPE_CODE[p.dtype], d.x.data_ptr() if p.n else None,
                               y.data_ptr(), alpha, beta, stream)
    s.check(st, "spmv_csr_run_static")
    torch.cuda.synchronize()
    return y.cpu().numpy()


def both(p, alpha, beta):
    d = DeviceProblem(p)
    y_init = d.y0 if p.y0 is not None else torch.full((p.m,), float("nan"), dtype=torch.float32, device="cuda")
    if beta != 0.0 and p.y0 is None:
        y_init = torch.linspace(-1, 1, p.m, dtype=torch.float32, device="cuda")
    A = d.matrix(dict(plan=s.SPMV_PLAN_MERGE))
    assert A.info.items_per_chunk == 2048
    y_handle = d.run(A, alpha, beta, y_init)
    A.close()
    y_static = run_static(d, alpha, beta, y_init)
    return d, y_init, y_handle, y_static


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_two_calls_in_a_row_the_second_smaller(dtype):
    big = w.powerlaw(300_000, dtype=dtype)        # several hundred chunks, rows cut by chunk boundaries
    small = w.powerlaw(9_000, dtype=dtype)        # fewer chunks than the call before: stale carries must not leak in
    for p, alpha, beta in ((big, 1.0, 0.0), (small, 1.0, 0.0), (small, -0.75, 0.5)):
        print(f"case {p.name} {dtype} m={p.m} nnz={p.nnz} alpha={alpha} beta={beta}", flush=True)
        d, y_init, y_handle, y_static = both(p, alpha, beta)
        assert np.array_equal(y_handle.view(np.uint32), y_static.view(np.uint32)), p.name
        if beta != 0.0 and p.y0 is None:
            p.y0 = y_init.cpu().numpy()
        y_ref, S_ref = reference(p, alpha, beta)
        assert_close(p, y_static, y_ref, S_ref, alpha, beta, what="static")


def test_adversarial_shapes_and_a_long_row():
    for p in w.tiny_adversarial():
        print(f"case {p.name} m={p.m} n={p.n} nnz={p.nnz}", flush=True)
        d, y_init, y_handle, y_static = both(p, p.alpha, p.beta)
        assert np.array_equal(y_handle.view(np.uint32), y_static.view(np.uint32)), p.name
    p = w.exact_integer([3] * 1500 + [200_000] + [5] * 1500 + [0] * 7, 250_000, beta=0.5)
    print(f"case {p.name} m={p.m} nnz={p.nnz}", flush=True)
    d, y_init, y_handle, y_static = both(p, p.alpha, p.beta)
    y_ref, _ = reference(p)
    assert np.array_equal(y_static.astype(np.float64), y_ref)       # integer-valued: exact in any order
    assert np.array_equal(y_handle.view(np.uint32), y_static.view(np.uint32))


def test_on_a_side_stream_and_sizes_refused():
    p = w.laplace2d(200)
    d = DeviceProblem(p)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        y = run_static(d, p.alpha, p.beta, d.y0, side.cuda_stream)
    y_ref, S_ref = reference(p)
    assert_close(p, y, y_ref, S_ref, p.alpha, p.beta, strict=True, what="static, side stream")
    # beyond the fixed array: refused before anything is enqueued (the pointers are never touched)
    st = s.spmv_csr_run_static(1 << 27, 1 << 27, 1 << 27, d.rowptr.data_ptr(), d.colidx.data_ptr(), d.vals.data_ptr(),
                               s.SPMV_F32, d.x.data_ptr(), d.y0.data_ptr(), 1.0, 0.0, None)
    assert st == s.SPMV_ERR_UNSUPPORTED
