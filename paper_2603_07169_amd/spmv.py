"""ctypes binding of libspmv_mi355.so: same names and argument lists as include/spmv_mi355.h.

Marshalling only.  Device arrays are passed as raw addresses (e.g. torch.Tensor.data_ptr()),
streams as hipStream_t handles (torch.cuda.current_stream().cuda_stream).  There is no
fallback: if the library is not built, importing the symbols raises.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path

import numpy as np

from . import build as _build

SPMV_F32, SPMV_BF16 = 0, 1
SPMV_OK = 0
(SPMV_ERR_INVALID_ARG, SPMV_ERR_BAD_STRUCTURE, SPMV_ERR_UNSUPPORTED, SPMV_ERR_NOT_ANALYZED, SPMV_ERR_ALLOC,
 SPMV_ERR_HIP, SPMV_ERR_BUSY) = range(1, 8)
(SPMV_PLAN_AUTO, SPMV_PLAN_SCALAR, SPMV_PLAN_VECTOR, SPMV_PLAN_BINNED, SPMV_PLAN_ADAPTIVE, SPMV_PLAN_MERGE,
 SPMV_PLAN_WINDOWED, SPMV_PLAN_COLBLOCK, SPMV_PLAN_TWOPHASE, SPMV_PLAN_SELL) = range(10)
PLAN_NAMES = {0: "auto", 1: "scalar", 2: "vector", 3: "binned", 4: "adaptive", 5: "merge", 6: "windowed", 7: "colblock",
              8: "twophase", 9: "sell"}
SPMV_SELL_HEIGHT = 64
SPMV_TP_SNAP = 512
SPMV_NUM_BINS = 33
SPMV_MAX_X_VECTORS = 1024
SPMV_MAX_SIZE = 2 ** 31 - 2 ** 22
SPMV_STATIC_MAX_ITEMS = 2 ** 28 - 2048

EXPORTS = [
    "spmv_csr_create", "spmv_csr_analyze", "spmv_csr_run", "spmv_csr_refresh_values", "spmm_csr_run", "spmv_coo_run", "spmv_csc_run", "spmv_ell_run", "spmv_csr_run_static", "spmv_destroy", "spmv_csr_get_analysis_info",
    "spmv_csr_get_analysis", "spmv_analyze_host", "spmv_selftest_reduce", "spmv_csr_main_kernel_name",
    "spmv_status_string", "spmv_last_hip_error",
]


class spmv_analyze_params_t(C.Structure):
    _fields_ = [("plan", C.c_int32), ("block_nnz", C.c_int32), ("rows_max", C.c_int32),
                ("items_per_chunk", C.c_int32), ("vector_lanes", C.c_int32), ("skip_validation", C.c_int32),
                ("prepare_spmm", C.c_int32), ("reserved", C.c_int32)]


class spmv_analysis_info_t(C.Structure):
    _fields_ = [("m", C.c_int64), ("n", C.c_int64), ("nnz", C.c_int64), ("min_len", C.c_int64),
                ("max_len", C.c_int64), ("n_empty", C.c_int64), ("num_row_blocks", C.c_int64),
                ("num_chunks", C.c_int64), ("num_x_vectors", C.c_int64), ("plan", C.c_int32),
                ("vector_lanes", C.c_int32), ("block_nnz", C.c_int32), ("rows_max", C.c_int32),
                ("items_per_chunk", C.c_int32), ("max_x_vectors", C.c_int32), ("num_col_blocks", C.c_int32),
                ("col_block_width", C.c_int32), ("spmm_prepared", C.c_int32), ("spmm_col_bytes", C.c_int32),
                ("spmm_num_blocks", C.c_int64), ("tp_slots", C.c_int64), ("tp_col_shift", C.c_int32),
                ("tp_items", C.c_int32), ("tp_num_col_blocks", C.c_int32), ("tp_num_chunks", C.c_int32),
                ("tp_num_pieces", C.c_int32), ("lidx_grouped", C.c_int32), ("lidx_patterned", C.c_int32),
                ("pat_cap", C.c_int32), ("pat_entries", C.c_int64), ("sell_slots", C.c_int64), ("sell_num_slices", C.c_int32),
                ("tp_group", C.c_int32), ("tp_piece_groups", C.c_int32), ("tp_resident", C.c_int32)]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_ if k != "reserved"}


class spmv_analysis_host_t(C.Structure):
    _fields_ = [("bin_count", C.c_void_p), ("bin_offset", C.c_void_p), ("bin_rows", C.c_void_p),
                ("row_blocks", C.c_void_p), ("mp_row", C.c_void_p), ("mp_nz", C.c_void_p),
                ("xv_ptr", C.c_void_p), ("xv_start", C.c_void_p), ("xv_pad", C.c_void_p), ("lidx", C.c_void_p),
                ("run_desc", C.c_void_p), ("pat_pad", C.c_void_p),
                ("cb_ptr", C.c_void_p), ("cb_row", C.c_void_p), ("cb_col", C.c_void_p), ("cb_src", C.c_void_p),
                ("tp_row", C.c_void_p), ("tp_nz", C.c_void_p), ("tp_piece_c", C.c_void_p), ("tp_piece_g", C.c_void_p),
                ("tp_chunk_g", C.c_void_p), ("tp_col", C.c_void_p), ("tp_src", C.c_void_p), ("tp_from", C.c_void_p),
                ("tp_pos", C.c_void_p),
                ("spmm_rows", C.c_void_p), ("spmm_desc", C.c_void_p), ("spmm_col", C.c_void_p), ("spmm_val", C.c_void_p),
                ("sell_ptr", C.c_void_p), ("sell_col", C.c_void_p), ("sell_src", C.c_void_p)]


class SpmvError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {spmv_status_string(status)} (status {int(status)}, hip error {spmv_last_hip_error()})")


_lib = None


def library_path() -> Path:
    return _build.LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not _build.LIB_PATH.exists():
        _build.build()
    lib = C.CDLL(str(_build.LIB_PATH))
    vp, i64, i32, f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_float
    lib.spmv_csr_create.argtypes = [C.POINTER(vp), i64, i64, i64, vp, vp, vp, C.c_int]
    lib.spmv_csr_analyze.argtypes = [vp, C.POINTER(spmv_analyze_params_t)]
    lib.spmv_csr_run.argtypes = [vp, vp, vp, f32, f32, vp]
    lib.spmm_csr_run.argtypes = [vp, vp, i64, vp, i64, i64, f32, f32, vp]
    lib.spmm_csr_run.restype = C.c_int
    lib.spmv_coo_run.argtypes = [i64, i64, i64, vp, vp, vp, C.c_int, vp, vp, f32, f32, vp]
    lib.spmv_csc_run.argtypes = [i64, i64, i64, vp, vp, vp, C.c_int, vp, vp, f32, f32, vp]
    lib.spmv_ell_run.argtypes = [i64, i64, i64, vp, vp, C.c_int, vp, vp, f32, f32, vp]
    lib.spmv_csr_run_static.argtypes = [i64, i64, i64, vp, vp, vp, C.c_int, vp, vp, f32, f32, vp]
    for name in ("spmv_coo_run", "spmv_csc_run", "spmv_ell_run", "spmv_csr_run_static"):
        getattr(lib, name).restype = C.c_int
    lib.spmv_destroy.argtypes = [vp]
    lib.spmv_csr_refresh_values.argtypes = [vp, vp]
    lib.spmv_csr_get_analysis_info.argtypes = [vp, C.POINTER(spmv_analysis_info_t)]
    lib.spmv_csr_get_analysis.argtypes = [vp, C.POINTER(spmv_analysis_host_t)]
    lib.spmv_analyze_host.argtypes = [i64, i64, i64, vp, C.POINTER(spmv_analyze_params_t),
                                      C.POINTER(spmv_analysis_info_t), C.POINTER(spmv_analysis_host_t)]
    lib.spmv_selftest_reduce.argtypes = [vp, vp, vp]
    for name in ("spmv_csr_create", "spmv_csr_analyze", "spmv_csr_run", "spmv_csr_refresh_values", "spmv_destroy", "spmv_csr_get_analysis_info",
                 "spmv_csr_get_analysis", "spmv_analyze_host", "spmv_selftest_reduce"):
        getattr(lib, name).restype = C.c_int
    lib.spmv_csr_main_kernel_name.argtypes = [vp]
    lib.spmv_csr_main_kernel_name.restype = C.c_char_p
    lib.spmv_status_string.argtypes = [C.c_int]
    lib.spmv_status_string.restype = C.c_char_p
    lib.spmv_last_hip_error.argtypes = []
    lib.spmv_last_hip_error.restype = C.c_int
    _lib = lib
    return lib


def _params(params):
    if params is None:
        return None
    if isinstance(params, spmv_analyze_params_t):
        return C.byref(params)
    p = spmv_analyze_params_t()
    for k, v in dict(params).items():
        setattr(p, k, int(v))
    return C.byref(p)


# ------------------------------------------------------------------ the C entry points, one to one
def spmv_status_string(status) -> str:
    return _load().spmv_status_string(int(status)).decode()


def spmv_last_hip_error() -> int:
    return int(_load().spmv_last_hip_error())


def spmv_csr_create(m, n, nnz, rowptr, colidx, vals, dtype):
    """rowptr / colidx / vals: device addresses (int).  Returns (status, handle)."""
    h = C.c_void_p()
    st = _load().spmv_csr_create(C.byref(h), m, n, nnz, rowptr, colidx, vals, dtype)
    return st, h


def spmv_csr_analyze(handle, params=None):
    return _load().spmv_csr_analyze(handle, _params(params))


def spmv_csr_run(handle, x, y, alpha, beta, stream=None):
    return _load().spmv_csr_run(handle, x, y, alpha, beta, stream)


def spmm_csr_run(handle, B, ldb, C_, ldc, K, alpha, beta, stream=None):
    """B, C_: device addresses of row-major float arrays with leading dimensions ldb, ldc."""
    return _load().spmm_csr_run(handle, B, ldb, C_, ldc, K, alpha, beta, stream)


def spmv_coo_run(m, n, nnz, row_indices, col_indices, vals, dtype, x, y, alpha, beta, stream=None):
    return _load().spmv_coo_run(m, n, nnz, row_indices, col_indices, vals, dtype, x, y, alpha, beta, stream)


def spmv_csc_run(m, n, nnz, col_offsets, row_indices, vals, dtype, x, y, alpha, beta, stream=None):
    return _load().spmv_csc_run(m, n, nnz, col_offsets, row_indices, vals, dtype, x, y, alpha, beta, stream)


def spmv_ell_run(m, n, width, col_ids, vals, dtype, x, y, alpha, beta, stream=None):
    return _load().spmv_ell_run(m, n, width, col_ids, vals, dtype, x, y, alpha, beta, stream)


def spmv_csr_run_static(m, n, nnz, rowptr, colidx, vals, dtype, x, y, alpha, beta, stream=None):
    return _load().spmv_csr_run_static(m, n, nnz, rowptr, colidx, vals, dtype, x, y, alpha, beta, stream)


def spmv_csr_refresh_values(handle, stream=None):
    return _load().spmv_csr_refresh_values(handle, stream)


def spmv_destroy(handle):
    return _load().spmv_destroy(handle)


def spmv_csr_get_analysis_info(handle):
    info = spmv_analysis_info_t()
    st = _load().spmv_csr_get_analysis_info(handle, C.byref(info))
    return st, info


def _host_buffers(info):
    bufs = {
        "bin_count": np.zeros(SPMV_NUM_BINS, np.int32), "bin_offset": np.zeros(SPMV_NUM_BINS + 1, np.int32),
        "bin_rows": np.zeros(info.m, np.int32), "row_blocks": np.zeros(info.num_row_blocks + 1, np.int32),
        "mp_row": np.zeros(info.num_chunks + 1, np.int32), "mp_nz": np.zeros(info.num_chunks + 1, np.int32),
    }
    if info.plan == SPMV_PLAN_WINDOWED:
        bufs.update(xv_ptr=np.zeros(info.num_row_blocks + 1, np.int32), xv_start=np.zeros(info.num_x_vectors, np.int32),
                    xv_pad=np.zeros(info.num_row_blocks * max(1, info.max_x_vectors), np.int32),
                    lidx=np.zeros(info.nnz, np.uint16))
        if info.lidx_patterned:
            bufs.update(run_desc=np.zeros(8 * info.num_row_blocks, np.int32),
                        pat_pad=np.zeros(info.num_row_blocks * info.pat_cap, np.uint16))
    if info.plan == SPMV_PLAN_COLBLOCK:
        bufs.update(cb_ptr=np.zeros(info.num_col_blocks + 1, np.int32), cb_row=np.zeros(info.nnz, np.int32),
                    cb_col=np.zeros(info.nnz, np.int32), cb_src=np.zeros(info.nnz, np.int32))
    if info.plan == SPMV_PLAN_TWOPHASE:
        bufs.update(tp_row=np.zeros(info.tp_num_chunks + 1, np.int32), tp_nz=np.zeros(info.tp_num_chunks + 1, np.int32),
                    tp_piece_c=np.zeros(info.tp_num_pieces, np.int32), tp_piece_g=np.zeros(info.tp_num_pieces + 1, np.int32),
                    tp_chunk_g=np.zeros(info.tp_num_chunks + 1, np.int32), tp_col=np.zeros(info.tp_slots, np.uint16),
                    tp_src=np.zeros(info.tp_slots, np.int32), tp_from=np.zeros(info.tp_slots // 4, np.int32),
                    tp_pos=np.zeros(info.tp_slots, np.uint16))
    if info.plan == SPMV_PLAN_SELL:
        bufs.update(sell_ptr=np.zeros(info.sell_num_slices + 1, np.int32), sell_col=np.zeros(info.sell_slots, np.int32),
                    sell_src=np.zeros(info.sell_slots, np.int32))
    if info.spmm_prepared:
        bufs.update(spmm_rows=np.zeros(info.m, np.int32))
    if info.spmm_prepared == 2:
        slots = info.spmm_num_blocks * 256
        bufs.update(spmm_desc=np.zeros(2 * ((info.m + 15) // 16) + 2, np.int32),
                    spmm_col=np.zeros(slots, np.uint16 if info.spmm_col_bytes == 2 else np.int32),
                    spmm_val=np.zeros(slots, np.float32))
    out = spmv_analysis_host_t(**{k: v.ctypes.data for k, v in bufs.items()})
    return bufs, out


def spmv_csr_get_analysis(handle):
    """Returns (status, dict of numpy arrays)."""
    st, info = spmv_csr_get_analysis_info(handle)
    if st != SPMV_OK:
        return st, None
    bufs, out = _host_buffers(info)
    st = _load().spmv_csr_get_analysis(handle, C.byref(out))
    return st, bufs


def spmv_analyze_host(m, n, nnz, rowptr_host: np.ndarray, params=None):
    """Host-only analysis of a numpy rowptr.  Returns (status, info, dict of numpy arrays)."""
    assert rowptr_host.dtype == np.int32 and rowptr_host.flags.c_contiguous and rowptr_host.size == m + 1
    info = spmv_analysis_info_t()
    lib = _load()
    st = lib.spmv_analyze_host(m, n, nnz, rowptr_host.ctypes.data, _params(params), C.byref(info), None)
    if st != SPMV_OK:
        return st, None, None
    bufs, out = _host_buffers(info)
    st = lib.spmv_analyze_host(m, n, nnz, rowptr_host.ctypes.data, _params(params), C.byref(info), C.byref(out))
    return st, info, bufs


def spmv_selftest_reduce(in_dev, out_dev, stream=None):
    return _load().spmv_selftest_reduce(in_dev, out_dev, stream)


def spmv_csr_main_kernel_name(handle) -> str:
    return _load().spmv_csr_main_kernel_name(handle).decode()


def check(status, where="spmv"):
    if status != SPMV_OK:
        raise SpmvError(status, where)


# ------------------------------------------------------------------ convenience wrapper (still marshalling only)
class CsrMatrix:
    """Owns a handle; keeps the torch tensors it borrows alive."""

    def __init__(self, m, n, rowptr_t, colidx_t, vals_t, dtype, params=None):
        self._keep = (rowptr_t, colidx_t, vals_t)
        nnz = int(colidx_t.numel())
        st, self.handle = spmv_csr_create(m, n, nnz, rowptr_t.data_ptr(), colidx_t.data_ptr() if nnz else None,
                                          vals_t.data_ptr() if nnz else None, dtype)
        check(st, "spmv_csr_create")
        self.m, self.n, self.nnz, self.dtype = m, n, nnz, dtype
        self.analyze(params)

    def analyze(self, params=None):
        check(spmv_csr_analyze(self.handle, params), "spmv_csr_analyze")
        st, info = spmv_csr_get_analysis_info(self.handle)
        check(st, "spmv_csr_get_analysis_info")
        self.info = info
        return info

    def run(self, x_t, y_t, alpha=1.0, beta=0.0, stream=None):
        check(spmv_csr_run(self.handle, x_t.data_ptr() if x_t is not None else None, y_t.data_ptr(), alpha, beta,
                           stream), "spmv_csr_run")

    def refresh_values(self, stream=None):
        check(spmv_csr_refresh_values(self.handle, stream), "spmv_csr_refresh_values")

    def spmm(self, B_t, C_t, alpha=1.0, beta=0.0, stream=None):
        """C_t <- alpha*A*B_t + beta*C_t for 2-D row-major torch tensors (column slices allowed)."""
        assert B_t.stride(1) == 1 and C_t.stride(1) == 1 and B_t.shape[1] == C_t.shape[1]
        check(spmm_csr_run(self.handle, B_t.data_ptr(), B_t.stride(0), C_t.data_ptr(), C_t.stride(0), B_t.shape[1],
                           alpha, beta, stream), "spmm_csr_run")

    def analysis(self):
        st, bufs = spmv_csr_get_analysis(self.handle)
        check(st, "spmv_csr_get_analysis")
        return bufs

    def close(self):
        if getattr(self, "handle", None):
            spmv_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
