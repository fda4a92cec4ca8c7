"""ctypes access to the CPU oracle (oracle/*.cpp).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library and its Python binding never do.  The wrappers below only
marshal numpy arrays; all arithmetic is in the C++ files.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
# SPMV_ORACLE_LIB: load that library instead (the mutation check of the pins builds deliberately
# wrong copies of the sources below into libraries of their own and points the pin tests at them).
LIB_PATH = Path(os.environ["SPMV_ORACLE_LIB"]) if os.environ.get("SPMV_ORACLE_LIB") else _HERE / "liboracle.so"
SOURCES = [_HERE / "spmv_oracle.cpp", _HERE / "analysis_oracle.cpp", _HERE / "spmm_oracle.cpp", _HERE / "formats_oracle.cpp"]
_lib = None

NUM_BINS = 33
PLAN_NAMES = {1: "scalar", 2: "vector", 3: "binned", 4: "adaptive", 5: "merge", 6: "windowed", 7: "colblock", 8: "twophase"}
TP_SHIFT, TP_ITEMS, TP_PIECE_GROUPS = 14, 8192, 8192
TP_SNAP = 512            # rows of at most this many entries are never cut by a chunk of the two-pass plan
TP_PIECE_CAP, TP_PIECE_FLOOR, TP_WAVES = 16384, 2048, 2   # the library's rule for the piece size
MAX_X_VECTORS = 1024
MAX_PATTERN_RUNS, MAX_PATTERN_LEN = 4, 64
SELL_HEIGHT = 64
TP_GROUP = 8                       # entries per group of the two-pass plan on groups
TP_GROUP_SHIFT = {"bf16": 12, "f32": 11}   # log2 of the groups' columns per block: 64 KB of x either way


def build(force: bool = True) -> Path:
    """Compile the oracle with the host compiler (no HIP involved)."""
    if not force and LIB_PATH.exists() and all(LIB_PATH.stat().st_mtime >= s.stat().st_mtime for s in SOURCES):
        return LIB_PATH
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra", "-ffp-contract=off",
           "-o", str(LIB_PATH)] + [str(s) for s in SOURCES]
    subprocess.run(cmd, check=True)
    global _lib
    _lib = None
    return LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            build()
        _lib = C.CDLL(str(LIB_PATH))
        i64, i32, f32, vp = C.c_int64, C.c_int32, C.c_float, C.c_void_p
        _lib.oracle_spmv_csr_f32.argtypes = [i64, i64, vp, vp, vp, vp, vp, f32, f32, vp, vp]
        _lib.oracle_spmv_csr_f32.restype = C.c_int
        _lib.oracle_spmv_csr_bf16.argtypes = [i64, i64, vp, vp, vp, vp, vp, f32, f32, vp, vp]
        _lib.oracle_spmv_csr_bf16.restype = C.c_int
        _lib.oracle_spmm_csr_f32.argtypes = [i64, i64, i64, vp, vp, vp, vp, i64, vp, i64, f32, f32, vp, vp]
        _lib.oracle_spmm_csr_f32.restype = C.c_int
        _lib.oracle_spmm_csr_bf16.argtypes = [i64, i64, i64, vp, vp, vp, vp, i64, vp, i64, f32, f32, vp, vp]
        _lib.oracle_spmm_csr_bf16.restype = C.c_int
        _lib.oracle_spmm_row_order.argtypes = [i64, vp, i64, vp]
        _lib.oracle_spmm_row_order.restype = None
        _lib.oracle_spmm_packed_layout.argtypes = [i64, vp, vp, vp]
        _lib.oracle_spmm_packed_layout.restype = i64
        _lib.oracle_spmm_pack.argtypes = [i64, vp, vp, vp, vp, vp, vp, vp]
        _lib.oracle_spmm_pack.restype = None
        _lib.oracle_spmm_packed_choice.argtypes = [i64, i64]
        _lib.oracle_spmm_packed_choice.restype = C.c_int
        _lib.oracle_spmv_coo.argtypes = [i64, i64, i64, vp, vp, vp, C.c_int, vp, vp, f32, f32, vp, vp]
        _lib.oracle_spmv_csc.argtypes = [i64, i64, vp, vp, vp, C.c_int, vp, vp, f32, f32, vp, vp]
        _lib.oracle_spmv_ell.argtypes = [i64, i64, i64, vp, vp, C.c_int, vp, vp, f32, f32, vp, vp]
        for fn in (_lib.oracle_spmv_coo, _lib.oracle_spmv_csc, _lib.oracle_spmv_ell):
            fn.restype = C.c_int
        _lib.oracle_row_stats.argtypes = [i64, vp, vp]
        _lib.oracle_row_stats.restype = None
        _lib.oracle_row_bins.argtypes = [i64, vp, vp, vp, vp]
        _lib.oracle_row_bins.restype = None
        _lib.oracle_row_blocks.argtypes = [i64, vp, i32, i32, vp]
        _lib.oracle_row_blocks.restype = i64
        _lib.oracle_merge_path.argtypes = [i64, i64, vp, i32, vp, vp]
        _lib.oracle_merge_path.restype = i64
        _lib.oracle_tile_shape.argtypes = [i64, i64, vp, vp]
        _lib.oracle_tile_shape.restype = None
        _lib.oracle_plan.argtypes = [i64, i64, i64, i32]
        _lib.oracle_plan.restype = i32
        _lib.oracle_vector_lanes.argtypes = [i64, i64]
        _lib.oracle_vector_lanes.restype = i32
        _lib.oracle_x_windows.argtypes = [i64, vp, vp, vp, i32, i32, vp, vp, vp]
        _lib.oracle_x_windows.restype = i64
        _lib.oracle_window_choice.argtypes = [i64, vp, i64, i32]
        _lib.oracle_window_choice.restype = i32
        _lib.oracle_lidx_grouped.argtypes = [i64, vp, i64, vp, vp]
        _lib.oracle_lidx_grouped.restype = i32
        _lib.oracle_row_patterns.argtypes = [i64, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        _lib.oracle_row_patterns.restype = i64
        _lib.oracle_pattern_choice.argtypes = [i64, i64]
        _lib.oracle_pattern_choice.restype = i32
        _lib.oracle_column_blocks.argtypes = [i64, i64, vp, vp, i64, vp, vp, vp, vp]
        _lib.oracle_column_blocks.restype = i64
        _lib.oracle_column_block_width.argtypes = [i32]
        _lib.oracle_column_block_width.restype = i64
        _lib.oracle_column_block_choice.argtypes = [i64, i64, i32, i32, i64, i64]
        _lib.oracle_column_block_choice.restype = i32
        _lib.oracle_two_phase_sizes.argtypes = [i64, i64, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]
        _lib.oracle_two_phase_sizes.restype = None
        _lib.oracle_two_phase_layout.argtypes = [i64, i64, vp, vp, i32, i32, i32, i32] + [vp] * 9
        _lib.oracle_merge_path_snapped.argtypes = [i64, i64, vp, i32, i32, vp, vp]
        _lib.oracle_merge_path_snapped.restype = i64
        _lib.oracle_two_phase_layout.restype = None
        _lib.oracle_two_phase_choice.argtypes = [i64, i64, i64, i32, i32, i32, i32, i64, i64]
        _lib.oracle_scatter_counts.argtypes = [i64, vp, vp, i32, vp, vp, vp]
        _lib.oracle_scatter_counts.restype = None
        _lib.oracle_two_phase_choice.restype = i32
        _lib.oracle_csr_groups.argtypes = [i64, i64, vp, vp, i32]
        _lib.oracle_csr_groups.restype = i32
        _lib.oracle_group_matrix.argtypes = [i64, i64, vp, vp, i32, vp, vp]
        _lib.oracle_group_matrix.restype = None
        _lib.oracle_two_phase_piece_groups.argtypes = [i64, vp, i32, i32, i32, i32]
        _lib.oracle_two_phase_piece_groups.restype = i32
        _lib.oracle_grouped_two_phase_choice.argtypes = [i64, i64, i64, i32, i32, i32, i32, i32, i32, i64, i64]
        _lib.oracle_grouped_two_phase_choice.restype = i32
        _lib.oracle_sell_slices.argtypes = [i64, vp, i64, vp]
        _lib.oracle_sell_slices.restype = i64
        _lib.oracle_sell_fill.argtypes = [i64, vp, vp, i64, vp, vp, vp]
        _lib.oracle_sell_fill.restype = None
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype, size=None):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, (type(a), getattr(a, "dtype", None))
    if size is not None:
        assert a.size == size, (a.size, size)
    return a


def spmv_csr(dtype, m, n, rowptr, colidx, vals, x, y0=None, alpha=1.0, beta=0.0):
    """Returns (y_ref float64[m], S_ref float64[m]); S_ref[i] = sum_k |a_ik x_k|."""
    lib = _load()
    _chk(rowptr, np.int32, m + 1)
    nnz = int(rowptr[-1]) if m >= 0 else 0
    _chk(colidx, np.int32, nnz)
    if dtype == "f32":
        _chk(vals, np.float32, nnz), _chk(x, np.float32, n)
        fn = lib.oracle_spmv_csr_f32
    elif dtype == "bf16":
        _chk(vals, np.uint16, nnz), _chk(x, np.uint16, n)
        fn = lib.oracle_spmv_csr_bf16
    else:
        raise ValueError(dtype)
    if beta != 0.0:
        _chk(y0, np.float32, m)
    else:
        y0 = None
    y = np.empty(m, dtype=np.float64)
    S = np.empty(m, dtype=np.float64)
    rc = fn(m, n, _p(rowptr), _p(colidx), _p(vals), _p(x), _p(y0), alpha, beta, _p(y), _p(S))
    if rc != 0:
        raise ValueError("malformed CSR input")
    return y, S


def spmv_problem(p):
    """Oracle result for a workloads.CsrProblem-like object."""
    return spmv_csr(p.dtype, p.m, p.n, p.rowptr, p.colidx, p.vals, p.x, p.y0, p.alpha, p.beta)


def spmm_csr(m, n, rowptr, colidx, vals, B, C0=None, alpha=1.0, beta=0.0):
    """C <- alpha*A*B + beta*C0 for CSR A (m x n) and dense row-major B (n x K), possibly a column slice of a wider
    array; vals and B both float32, or both uint16 (bf16 bit patterns).  C0 is float32.
    Returns (C_ref float64[m, K], S_ref float64[m, K])."""
    lib = _load()
    _chk(rowptr, np.int32, m + 1), _chk(colidx, np.int32)
    assert vals.dtype == B.dtype and vals.dtype in (np.float32, np.uint16) and vals.flags.c_contiguous
    esz = B.dtype.itemsize
    assert B.ndim == 2 and B.shape[0] == n and B.strides[1] == esz
    K = B.shape[1]
    ldb = B.strides[0] // esz
    ldc = 0
    if beta != 0.0:
        assert C0.dtype == np.float32 and C0.shape == (m, K) and C0.strides[1] == 4
        ldc = C0.strides[0] // 4
    else:
        C0 = None
    Cr = np.empty((m, K), dtype=np.float64)
    S = np.empty((m, K), dtype=np.float64)
    fn = lib.oracle_spmm_csr_f32 if esz == 4 else lib.oracle_spmm_csr_bf16
    rc = fn(m, n, K, _p(rowptr), _p(colidx), _p(vals), B.ctypes.data_as(C.c_void_p), ldb,
            None if C0 is None else C0.ctypes.data_as(C.c_void_p), ldc, alpha, beta, _p(Cr), _p(S))
    if rc != 0:
        raise ValueError("malformed CSR input")
    return Cr, S


def _dt(dtype, vals, x):
    want = np.float32 if dtype == "f32" else np.uint16
    assert vals.dtype == want and x.dtype == want and vals.flags.c_contiguous and x.flags.c_contiguous, (vals.dtype, x.dtype)
    return 0 if dtype == "f32" else 1


def _y0(y0, m, beta):
    if beta == 0.0:
        return None
    return _chk(y0, np.float32, m)


def spmv_coo(dtype, m, n, row, col, vals, x, y0=None, alpha=1.0, beta=0.0):
    _chk(row, np.int32), _chk(col, np.int32, row.size)
    y, S = np.empty(m, np.float64), np.empty(m, np.float64)
    rc = _load().oracle_spmv_coo(m, n, row.size, _p(row), _p(col), _p(vals), _dt(dtype, vals, x), _p(x),
                                 _p(_y0(y0, m, beta)), alpha, beta, _p(y), _p(S))
    if rc:
        raise ValueError("index out of range")
    return y, S


def spmv_csc(dtype, m, n, col_offsets, row, vals, x, y0=None, alpha=1.0, beta=0.0):
    _chk(col_offsets, np.int32, n + 1), _chk(row, np.int32)
    y, S = np.empty(m, np.float64), np.empty(m, np.float64)
    rc = _load().oracle_spmv_csc(m, n, _p(col_offsets), _p(row), _p(vals), _dt(dtype, vals, x), _p(x),
                                 _p(_y0(y0, m, beta)), alpha, beta, _p(y), _p(S))
    if rc:
        raise ValueError("malformed CSC input")
    return y, S


def spmv_ell(dtype, m, n, width, col_ids, vals, x, y0=None, alpha=1.0, beta=0.0):
    _chk(col_ids, np.int32, m * width)
    assert vals.size == m * width
    y, S = np.empty(m, np.float64), np.empty(m, np.float64)
    rc = _load().oracle_spmv_ell(m, n, width, _p(col_ids), _p(vals), _dt(dtype, vals, x), _p(x),
                                 _p(_y0(y0, m, beta)), alpha, beta, _p(y), _p(S))
    if rc:
        raise ValueError("column out of range")
    return y, S


def row_stats(rowptr):
    lib = _load()
    m = rowptr.size - 1
    out = np.zeros(3, dtype=np.int64)
    lib.oracle_row_stats(m, _p(_chk(rowptr, np.int32)), _p(out))
    return {"min_len": int(out[0]), "max_len": int(out[1]), "n_empty": int(out[2])}


def row_bins(rowptr):
    lib = _load()
    m = rowptr.size - 1
    cnt = np.zeros(NUM_BINS, dtype=np.int32)
    off = np.zeros(NUM_BINS + 1, dtype=np.int32)
    rows = np.zeros(m, dtype=np.int32)
    lib.oracle_row_bins(m, _p(_chk(rowptr, np.int32)), _p(cnt), _p(off), _p(rows))
    return cnt, off, rows


def row_blocks(rowptr, block_nnz, rows_max):
    lib = _load()
    m = rowptr.size - 1
    out = np.zeros(m + 1, dtype=np.int32)
    nb = lib.oracle_row_blocks(m, _p(_chk(rowptr, np.int32)), block_nnz, rows_max, _p(out))
    return out[: nb + 1].copy()


def merge_path(rowptr, ipc):
    lib = _load()
    m = rowptr.size - 1
    nnz = int(rowptr[-1])
    P = (m + nnz + ipc - 1) // ipc
    mp_row = np.zeros(P + 1, dtype=np.int32)
    mp_nz = np.zeros(P + 1, dtype=np.int32)
    P2 = lib.oracle_merge_path(m, nnz, _p(_chk(rowptr, np.int32)), ipc, _p(mp_row), _p(mp_nz))
    assert P2 == P
    return mp_row, mp_nz


def tile_shape(m, nnz):
    """Default (block_nnz, rows_max) for a matrix of m rows and nnz entries."""
    out = np.zeros(2, dtype=np.int32)
    _load().oracle_tile_shape(m, nnz, out[0:1].ctypes.data_as(C.c_void_p), out[1:2].ctypes.data_as(C.c_void_p))
    return int(out[0]), int(out[1])


def plan(m, nnz, max_len, block_nnz):
    return int(_load().oracle_plan(m, nnz, max_len, block_nnz))


def vector_lanes(m, nnz):
    return int(_load().oracle_vector_lanes(m, nnz))


def x_windows(rowptr, colidx, row_blocks, block_nnz, vec_elems):
    """(nv[nb], xv_ptr[nb+1], xv_start[sum nv], lidx[nnz]) of the row blocks' x windows."""
    lib = _load()
    _chk(rowptr, np.int32), _chk(colidx, np.int32), _chk(row_blocks, np.int32)
    nb = row_blocks.size - 1
    nv = np.zeros(max(nb, 1), dtype=np.int32)
    args = (nb, _p(row_blocks), _p(rowptr), _p(colidx), block_nnz, vec_elems, _p(nv))
    total = lib.oracle_x_windows(*args, None, None)
    xv_start = np.zeros(max(total, 1), dtype=np.int32)
    lidx = np.zeros(max(colidx.size, 1), dtype=np.uint16)
    assert lib.oracle_x_windows(*args, _p(xv_start), _p(lidx)) == total
    nv = nv[:nb]
    xv_ptr = np.concatenate([[0], np.cumsum(nv, dtype=np.int64)]).astype(np.int32)
    return nv, xv_ptr, xv_start[:total], lidx[: colidx.size]


def window_choice(nv, nnz, max_vectors=MAX_X_VECTORS):
    nv = np.ascontiguousarray(nv, dtype=np.int32)
    return bool(_load().oracle_window_choice(nv.size, _p(nv), nnz, max_vectors))


def lidx_grouped(rowptr, row_blocks, lidx):
    """Whether the window positions come in aligned groups of eight consecutive numbers."""
    lidx = np.ascontiguousarray(lidx, dtype=np.uint16)
    return bool(_load().oracle_lidx_grouped(int(rowptr[-1]), _p(lidx), row_blocks.size - 1, _p(_chk(row_blocks, np.int32)),
                                            _p(_chk(rowptr, np.int32))))


def row_patterns(rowptr, row_blocks, lidx, block_nnz, max_runs=MAX_PATTERN_RUNS, max_len=MAX_PATTERN_LEN):
    """Runs of rows whose window positions repeat with a constant step.  Returns a dict: n_runs[nb]; run_rows, run_len,
    run_base, run_stride, each [nb, max_runs]; pat_ptr[nb+1], pat[pat_ptr[nb]]; covered (entries of patterned blocks)."""
    lib = _load()
    _chk(rowptr, np.int32), _chk(row_blocks, np.int32)
    lidx = np.ascontiguousarray(lidx, dtype=np.uint16)
    nb = row_blocks.size - 1
    out = dict(n_runs=np.zeros(max(nb, 1), np.int32))
    for name in ("run_rows", "run_len", "run_base", "run_stride"):
        out[name] = np.zeros((max(nb, 1), max_runs), np.int32)
    pat_ptr = np.zeros(nb + 1, np.int32)
    args = (nb, _p(row_blocks), _p(rowptr), _p(lidx), block_nnz, max_runs, max_len, _p(out["n_runs"]), _p(out["run_rows"]),
            _p(out["run_len"]), _p(out["run_base"]), _p(out["run_stride"]), _p(pat_ptr))
    covered = lib.oracle_row_patterns(*args, None)
    pat = np.zeros(max(int(pat_ptr[-1]), 1), np.uint16)
    assert lib.oracle_row_patterns(*args, _p(pat)) == covered
    for name in ("n_runs", "run_rows", "run_len", "run_base", "run_stride"):
        out[name] = out[name][:nb]
    out.update(pat_ptr=pat_ptr, pat=pat[: int(pat_ptr[-1])], covered=int(covered))
    return out


def pattern_choice(nnz, covered):
    return bool(_load().oracle_pattern_choice(nnz, covered))


def column_blocks(m, n, rowptr, colidx, width):
    """(cb_ptr[C+1], cb_row[nnz], cb_col[nnz], cb_src[nnz]) of the column-blocked regrouping."""
    _chk(rowptr, np.int32, m + 1), _chk(colidx, np.int32)
    C = (n + width - 1) // width
    nnz = colidx.size
    ptr = np.zeros(C + 1, np.int32)
    row, col, src = (np.zeros(max(nnz, 1), np.int32) for _ in range(3))
    assert _load().oracle_column_blocks(m, n, _p(rowptr), _p(colidx), width, _p(ptr), _p(row), _p(col), _p(src)) == C
    return ptr, row[:nnz], col[:nnz], src[:nnz]


def column_block_width(dtype):
    return int(_load().oracle_column_block_width(4 if dtype == "f32" else 2))


def spmm_row_order(rowptr, window=4096):
    """Inside every window of `window` consecutive rows: row ids by decreasing
    min(ceil(len / 4), 64), rows of equal key ascending (int32[m])."""
    m = rowptr.size - 1
    _chk(rowptr, np.int32, m + 1)
    assert window >= 1
    rows = np.empty(m, dtype=np.int32)
    _load().oracle_spmm_row_order(m, _p(rowptr), window, _p(rows))
    return rows


def spmm_packed_layout(rowptr, rows):
    """(desc int32[2G+2], number of blocks) of the packed copy for the row order `rows`."""
    m = rowptr.size - 1
    _chk(rowptr, np.int32, m + 1), _chk(rows, np.int32, m)
    desc = np.zeros(2 * ((m + 15) // 16) + 2, dtype=np.int32)
    blocks = _load().oracle_spmm_packed_layout(m, _p(rowptr), _p(rows), _p(desc))
    return desc, int(blocks)


def spmm_pack(rowptr, colidx, vals, rows, desc):
    """(columns int32 with -1 as padding, values float32) of the packed copy, one slot each."""
    m = rowptr.size - 1
    _chk(rowptr, np.int32, m + 1), _chk(colidx, np.int32), _chk(vals, np.float32), _chk(rows, np.int32, m)
    slots = int(desc[-2]) * 256
    pcol, pval = np.zeros(slots, dtype=np.int32), np.zeros(slots, dtype=np.float32)
    _load().oracle_spmm_pack(m, _p(rowptr), _p(colidx), _p(vals), _p(rows), _p(desc), _p(pcol), _p(pval))
    return pcol, pval


def spmm_packed_choice(nnz, blocks):
    return bool(_load().oracle_spmm_packed_choice(nnz, blocks))


def column_block_choice(n, nnz, dtype, plan, vectors, entries):
    """vectors, entries: scatter_counts() of the row blocks' x windows (vectors < 0: not counted)."""
    return bool(_load().oracle_column_block_choice(n, nnz, 4 if dtype == "f32" else 2, plan, vectors, entries))


def merge_path_snapped(rowptr, ipc, snap):
    """Splits of the two-pass plan's chunks: (row, nz), each of P + 1 entries."""
    m = rowptr.size - 1
    nnz = int(rowptr[-1])
    room = (m + nnz) // (ipc - snap) + 2
    row, nz = np.zeros(room, np.int32), np.zeros(room, np.int32)
    P = _load().oracle_merge_path_snapped(m, nnz, _p(_chk(rowptr, np.int32)), ipc, snap, _p(row), _p(nz))
    return row[:P + 1].copy(), nz[:P + 1].copy()


def two_phase_layout(m, n, rowptr, colidx, shift=TP_SHIFT, items=TP_ITEMS, piece_groups=TP_PIECE_GROUPS, snap=TP_SNAP):
    """The two-pass plan's regrouping: dict with C, P, S, Q and the arrays tp_row, tp_nz, tp_piece_c, tp_piece_g,
    tp_chunk_g, tp_col, tp_src, tp_from, tp_pos."""
    lib = _load()
    _chk(rowptr, np.int32, m + 1), _chk(colidx, np.int32)
    sizes = [C.c_int64() for _ in range(4)]
    lib.oracle_two_phase_sizes(m, n, _p(rowptr), _p(colidx), shift, items, snap, piece_groups, *[C.byref(v) for v in sizes])
    S, Q, P, Cn = (int(v.value) for v in sizes)
    out = dict(tp_row=np.zeros(P + 1, np.int32), tp_nz=np.zeros(P + 1, np.int32), tp_piece_c=np.zeros(Q, np.int32),
               tp_piece_g=np.zeros(Q + 1, np.int32), tp_chunk_g=np.zeros(P + 1, np.int32), tp_col=np.zeros(S, np.uint16),
               tp_src=np.zeros(S, np.int32), tp_from=np.zeros(S // 4, np.int32), tp_pos=np.zeros(S, np.uint16))
    lib.oracle_two_phase_layout(m, n, _p(rowptr), _p(colidx), shift, items, snap, piece_groups, *[_p(v) for v in out.values()])
    out.update(C=Cn, P=P, S=S, Q=Q)
    return out


def two_phase_piece_groups(groups, resident, waves=TP_WAVES, cap=TP_PIECE_CAP, floor=TP_PIECE_FLOOR):
    """The library's cap on a piece's groups; groups[c] = groups of four slots of column block c."""
    g = np.ascontiguousarray(groups, dtype=np.int64)
    return int(_load().oracle_two_phase_piece_groups(g.size, _p(g), resident, waves, cap, floor))


def grouped_two_phase_choice(m, n, nnz, dtype, plan, group_aligned, vectors, entries, items=TP_ITEMS):
    eb, ve = (4, 4) if dtype == "f32" else (2, 8)
    return int(_load().oracle_grouped_two_phase_choice(m, n, nnz, eb, ve, plan, int(group_aligned), TP_GROUP_SHIFT[dtype], items,
                                                       vectors, entries))


def csr_groups(m, rowptr, colidx, width=TP_GROUP):
    """1 when the matrix is group-aligned (whole groups of `width` consecutive, aligned columns), else 0."""
    _chk(rowptr, np.int32, m + 1), _chk(colidx, np.int32)
    return int(_load().oracle_csr_groups(m, colidx.size, _p(rowptr), _p(colidx), width))


def group_matrix(m, rowptr, colidx, width=TP_GROUP):
    """(rowptr_g, col_g) of the matrix of groups."""
    _chk(rowptr, np.int32, m + 1), _chk(colidx, np.int32)
    rp, cg = np.zeros(m + 1, np.int32), np.zeros(colidx.size // width, np.int32)
    _load().oracle_group_matrix(m, colidx.size, _p(rowptr), _p(colidx), width, _p(rp), _p(cg))
    return rp, cg


def sell_layout(m, rowptr, colidx, height=SELL_HEIGHT):
    """The sliced ELL re-layout: dict with ns (slices), S (slots) and the arrays sell_ptr (int32, ns + 1),
    sell_col, sell_src (int32, S; -1 where a slot holds no entry)."""
    lib = _load()
    _chk(rowptr, np.int32, m + 1), _chk(colidx, np.int32)
    ns = (m + height - 1) // height
    ptr = np.zeros(ns + 1, np.int64)
    S = int(lib.oracle_sell_slices(m, _p(rowptr), height, _p(ptr)))
    col, src = np.zeros(S, np.int32), np.zeros(S, np.int32)
    lib.oracle_sell_fill(m, _p(rowptr), _p(colidx), height, _p(ptr), _p(col), _p(src))
    assert S < 2 ** 31
    return dict(ns=ns, S=S, sell_ptr=ptr.astype(np.int32), sell_col=col, sell_src=src)


def scatter_counts(rowptr, row_blocks, block_nnz, nv):
    """(distinct x vectors of the row blocks summed, entries of the blocks that were counted)."""
    nv = np.ascontiguousarray(nv, dtype=np.int32)
    vectors, entries = C.c_int64(), C.c_int64()
    _load().oracle_scatter_counts(row_blocks.size - 1, _p(_chk(row_blocks, np.int32)), _p(_chk(rowptr, np.int32)), block_nnz, _p(nv),
                                  C.byref(vectors), C.byref(entries))
    return int(vectors.value), int(entries.value)


def two_phase_choice(m, n, nnz, dtype, plan, vectors, entries, shift=TP_SHIFT, items=TP_ITEMS):
    """vectors, entries: scatter_counts() of the row blocks' x windows (vectors < 0: not counted)."""
    return bool(_load().oracle_two_phase_choice(m, n, nnz, 4 if dtype == "f32" else 2, plan, shift, items, vectors, entries))
