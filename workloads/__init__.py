"""Seeded synthetic CSR workloads.

This module only *builds inputs*: index arrays, value arrays, vectors and the
scalars alpha/beta.  It contains none of the sparse product's arithmetic and is
the one module that both the CPU oracle's tests and the HIP path's tests/bench
import.  Neither of those two imports the other.

All arrays are numpy, host side:
  rowptr  int32[m+1]   "starting index of each row" (CSR row offsets, App. C task 12)
  colidx  int32[nnz]   column index of every stored entry
  vals    float32[nnz] (dtype "f32")  or uint16[nnz] bf16 bit patterns (dtype "bf16")
  x       float32[n]   or uint16[n] bf16 bit patterns
  y0      float32[m]   initial y (only read by the operation when beta != 0)

bf16 rounding (round-to-nearest-even on the upper 16 bits of an IEEE float32)
is done here, once, so every consumer receives identical bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

SEED_BASE = 260307169  # seed of config k (1-based) is SEED_BASE + k

__all__ = [
    "CsrProblem", "SEED_BASE", "f32_to_bf16_bits", "bf16_bits_to_f32",
    "uniform_rows", "laplace2d", "stencil27", "powerlaw", "block_clustered",
    "density_random", "clustered_arithmetic", "from_row_lengths", "exact_integer", "tiny_adversarial",
    "config", "CONFIG_NAMES", "to_coo", "to_csc", "to_ell",
]


# ----------------------------------------------------------------------------- helpers
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round-to-nearest-even, finite inputs."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> the float32 it denotes (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def _uniform_pm1(rng: np.random.Generator, size) -> np.ndarray:
    """U(-1, 1) as float32."""
    u = rng.random(size, dtype=np.float32)
    return (u * np.float32(2.0) - np.float32(1.0)).astype(np.float32)


@dataclass
class CsrProblem:
    name: str
    dtype: str                      # "f32" | "bf16"  (storage type of vals and x; y is always float32)
    m: int
    n: int
    rowptr: np.ndarray
    colidx: np.ndarray
    vals: np.ndarray
    x: np.ndarray
    y0: Optional[np.ndarray]
    alpha: float = 1.0
    beta: float = 0.0
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def algorithmic_bytes(self) -> int:
        """Compulsory traffic of one y = alpha*A*x + beta*y:
        vals + colidx + rowptr + x + y written (+ y read when beta != 0)."""
        e = 4 if self.dtype == "f32" else 2
        b = self.nnz * (e + 4) + 4 * (self.m + 1) + e * self.n + 4 * self.m
        if self.beta != 0.0:
            b += 4 * self.m
        return b

    def flops(self) -> int:
        return 2 * self.nnz


def _finish(name, dtype, m, n, rowptr, colidx, vals_f32, x_f32, y0, alpha, beta, meta=None) -> CsrProblem:
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    assert rowptr[-1] < 2 ** 31
    rowptr = rowptr.astype(np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    if dtype == "bf16":
        vals = f32_to_bf16_bits(vals_f32)
        x = f32_to_bf16_bits(x_f32)
    else:
        vals = np.ascontiguousarray(vals_f32, dtype=np.float32)
        x = np.ascontiguousarray(x_f32, dtype=np.float32)
    if y0 is not None:
        y0 = np.ascontiguousarray(y0, dtype=np.float32)
    return CsrProblem(name, dtype, int(m), int(n), rowptr, colidx, vals, x, y0, float(alpha), float(beta), meta or {})


def _distinct_sorted_per_row(rng, lens: np.ndarray, hi: int) -> np.ndarray:
    """For every row r draw lens[r] distinct integers uniformly from [0, hi), ascending.

    Draw with replacement, sort by (row, value), redraw the members of rows that hold
    a repeated value, until no row has one.  Needs lens[r] <= hi.
    """
    lens = np.asarray(lens, dtype=np.int64)
    assert lens.max(initial=0) <= hi
    nnz = int(lens.sum())
    rows = np.repeat(np.arange(lens.size, dtype=np.int64), lens)
    cols = rng.integers(0, hi, size=nnz, dtype=np.int64)
    shift = np.int64(hi)
    key = rows * shift + cols
    key.sort(kind="stable")
    starts = np.concatenate(([0], np.cumsum(lens)))
    while True:
        # a repeated (row, value) pair: keep its first copy, redraw the later ones --
        # the same distribution as drawing one at a time and rejecting values already held
        dup = np.flatnonzero(key[1:] == key[:-1]) + 1
        if dup.size == 0:
            break
        key[dup] = (key[dup] // shift) * shift + rng.integers(0, hi, size=dup.size, dtype=np.int64)
        bad_rows = np.unique(key[dup] // shift)
        if bad_rows.size <= 4096:
            for r in bad_rows:          # re-sort only inside the touched rows
                key[starts[r]:starts[r + 1]].sort()
        else:
            key.sort(kind="stable")
    return (key % shift).astype(np.int32)


# ----------------------------------------------------------------------------- generators
def uniform_rows(m=4096, n=4096, per_row=16, seed=SEED_BASE + 1, dtype="f32", alpha=1.0, beta=0.0) -> CsrProblem:
    """Exactly `per_row` stored entries in every row, columns uniform without
    replacement, ascending; vals and x ~ U(-1,1)."""
    rng = _rng(seed)
    lens = np.full(m, per_row, dtype=np.int64)
    colidx = _distinct_sorted_per_row(rng, lens, n)
    rowptr = np.arange(m + 1, dtype=np.int64) * per_row
    vals = _uniform_pm1(rng, m * per_row)
    x = _uniform_pm1(rng, n)
    y0 = _uniform_pm1(rng, m) if beta != 0.0 else None
    return _finish(f"uniform{per_row}_{m}x{n}", dtype, m, n, rowptr, colidx, vals, x, y0, alpha, beta,
                   {"per_row": per_row})


def laplace2d(grid=1024, seed=SEED_BASE + 2, dtype="f32", alpha=1.0, beta=0.5) -> CsrProblem:
    """5-point Laplacian on a grid x grid mesh, row id = iy*grid + ix, diagonal 4,
    in-grid neighbours -1, out-of-grid neighbours dropped (homogeneous Dirichlet)."""
    rng = _rng(seed)
    N = grid * grid
    r = np.arange(N, dtype=np.int64)
    ix = r % grid
    iy = r // grid
    cand = np.stack([r - grid, r - 1, r, r + 1, r + grid], axis=1)
    ok = np.stack([iy > 0, ix > 0, np.ones(N, bool), ix < grid - 1, iy < grid - 1], axis=1)
    v = np.broadcast_to(np.array([-1.0, -1.0, 4.0, -1.0, -1.0], dtype=np.float32), (N, 5))
    lens = ok.sum(axis=1)
    rowptr = np.concatenate(([0], np.cumsum(lens)))
    colidx = cand[ok]
    vals = v[ok]
    x = _uniform_pm1(rng, N)
    y0 = _uniform_pm1(rng, N)
    return _finish(f"laplace2d_{grid}", dtype, N, N, rowptr, colidx, vals, x, y0 if beta != 0.0 else None, alpha, beta,
                   {"grid": grid})


def stencil27(grid=128, seed=SEED_BASE + 3, dtype="bf16", alpha=1.0, beta=0.0) -> CsrProblem:
    """27-point stencil on a grid^3 mesh truncated at the faces, row id = (iz*grid+iy)*grid+ix.
    Diagonal exactly 26.0, every other stored entry ~ U(-1,1) drawn independently."""
    rng = _rng(seed)
    g = grid
    N = g * g * g
    r = np.arange(N, dtype=np.int64)
    ix = r % g
    iy = (r // g) % g
    iz = r // (g * g)
    cand = np.empty((N, 27), dtype=np.int32)
    ok = np.empty((N, 27), dtype=bool)
    j = 0
    diag_slot = None
    for dz in (-1, 0, 1):
        okz = (iz + dz >= 0) & (iz + dz < g)
        for dy in (-1, 0, 1):
            oky = okz & (iy + dy >= 0) & (iy + dy < g)
            for dx in (-1, 0, 1):
                ok[:, j] = oky & (ix + dx >= 0) & (ix + dx < g)
                cand[:, j] = r + (dz * g + dy) * g + dx
                if dz == 0 and dy == 0 and dx == 0:
                    diag_slot = j
                j += 1
    lens = ok.sum(axis=1)
    rowptr = np.concatenate(([0], np.cumsum(lens)))
    colidx = cand[ok]
    v = _uniform_pm1(rng, (N, 27))
    v[:, diag_slot] = np.float32(26.0)
    vals = v[ok]
    del v, cand
    x = _uniform_pm1(rng, N)
    y0 = _uniform_pm1(rng, N) if beta != 0.0 else None
    return _finish(f"stencil27_{grid}", dtype, N, N, rowptr, colidx, vals, x, y0, alpha, beta, {"grid": grid})


def powerlaw_lengths(rng, m: int, shape=1.5, scale=3.75, cap=200_000, literal=False) -> np.ndarray:
    """Row lengths of the power-law workload.

    Primary reading: discrete Lomax (Pareto type II) with location 1:
        len = min(cap, 1 + floor(scale * (U^(-1/shape) - 1))),  U in (0, 1]
    scale = 3.75 makes the mean 8.0005 with shape 1.5, minimum 1.
    literal=True: type-I Pareto  len = min(cap, floor(U^(-1/shape)))  (mean 2.61)."""
    u = 1.0 - rng.random(m)  # (0, 1]
    t = u ** (-1.0 / shape)
    if literal:
        ln = np.floor(t)
    else:
        ln = 1.0 + np.floor(scale * (t - 1.0))
    return np.minimum(ln, float(cap)).astype(np.int64)


def powerlaw(m=4_000_000, n=None, seed=SEED_BASE + 4, dtype="f32", shape=1.5, scale=3.75, cap=200_000,
             literal=False, alpha=1.0, beta=0.0) -> CsrProblem:
    rng = _rng(seed)
    n = m if n is None else n
    lens = powerlaw_lengths(rng, m, shape, scale, min(cap, n), literal)
    colidx = _distinct_sorted_per_row(rng, lens, n)
    rowptr = np.concatenate(([0], np.cumsum(lens)))
    vals = _uniform_pm1(rng, int(rowptr[-1]))
    x = _uniform_pm1(rng, n)
    y0 = _uniform_pm1(rng, m) if beta != 0.0 else None
    return _finish(f"powerlaw{'_literal' if literal else ''}_{m}", dtype, m, n, rowptr, colidx, vals, x, y0, alpha, beta,
                   {"shape": shape, "scale": scale, "cap": cap, "literal": literal})


def block_clustered(m=1_000_000, n=None, blocks_per_row=16, width=8, seed=SEED_BASE + 5, dtype="bf16",
                    alpha=1.0, beta=0.0) -> CsrProblem:
    """Every row holds `blocks_per_row` distinct `width`-aligned runs of `width`
    consecutive columns, runs chosen uniformly without replacement; vals, x ~ N(0,1)."""
    rng = _rng(seed)
    n = m if n is None else n
    slots = n // width
    lens = np.full(m, blocks_per_row, dtype=np.int64)
    b = _distinct_sorted_per_row(rng, lens, slots).astype(np.int64).reshape(m, blocks_per_row, 1)
    colidx = (b * width + np.arange(width, dtype=np.int64)).reshape(-1)
    per_row = blocks_per_row * width
    rowptr = np.arange(m + 1, dtype=np.int64) * per_row
    vals = rng.standard_normal(m * per_row, dtype=np.float32)
    x = rng.standard_normal(n, dtype=np.float32)
    y0 = rng.standard_normal(m, dtype=np.float32) if beta != 0.0 else None
    return _finish(f"blockclustered_{m}", dtype, m, n, rowptr, colidx, vals, x, y0, alpha, beta,
                   {"blocks_per_row": blocks_per_row, "width": width})


def density_random(rows=1024, cols=2048, density=0.01, seed=SEED_BASE + 12, dtype="f32", alpha=1.0, beta=0.0) -> CsrProblem:
    """The benchmark's own shape for this operation (App. C task 12): nnz = rows*cols*density
    positions chosen uniformly without replacement over the whole matrix."""
    rng = _rng(seed)
    nnz = int(rows * cols * density)
    flat = rng.choice(rows * cols, size=nnz, replace=False)
    flat.sort()
    r = flat // cols
    colidx = flat % cols
    lens = np.bincount(r, minlength=rows)
    rowptr = np.concatenate(([0], np.cumsum(lens)))
    vals = _uniform_pm1(rng, nnz)
    x = _uniform_pm1(rng, cols)
    y0 = _uniform_pm1(rng, rows) if beta != 0.0 else None
    return _finish(f"density{density}_{rows}x{cols}", dtype, rows, cols, rowptr, colidx, vals, x, y0, alpha, beta,
                   {"density": density})


def clustered_arithmetic(m=2 ** 23, runs=17, width=8, n=2 ** 22, seed=SEED_BASE + 31, alpha=1.0, beta=0.5) -> CsrProblem:
    """A bf16 matrix of more than 2^30 stored entries at the default size (m * runs * width =
    1 140 850 688), laid out in seconds and without large temporaries: run j of row r covers the
    `width` columns from width * ((3 r + 24671 j) mod (n / width)) on (24671 is odd, so the runs
    of a row are distinct while runs <= n / width <= 2^31 / width).  Values are a seeded N(0,1)
    pattern of 1 000 003 numbers repeated over the entries: the period shares no factor with a
    power of two, so an entry index that is off by 2^k meets a different value.  x, y0 ~ N(0,1)."""
    rng = _rng(seed)
    slots = n // width
    assert slots >= runs and 3 * m + 24671 * runs < 2 ** 31 and m * runs * width < 2 ** 31
    r = np.arange(m, dtype=np.int32).reshape(m, 1)
    j = np.arange(runs, dtype=np.int32).reshape(1, runs)
    starts = ((3 * r + 24671 * j) % np.int32(slots)) * np.int32(width)          # int32 [m, runs]
    colidx = np.empty((m, runs, width), dtype=np.int32)
    np.add(starts.reshape(m, runs, 1), np.arange(width, dtype=np.int32), out=colidx)
    per_row = runs * width
    rowptr = (np.arange(m + 1, dtype=np.int64) * per_row).astype(np.int32)
    pattern = f32_to_bf16_bits(rng.standard_normal(1_000_003, dtype=np.float32))
    vals = np.resize(pattern, m * per_row)
    x = f32_to_bf16_bits(rng.standard_normal(n, dtype=np.float32))
    y0 = rng.standard_normal(m, dtype=np.float32) if beta != 0.0 else None
    return CsrProblem(f"clustered_arithmetic_{m}x{per_row}", "bf16", int(m), int(n), rowptr, colidx.reshape(-1), vals, x, y0,
                      float(alpha), float(beta), {"runs": runs, "width": width})


def banded_random(m, half_width, per_row, seed=SEED_BASE + 41, dtype="f32", alpha=1.0, beta=0.0) -> CsrProblem:
    """Square matrix with `per_row` entries a row at random columns within `half_width` of the diagonal: the band is cut
    into `per_row` equal strata and every row draws one column from each (so they are distinct and ascending; clipped at the
    matrix edges, where columns may then repeat).  Clustered columns that need not fit an x window."""
    rng = _rng(seed)
    stratum = (2 * half_width + 1) // per_row
    assert stratum >= 1
    off = np.arange(per_row, dtype=np.int64)[None, :] * stratum + rng.integers(0, stratum, (m, per_row)) - half_width
    cols = np.clip(np.arange(m, dtype=np.int64)[:, None] + off, 0, m - 1)
    rowptr = np.arange(m + 1, dtype=np.int64) * per_row
    colidx = cols.reshape(-1)
    vals = _uniform_pm1(rng, colidx.size)
    x = _uniform_pm1(rng, m)
    y0 = _uniform_pm1(rng, m) if beta != 0.0 else None
    return _finish(f"banded{half_width}_{per_row}_{m}", dtype, m, m, rowptr, colidx, vals, x, y0, alpha, beta)


def from_row_lengths(lens, n, seed=1, dtype="f32", alpha=1.0, beta=0.0, sort_cols=True, allow_dup=False,
                     normal=False, name="custom") -> CsrProblem:
    """Arbitrary row-length profile; columns uniform (distinct + ascending unless asked otherwise)."""
    rng = _rng(seed)
    lens = np.asarray(lens, dtype=np.int64)
    m = lens.size
    nnz = int(lens.sum())
    if allow_dup:
        colidx = rng.integers(0, n, size=nnz, dtype=np.int64)
    else:
        colidx = _distinct_sorted_per_row(rng, lens, n).astype(np.int64)
    rowptr = np.concatenate(([0], np.cumsum(lens)))
    if not sort_cols:
        for r in range(m):
            s, e = rowptr[r], rowptr[r + 1]
            colidx[s:e] = rng.permutation(colidx[s:e])
    if normal:
        vals = rng.standard_normal(nnz, dtype=np.float32)
        x = rng.standard_normal(n, dtype=np.float32)
        y0 = rng.standard_normal(m, dtype=np.float32)
    else:
        vals = _uniform_pm1(rng, nnz)
        x = _uniform_pm1(rng, n)
        y0 = _uniform_pm1(rng, m)
    return _finish(name, dtype, m, n, rowptr, colidx, vals, x, y0, alpha, beta)


def exact_integer(lens, n, seed=2, dtype="f32", alpha=1.0, beta=0.0, name="exact_int") -> CsrProblem:
    """vals in {-2..2}, x in {-4..4}, y0 in {-8..8}: all representable in bf16 and every
    partial sum an integer far below 2^24, so any summation order gives the same float."""
    rng = _rng(seed)
    lens = np.asarray(lens, dtype=np.int64)
    m = lens.size
    nnz = int(lens.sum())
    colidx = _distinct_sorted_per_row(rng, lens, n)
    rowptr = np.concatenate(([0], np.cumsum(lens)))
    vals = rng.integers(-2, 3, size=nnz).astype(np.float32)
    x = rng.integers(-4, 5, size=n).astype(np.float32)
    y0 = rng.integers(-8, 9, size=m).astype(np.float32)
    return _finish(name, dtype, m, n, rowptr, colidx, vals, x, y0, alpha, beta)


def tiny_adversarial(seed=7, dtype="f32"):
    """Small shapes aimed at indexing mistakes: empty rows (leading, trailing, runs),
    a single very long row, lengths straddling vector widths and tile sizes, m != n,
    unsorted and repeated columns."""
    out = []
    mk = lambda lens, n, **kw: from_row_lengths(lens, n, seed=seed + len(out), dtype=dtype, **kw)
    out.append(mk([0, 0, 0], 5, name="all_empty", beta=0.5))
    out.append(mk([3], 3, name="one_full_row"))
    out.append(mk([0, 1, 0, 0, 2, 0], 7, name="empty_runs", beta=-1.25, alpha=0.5))
    out.append(mk([1] * 130, 9, name="len1_rows"))
    out.append(mk(list(range(0, 70)), 97, name="ramp_0_69", beta=2.0))
    out.append(mk([5000], 6000, name="single_long_row"))
    out.append(mk([0, 0, 4100, 0, 3, 0], 4500, name="long_between_empty", alpha=-2.0))
    out.append(mk([7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257], 300, name="pow2_edges"))
    out.append(mk([2047, 1, 2048, 1, 2049, 1], 2100, name="tile_edges", beta=1.0))
    out.append(mk([4] * 1000 + [0] * 300 + [5] * 777, 50, name="short_mixed", beta=0.5))
    out.append(mk([6] * 40, 11, name="dup_unsorted", allow_dup=True, sort_cols=False))
    out.append(mk([3] * 5, 100000, name="wide_n"))
    return out


# ----------------------------------------------------------------------------- the five configs
CONFIG_NAMES = {
    1: "cfg1_uniform16_4096_f32",
    2: "cfg2_laplace2d_1024_f32",
    3: "cfg3_stencil27_128_bf16",
    4: "cfg4_powerlaw_4M_f32",
    5: "cfg5_blockclustered_1M_bf16",
}


def config(k: int, scale: float = 1.0) -> CsrProblem:
    """The k-th (1-based) benchmark configuration; scale < 1 shrinks it for CPU-side tests."""
    if k == 1:
        m = max(64, int(4096 * scale))
        p = uniform_rows(m, m, 16)
    elif k == 2:
        p = laplace2d(max(8, int(1024 * scale)))
    elif k == 3:
        p = stencil27(max(4, int(128 * scale)))
    elif k == 4:
        p = powerlaw(max(1000, int(4_000_000 * scale)))
    elif k == 5:
        p = block_clustered(max(1024, int(1_000_000 * scale)))
    else:
        raise ValueError(k)
    if scale == 1.0:
        p.name = CONFIG_NAMES[k]
    return p


# ----------------------------------------------------------------------------- other storage layouts
# Pure re-layouts of a CsrProblem (no arithmetic of the method): App. C tasks 8 (COO), 10 (CSC), 14 (ELL).
def to_coo(p: CsrProblem, shuffle_seed=None):
    """(row_indices, col_indices, values) in CSR order, or scrambled with the given seed."""
    row = np.repeat(np.arange(p.m, dtype=np.int32), np.diff(p.rowptr))
    col, vals = p.colidx.copy(), p.vals.copy()
    if shuffle_seed is not None:
        perm = np.random.default_rng(shuffle_seed).permutation(p.nnz)
        row, col, vals = row[perm], col[perm], vals[perm]
    return np.ascontiguousarray(row), np.ascontiguousarray(col), np.ascontiguousarray(vals)


def to_csc(p: CsrProblem):
    """(col_offsets[n+1], row_indices, values), entries of a column in ascending row order."""
    row = np.repeat(np.arange(p.m, dtype=np.int32), np.diff(p.rowptr))
    order = np.argsort(p.colidx, kind="stable")
    counts = np.bincount(p.colidx, minlength=p.n)
    col_offsets = np.concatenate(([0], np.cumsum(counts))).astype(np.int32)
    return col_offsets, np.ascontiguousarray(row[order]), np.ascontiguousarray(p.vals[order])


def to_ell(p: CsrProblem, width=None):
    """(width, col_ids[m*width], values[m*width]) row-major; padding slots have col_id -1 and value -1."""
    lens = np.diff(p.rowptr)
    width = int(lens.max(initial=0)) if width is None else int(width)
    assert width >= lens.max(initial=0)
    col_ids = np.full((p.m, max(width, 0)), -1, dtype=np.int32)
    if p.dtype == "f32":
        vals = np.full((p.m, width), -1.0, dtype=np.float32)
    else:
        vals = np.full((p.m, width), f32_to_bf16_bits(np.array([-1.0], np.float32))[0], dtype=np.uint16)
    slot = np.arange(p.nnz) - np.repeat(p.rowptr[:-1], lens)
    rows = np.repeat(np.arange(p.m), lens)
    col_ids[rows, slot] = p.colidx
    vals[rows, slot] = p.vals
    return width, col_ids.ravel().copy(), vals.ravel().copy()
