"""Pins for the CPU oracle of the analysis outputs (row statistics, length bins, row blocks,
merge-path splits, plan).  Checked against hand-worked fixtures, closed-form counts of the
structured workloads, defining invariants, and tiny brute-force restatements in Python."""
import json
import math

import numpy as np
import pytest

import oracle
import workloads as w


def rowptr_of(lens):
    return np.concatenate(([0], np.cumsum(np.asarray(lens, dtype=np.int64)))).astype(np.int32)


RAGGED = [
    [],
    [0],
    [0, 0, 0],
    [5],
    [1, 0, 2, 0, 0, 7, 3],
    list(range(40)),
    [100, 1, 1, 1, 100, 0, 0, 250, 3],
    [2] * 1000,
]


@pytest.fixture(scope="module")
def hand(golden_dir):
    return json.loads((golden_dir / "analysis_handworked.json").read_text())


# ------------------------------------------------------------------ bins
def test_bins_handworked(hand):
    lens, want = hand["bins"]["lens"], hand["bins"]["bin"]
    cnt, off, rows = oracle.row_bins(rowptr_of(lens))
    got = np.empty(len(lens), dtype=int)
    for b in range(oracle.NUM_BINS):
        got[rows[off[b]:off[b + 1]]] = b
    assert got.tolist() == want


@pytest.mark.parametrize("lens", RAGGED + [np.random.default_rng(1).integers(0, 5000, 3000)])
def test_bins_invariants(lens):
    lens = np.asarray(lens, dtype=np.int64)
    rp = rowptr_of(lens)
    cnt, off, rows = oracle.row_bins(rp)
    m = lens.size
    assert cnt.sum() == m and off[0] == 0 and off[-1] == m
    assert np.array_equal(off[1:] - off[:-1], cnt)
    assert np.array_equal(np.sort(rows), np.arange(m))
    for b in range(oracle.NUM_BINS):
        seg = rows[off[b]:off[b + 1]]
        assert np.all(np.diff(seg) > 0)                   # ascending row id inside the bin
        L = lens[seg]
        if b == 0:
            assert np.all(L == 0)
        else:                                             # 2^(b-2) < len <= 2^(b-1)
            assert np.all(L <= 2 ** (b - 1)) and np.all(2 * L > 2 ** (b - 1))


def test_bins_closed_form_of_structured_workloads():
    g = 24
    cnt, _, _ = oracle.row_bins(w.laplace2d(g).rowptr)        # lengths 3 (4 corners), 4 (edges), 5 (interior)
    assert cnt[3] == 4 + 4 * (g - 2) and cnt[4] == (g - 2) ** 2 and cnt.sum() == g * g
    cnt, _, _ = oracle.row_bins(w.uniform_rows(512, 512, 16).rowptr)
    assert cnt[5] == 512
    g = 10
    cnt, _, _ = oracle.row_bins(w.stencil27(g).rowptr)        # 8 corners (len 8), edges 12, faces 18, interior 27
    assert cnt[4] == 8 and cnt[5] == 12 * (g - 2) and cnt[6] == 6 * (g - 2) ** 2 + (g - 2) ** 3
    cnt, _, _ = oracle.row_bins(w.block_clustered(2048).rowptr)
    assert cnt[8] == 2048                                      # 128 = 2^7 -> bin 8


def test_row_stats():
    assert oracle.row_stats(rowptr_of([])) == {"min_len": 0, "max_len": 0, "n_empty": 0}
    assert oracle.row_stats(rowptr_of([4, 0, 9, 0, 2])) == {"min_len": 0, "max_len": 9, "n_empty": 2}
    assert oracle.row_stats(rowptr_of([3, 3])) == {"min_len": 3, "max_len": 3, "n_empty": 0}
    assert oracle.row_stats(rowptr_of([1, 0, 1, 1, 7])) == {"min_len": 0, "max_len": 7, "n_empty": 1}   # a row of one entry is not empty
    assert oracle.row_stats(rowptr_of([1, 1])) == {"min_len": 1, "max_len": 1, "n_empty": 0}
    for lens in RAGGED[1:]:                                    # against numpy's own reductions
        a = np.asarray(lens)
        assert oracle.row_stats(rowptr_of(lens)) == {"min_len": int(a.min()), "max_len": int(a.max()), "n_empty": int((a == 0).sum())}


# ------------------------------------------------------------------ row blocks
def test_row_blocks_handworked(hand):
    h = hand["row_blocks"]
    assert oracle.row_blocks(rowptr_of(h["lens"]), h["block_nnz"], h["rows_max"]).tolist() == h["boundaries"]


@pytest.mark.parametrize("lens", RAGGED + [np.random.default_rng(2).integers(0, 300, 5000)])
@pytest.mark.parametrize("block_nnz,rows_max", [(2048, 256), (6, 3), (1, 1), (64, 1000)])
def test_row_blocks_invariants(lens, block_nnz, rows_max):
    lens = np.asarray(lens, dtype=np.int64)
    m = lens.size
    rp = rowptr_of(lens)
    rb = oracle.row_blocks(rp, block_nnz, rows_max)
    assert rb[0] == 0 and rb[-1] == m
    if m == 0:
        assert rb.tolist() == [0]
        return
    assert np.all(np.diff(rb) > 0)
    for b in range(rb.size - 1):
        s, e = int(rb[b]), int(rb[b + 1])
        held = int(rp[e] - rp[s])
        assert e - s <= rows_max
        assert held <= block_nnz or e - s == 1
        if e < m:                                         # maximal: the next row would break a limit
            assert e - s == rows_max or held + lens[e] > block_nnz


def test_row_blocks_closed_form_counts():
    assert oracle.row_blocks(w.uniform_rows(4096, 4096, 16).rowptr, 2048, 256).size - 1 == 32
    g = 64                                                # 5 entries a row at most: the row cap binds
    assert oracle.row_blocks(w.laplace2d(g).rowptr, 2048, 256).size - 1 == g * g // 256
    assert oracle.row_blocks(w.block_clustered(4096).rowptr, 2048, 256).size - 1 == 4096 // 16


# ------------------------------------------------------------------ merge path
def test_merge_path_handworked(hand):
    h = hand["merge_path"]
    rp = np.array(h["rowptr"], dtype=np.int32)
    for ipc, want in h["splits"].items():
        r, z = oracle.merge_path(rp, int(ipc))
        assert r.tolist() == want["row"] and z.tolist() == want["nz"], ipc


def merge_split_by_definition(rp, d):
    """Smallest i in [max(0,d-nnz), min(d,m)] that is min(d,m) or has rowptr[i+1] > d-i-1."""
    m, nnz = rp.size - 1, int(rp[-1])
    hi = min(d, m)
    for i in range(max(0, d - nnz), hi + 1):
        if i == hi or rp[i + 1] > d - i - 1:
            return i, d - i
    raise AssertionError


@pytest.mark.parametrize("lens", RAGGED + [np.random.default_rng(3).integers(0, 40, 300)])
@pytest.mark.parametrize("ipc", [1, 2, 7, 64, 4096])
def test_merge_path_invariants_and_diagonal_search(lens, ipc):
    rp = rowptr_of(lens)
    m, nnz = rp.size - 1, int(rp[-1])
    T = m + nnz
    r, z = oracle.merge_path(rp, ipc)
    P = math.ceil(T / ipc)
    assert r.size == P + 1 == z.size
    assert r[0] == 0 and z[0] == 0 and r[-1] == m and z[-1] == nnz
    assert np.all(np.diff(r) >= 0) and np.all(np.diff(z) >= 0)
    for p in range(P + 1):
        d = min(p * ipc, T)
        assert r[p] + z[p] == d
        if r[p] < m:
            assert rp[r[p]] <= z[p] <= rp[r[p] + 1]
        assert (int(r[p]), int(z[p])) == merge_split_by_definition(rp, d)


# ------------------------------------------------------------------ default tile shape
def test_default_tile_shape():
    """Worked by hand from the rule: small matrices (1024, 64); else 256/G rows with G the team
    size for the mean length, entries = rows * mean rounded up to 8, clamped to [2048, 8192]."""
    assert oracle.tile_shape(0, 0) == (1024, 64)
    assert oracle.tile_shape(4096, 65536) == (1024, 64)                    # <= 2^20 entries
    assert oracle.tile_shape(1048576, 5238784) == (2048, 256)              # mean 5: G 1, 256*5 = 1280 -> 2048
    assert oracle.tile_shape(2097152, 55742968) == (3456, 128)             # mean 27: G 2, 128*27 = 3456
    assert oracle.tile_shape(1000000, 128000000) == (4096, 32)             # mean 128: G 8, 32*128
    assert oracle.tile_shape(4000000, 31913584) == (2048, 256)             # mean 8: G 1
    assert oracle.tile_shape(1000, 3000000) == (8192, 4)                   # mean 3000: G 64, 4*3000 -> 8192
    assert oracle.tile_shape(100000, 1700000) == (2176, 128)               # mean 17: 16*1 < 17 -> G 2, 128*17 = 2176


# ------------------------------------------------------------------ plan
def test_plan_rule():
    assert oracle.plan(0, 0, 0, 2048) == 1
    assert oracle.plan(10, 0, 0, 2048) == 1
    assert oracle.plan(10, 100, 2048, 2048) == 4
    assert oracle.plan(10, 5000, 2049, 2048) == 5
    assert [oracle.vector_lanes(1, k) for k in (1, 8, 9, 16, 17, 27, 128, 129, 255, 257, 100000)] == \
        [2, 2, 2, 2, 4, 4, 16, 32, 32, 64, 64]
    assert oracle.vector_lanes(0, 0) == 2


# ---- x windows of row blocks ------------------------------------------------------------
def test_x_windows_handworked(hand):
    h = hand["x_windows"]
    rp, ci = np.array(h["rowptr"], np.int32), np.array(h["colidx"], np.int32)
    for c in h["cases"]:
        nv, xv_ptr, xv_start, lidx = oracle.x_windows(rp, ci, np.array(c["row_blocks"], np.int32), c["block_nnz"],
                                                      c["vec_elems"])
        assert nv.tolist() == c["nv"]
        assert xv_ptr.tolist() == np.concatenate([[0], np.cumsum(c["nv"])]).tolist()
        assert xv_start.tolist() == c["xv_start"]
        assert lidx.tolist() == c["lidx"]


def check_x_windows(p, block_nnz, rows_max, ve):
    """Properties that pin the window outputs without restating how they are built: laying the
    block's vectors out back to back and indexing with lidx gives back x[colidx]; the vectors of
    a block are aligned, distinct, ascending and all used."""
    rb = oracle.row_blocks(p.rowptr, block_nnz, rows_max)
    nv, xv_ptr, xv_start, lidx = oracle.x_windows(p.rowptr, p.colidx, rb, block_nnz, ve)
    assert nv.size == rb.size - 1 and xv_ptr[-1] == xv_start.size
    assert np.all(xv_start % ve == 0)
    xpad = np.concatenate([np.arange(p.n, dtype=np.int64), np.full(ve, -1, np.int64)])  # x[i] = i; padding never used
    for b in range(rb.size - 1):
        k0, k1 = p.rowptr[rb[b]], p.rowptr[rb[b + 1]]
        if k1 - k0 > block_nnz:
            assert nv[b] == 0 and not lidx[k0:k1].any()
            continue
        starts = xv_start[xv_ptr[b]:xv_ptr[b + 1]].astype(np.int64)
        assert np.all(np.diff(starts) > 0)
        buf = xpad[(starts[:, None] + np.arange(ve)[None, :]).ravel()] if starts.size else np.zeros(0, np.int64)
        li = lidx[k0:k1].astype(np.int64)
        assert np.array_equal(buf[li], p.colidx[k0:k1])
        assert np.array_equal(np.unique(li // ve), np.arange(nv[b]))  # no vector without an entry
    return nv


@pytest.mark.parametrize("ve", [4, 8])
def test_x_windows_properties(ve):
    import workloads as w
    cases = [(w.laplace2d(40), 256, 64), (w.stencil27(9), 512, 32), (w.uniform_rows(300, 300, 16), 128, 16),
             (w.powerlaw(2000), 64, 64), (w.block_clustered(500, blocks_per_row=16, width=8), 1024, 8)]
    cases += [(p, 8, 4) for p in w.tiny_adversarial()] + [(p, 8192, 1024) for p in w.tiny_adversarial()]
    for p, bn, rm in cases:
        check_x_windows(p, bn, rm, ve)


def test_x_windows_closed_form_counts():
    """5-point stencil on a g x g grid, blocks of whole grid lines: an interior block of L lines
    touches the columns of L+2 consecutive lines, one contiguous range."""
    import workloads as w
    g, ve = 64, 4
    p = w.laplace2d(g)
    rb = np.arange(0, g * g + 1, 2 * g, dtype=np.int32)  # two grid lines per block
    nv, _, xv_start, _ = oracle.x_windows(p.rowptr, p.colidx, rb, 1 << 20, ve)
    assert nv[0] == 3 * g // ve and nv[-1] == 3 * g // ve
    assert np.all(nv[1:-1] == 4 * g // ve)
    assert xv_start[: nv[0]].tolist() == list(range(0, 3 * g, ve))


def test_window_choice_rule():
    assert oracle.window_choice([10, 10], 80)
    assert not oracle.window_choice([10, 11], 80)          # 4 * 2 blocks * 11 slots > 80 entries
    assert not oracle.window_choice([1025, 0], 1 << 20)    # a block's vectors exceed the buffer
    assert oracle.window_choice([1024, 0], 1 << 20)
    assert not oracle.window_choice([], 0)
    assert not oracle.window_choice([1, 100], 500)         # the stride is the largest count: 4 * 2 * 100 > 500
    assert oracle.window_choice([1, 100], 800)


# ---- column blocks ----------------------------------------------------------------------
def test_column_blocks_handworked(hand):
    """rowptr [0,3,5,9], columns [1,9,17 | 8,3 | 40,16,2,41], width 16: block 0 holds columns 0..15
    (entries 0,1 of row 0; 3,4 of row 1; 7 of row 2), block 1 columns 16..31 (entry 2; entry 6),
    block 2 columns 32..47 (entries 5, 8)."""
    h = hand["x_windows"]
    rp, ci = np.array(h["rowptr"], np.int32), np.array(h["colidx"], np.int32)
    ptr, row, col, src = oracle.column_blocks(3, 42, rp, ci, 16)
    assert ptr.tolist() == [0, 5, 7, 9]
    assert src.tolist() == [0, 1, 3, 4, 7, 2, 6, 5, 8]
    assert row.tolist() == [0, 0, 1, 1, 2, 0, 2, 2, 2]
    assert col.tolist() == [1, 9, 8, 3, 2, 1, 0, 8, 9]


@pytest.mark.parametrize("width", [1, 7, 64, 1 << 20])
def test_column_blocks_properties(width):
    import workloads as w
    for p in [w.uniform_rows(200, 300, 9), w.powerlaw(1500), w.from_row_lengths([6] * 50, 40, allow_dup=True, sort_cols=False)] + w.tiny_adversarial():
        if (p.n + width - 1) // width > 5000:
            continue
        ptr, row, col, src = oracle.column_blocks(p.m, p.n, p.rowptr, p.colidx, width)
        C = ptr.size - 1
        assert ptr[0] == 0 and ptr[-1] == p.nnz and np.all(np.diff(ptr) >= 0)
        assert np.array_equal(np.sort(src), np.arange(p.nnz))                       # a permutation of the entries
        rows_of = np.repeat(np.arange(p.m, dtype=np.int32), np.diff(p.rowptr))
        assert np.array_equal(row, rows_of[src])
        blk = np.repeat(np.arange(C), np.diff(ptr))
        assert np.array_equal(col + blk * width, p.colidx[src]) and np.all((0 <= col) & (col < width))
        for b in range(C):
            assert np.all(np.diff(src[ptr[b]:ptr[b + 1]]) > 0)                       # original order kept inside a block


def test_column_block_choice_rule():
    assert oracle.column_block_width("f32") == 1 << 20 and oracle.column_block_width("bf16") == 1 << 21
    big = 1 << 22

    def f(n, nnz, dtype, plan, vectors=None, entries=None):      # scattered unless said otherwise: a vector per entry
        return oracle.column_block_choice(n, nnz, dtype, plan, nnz if vectors is None else vectors, nnz if entries is None else entries)
    assert f(4_000_000, 31_000_000, "f32", 5)
    assert f(4_000_000, 31_000_000, "f32", 4)
    assert not f(4_000_000, 31_000_000, "f32", 6)          # windows already keep x on chip
    assert not f(2 << 20, 31_000_000, "f32", 5)            # x is exactly two blocks
    assert f((2 << 20) + 1, big, "f32", 5)
    assert not f((2 << 20) + 1, big - 1, "f32", 5)         # too few entries to pay for the passes
    assert not f(4_000_000, 31_000_000, "bf16", 5)         # 8 MB of bf16 x: two blocks
    assert not f(17 << 20, 1 << 30, "f32", 5)              # more than 16 blocks
    assert f(4_000_000, 31_000_000, "f32", 5, vectors=3000, entries=4000)        # scattered columns only
    assert not f(4_000_000, 31_000_000, "f32", 5, vectors=2999, entries=4000)
    assert not f(4_000_000, 31_000_000, "f32", 5, vectors=-1, entries=-2)        # not counted: no


def test_lidx_grouped_handworked():
    rowptr = np.array([0, 8, 16, 20], np.int32)                       # 20 entries: two whole groups and a tail of four
    blocks = np.array([0, 1, 3], np.int32)                            # blocks start at entries 0 and 8
    run = np.arange(8)
    good = np.concatenate([run + 3, run + 40, [9, 9, 0, 1]])          # consecutive, from any start; the tail does not matter
    assert oracle.lidx_grouped(rowptr, blocks, good)
    for k in (1, 7, 9, 15):
        bad = good.copy()
        bad[k] += 1
        assert not oracle.lidx_grouped(rowptr, blocks, bad), k
    assert not oracle.lidx_grouped(np.array([0, 4, 16, 20], np.int32), blocks, good)         # a block starting at entry 4
    assert oracle.lidx_grouped(np.array([0, 4, 16, 20], np.int32), np.array([0, 2, 3], np.int32), good)   # ... unless no block starts there
    assert not oracle.lidx_grouped(np.array([0, 7], np.int32), np.array([0, 1], np.int32), np.arange(7))  # no whole group
    assert oracle.lidx_grouped(np.array([0, 8], np.int32), np.array([0, 1], np.int32), np.arange(8))


# ------------------------------------------------------------------ the two-pass layout
TP_ARRAYS = ("tp_row", "tp_nz", "tp_piece_c", "tp_piece_g", "tp_chunk_g", "tp_col", "tp_src", "tp_from", "tp_pos")


# ---- row patterns of the window positions --------------------------------------------------
def test_row_patterns_handworked(golden_dir):
    h = json.loads((golden_dir / "row_patterns_handworked.json").read_text())
    rp, li, rb = np.array(h["rowptr"], np.int32), np.array(h["lidx"], np.uint16), np.array(h["row_blocks"], np.int32)
    for c in h["cases"]:
        got = oracle.row_patterns(rp, rb, li, c["block_nnz"], c["max_runs"], c["max_len"])
        for name in ("n_runs", "run_rows", "run_len", "run_base", "run_stride", "pat_ptr", "pat"):
            assert got[name].tolist() == c[name], (name, c["why"])
        assert got["covered"] == c["covered"]


def check_row_patterns(rowptr, rb, lidx, block_nnz, max_runs, max_len):
    """Pins the run tables without restating how they are found: expanding them gives back lidx exactly; neighbouring
    runs cannot be merged; a block left out really breaks one of the four conditions (counted by brute force)."""
    got = oracle.row_patterns(rowptr, rb, lidx, block_nnz, max_runs, max_len)
    covered = 0
    for b in range(rb.size - 1):
        rows = np.arange(rb[b], rb[b + 1])
        lens = (rowptr[rows + 1] - rowptr[rows]).astype(np.int64)
        entries = int(lens.sum())
        R = int(got["n_runs"][b])
        table = got["pat"][got["pat_ptr"][b]:got["pat_ptr"][b + 1]].astype(np.int64)
        if R:
            covered += entries
            assert entries <= block_nnz and (lens <= max_len).all()
            assert got["run_rows"][b, :R].sum() == rows.size and (got["run_rows"][b, :R] > 0).all()
            assert not got["run_rows"][b, R:].any() and table.size == got["run_len"][b, :R].sum()
            i, t = 0, 0
            firsts = []
            for r in range(R):
                n, L, B, S = (int(got[name][b, r]) for name in ("run_rows", "run_len", "run_base", "run_stride"))
                firsts.append(i)
                for q in range(n):
                    k = rowptr[rows[i + q]]
                    assert lens[i + q] == L
                    assert np.array_equal(lidx[k:k + L].astype(np.int64), B + q * S + table[t:t + L]), (b, r, q)
                if n == 1:
                    assert S == 0
                i += n
                t += L
            # maximal: the first row of run r + 1 could not have stayed in run r
            for r in range(R - 1):
                n, L, S = (int(got[name][b, r]) for name in ("run_rows", "run_len", "run_stride"))
                L2 = int(got["run_len"][b, r + 1])
                same_rel = L2 == L and np.array_equal(table[sum(got["run_len"][b, :r]):][:L], table[sum(got["run_len"][b, :r + 1]):][:L])
                if same_rel:
                    step = (int(got["run_base"][b, r + 1]) - (int(got["run_base"][b, r]) + (n - 1) * S)) if L else 0
                    assert n >= 2 and step != S, (b, r)
        else:
            assert not any(got[name][b].any() for name in ("run_rows", "run_len", "run_base", "run_stride")) and table.size == 0
            # brute force: count the maximal runs straight from lidx
            bases = [int(lidx[rowptr[i]]) if rowptr[i + 1] > rowptr[i] else 0 for i in rows]
            rels = [tuple(int(v) - bases[j] for v in lidx[rowptr[i]:rowptr[i + 1]]) for j, i in enumerate(rows)]
            runs, in_run, stride = 0, 0, 0
            for j in range(rows.size):
                if in_run and rels[j] == rels[j - 1] and (in_run == 1 or bases[j] - bases[j - 1] == stride):
                    stride = bases[j] - bases[j - 1]
                    in_run += 1
                else:
                    runs, in_run, stride = runs + 1, 1, 0
            negative = any(v < 0 for rel in rels for v in rel)
            assert entries > block_nnz or (lens > max_len).any() or negative or runs > max_runs, b
    assert covered == got["covered"]
    return got


def test_row_patterns_properties():
    cases = [(w.laplace2d(40), 256, 64), (w.stencil27(9), 512, 32), (w.stencil27(6, dtype="f32"), 162, 6),
             (w.block_clustered(300, blocks_per_row=4, width=8), 1024, 8), (w.uniform_rows(300, 300, 16), 128, 16),
             (w.banded_random(400, 30, 5), 256, 64)]
    cases += [(p, 64, 8) for p in w.tiny_adversarial()] + [(p, 8192, 1024) for p in w.tiny_adversarial()]
    some = 0
    for p, bn, rm in cases:
        rb = oracle.row_blocks(p.rowptr, bn, rm)
        _, _, _, lidx = oracle.x_windows(p.rowptr, p.colidx, rb, bn, 8 if p.dtype == "bf16" else 4)
        for max_runs, max_len in ((4, 64), (2, 5), (1, 27)):
            some += check_row_patterns(p.rowptr, rb, lidx, bn, max_runs, max_len)["n_runs"].astype(bool).sum()
    assert some > 100


def test_row_patterns_closed_form_on_the_stencils():
    """Blocks that are whole grid lines (or aligned halves of one): every row of a line's interior has the positions of
    its left neighbour plus one, the rows at the two ends of a line have patterns of their own."""
    g = 32
    p = w.laplace2d(g)
    rb = np.arange(0, g * g + 1, g // 2, dtype=np.int32)           # half a grid line per block
    _, _, _, lidx = oracle.x_windows(p.rowptr, p.colidx, rb, 1 << 20, 4)
    got = oracle.row_patterns(p.rowptr, rb, lidx, 1 << 20)
    assert got["n_runs"].tolist() == [2] * (2 * g) and got["covered"] == p.nnz
    left, right = got["run_rows"][0::2], got["run_rows"][1::2]
    assert (left[:, :2] == [1, g // 2 - 1]).all() and (right[:, :2] == [g // 2 - 1, 1]).all()
    assert (got["run_stride"][0::2, 1] == 1).all() and (got["run_stride"][1::2, 0] == 1).all()
    assert got["run_len"][2, :2].tolist() == [4, 5] and got["run_len"][0, :2].tolist() == [3, 4]   # interior line, top line
    g = 8
    p = w.stencil27(g)
    rb = np.arange(0, g ** 3 + 1, g, dtype=np.int32)               # one grid line per block
    _, _, _, lidx = oracle.x_windows(p.rowptr, p.colidx, rb, 1 << 20, 8)
    got = oracle.row_patterns(p.rowptr, rb, lidx, 1 << 20)
    assert (got["n_runs"] == 3).all() and (got["run_rows"][:, :3] == [1, g - 2, 1]).all() and (got["run_stride"][:, 1] == 1).all()
    # block g + 1 is the line iy = 1, iz = 1: in the interior of the grid
    assert got["run_len"][g + 1, :3].tolist() == [18, 27, 18] and got["run_len"][0, :3].tolist() == [8, 12, 8]
    # nine neighbouring lines of g columns each sit back to back in the window: an entry (line q, dx) is at q*g + dx + 1 past the base
    assert got["pat"][got["pat_ptr"][g + 1] + 18:][:27].tolist() == [q * g + d for q in range(9) for d in range(3)]


def test_pattern_choice_rule():
    assert oracle.pattern_choice(10, 5) and not oracle.pattern_choice(11, 5)
    assert oracle.pattern_choice(10, 10) and not oracle.pattern_choice(0, 0) and not oracle.pattern_choice(10, 0)



def test_merge_path_snapped_handworked(golden_dir):
    for g in json.loads((golden_dir / "merge_path_snapped_handworked.json").read_text())["cases"]:
        rowptr = np.array(g["rowptr"], np.int32)
        row, nz = oracle.merge_path_snapped(rowptr, g["ipc"], g["snap"])
        assert row.tolist() == g["row"] and nz.tolist() == g["nz"], g["_note"]
        row, nz = oracle.merge_path_snapped(rowptr, g["ipc"], 0)
        assert row.tolist() == g["plain_row"] and nz.tolist() == g["plain_nz"]
        mr, mz = oracle.merge_path(rowptr, g["ipc"])
        assert mr.tolist() == g["plain_row"] and mz.tolist() == g["plain_nz"]


@pytest.mark.parametrize("ipc,snap", [(16, 4), (64, 63), (256, 32), (8192, 512), (5, 0)])
def test_merge_path_snapped_properties(ipc, snap):
    """From the splits alone: they start at (0, 0) and end at (m, nnz), move forward, no chunk is longer than ipc steps, only
    the last is shorter than ipc - snap + 1, a row of at most snap entries is never cut, a longer one is cut exactly where
    the count of steps says; snap = 0 is the plain merge path."""
    for p in (w.powerlaw(3000, n=900), w.uniform_rows(500, 4000, 7), w.from_row_lengths([0, 0, 900, 1, 0, 77, 3000, 0, 5, 5, 5], 3001, seed=5),
              w.from_row_lengths([0, 0, 0], 10), w.from_row_lengths([snap + 1] * 40 if snap else [3] * 40, 5000, seed=6),
              w.from_row_lengths([max(snap, 1)] * 60, 5000, seed=7)):
        rp = p.rowptr.astype(np.int64)
        row, nz = oracle.merge_path_snapped(p.rowptr, ipc, snap)
        assert (row[0], nz[0]) == (0, 0) and (row[-1], nz[-1]) == (p.m, p.nnz)
        d = row.astype(np.int64) + nz
        steps = np.diff(d)
        assert np.all(steps > 0) and np.all(steps <= ipc) and np.all(steps[:-1] >= ipc - snap)
        assert np.all(np.diff(row) >= 0) and np.all(np.diff(nz) >= 0)
        inner = np.arange(1, row.size - 1)
        r, k = row[inner].astype(np.int64), nz[inner].astype(np.int64)
        assert np.all(rp[r] <= k) and np.all(k <= rp[np.minimum(r + 1, p.m)])            # a split lies in the row after the finished ones
        cut = (rp[r] < k)                                                                  # entries of row r taken, row r not finished
        lens = rp[np.minimum(r + 1, p.m)] - rp[r]
        assert np.all(lens[cut] > snap)                                                    # short rows are whole
        assert np.all(steps[:-1][cut[: steps.size - 1]] == ipc) if cut.size else True      # a kept cut sits exactly ipc steps on
        if snap == 0:
            mr, mz = oracle.merge_path(p.rowptr, ipc)
            assert np.array_equal(row, mr) and np.array_equal(nz, mz)


def test_two_phase_layout_handworked(golden_dir):
    both = json.loads((golden_dir / "two_phase_handworked.json").read_text())
    for g in (both, both["second"]):
        L = oracle.two_phase_layout(g["m"], g["n"], np.array(g["rowptr"], np.int32), np.array(g["colidx"], np.int32),
                                    g["shift"], g["items"], g["piece_groups"], snap=0)
        for k in ("C", "P", "S", "Q"):
            assert L[k] == g[k], k
        for k in TP_ARRAYS:
            assert L[k].tolist() == g[k], k


@pytest.mark.parametrize("shift,items,piece_groups", [(3, 16, 4), (6, 256, 32), (14, 8192, 8192), (1, 5, 1)])
def test_two_phase_layout_properties(shift, items, piece_groups):
    """What the layout promises, checked from the arrays alone, and the product taken through it."""
    rng = np.random.default_rng(shift)
    for p in (w.powerlaw(2500, n=700), w.uniform_rows(300, 5000, 9), w.from_row_lengths([0, 0, 900, 1, 0, 77, 3000, 0], 3001, seed=5),
              w.from_row_lengths([0, 0, 0], 10)):
        snap = items // 4
        L = oracle.two_phase_layout(p.m, p.n, p.rowptr, p.colidx, shift, items, piece_groups, snap=snap)
        C, P, S = L["C"], L["P"], L["S"]
        mp_row, mp_nz = oracle.merge_path_snapped(p.rowptr, items, snap)
        assert np.array_equal(L["tp_row"], mp_row) and np.array_equal(L["tp_nz"], mp_nz)
        assert C == -(-p.n // (1 << shift)) and S % 4 == 0 and S >= p.nnz
        src, col, pos, frm = L["tp_src"], L["tp_col"], L["tp_pos"], L["tp_from"]
        real = src >= 0
        assert np.array_equal(np.sort(src[real]), np.arange(p.nnz))                       # every entry exactly once
        assert np.all(col[~real] == (1 << shift)) and np.all(col[real] < (1 << shift))
        # multiply order: pieces name the column block; with it the column comes back
        g_of_slot = np.arange(S) // 4
        piece_of_group = np.searchsorted(L["tp_piece_g"], np.arange(S // 4), side="right") - 1
        assert L["tp_piece_g"][0] == 0 and L["tp_piece_g"][-1] == S // 4 and np.all(np.diff(L["tp_piece_g"]) > 0)
        assert np.all(np.diff(L["tp_piece_g"]) <= piece_groups) and np.all(np.diff(L["tp_piece_c"]) >= 0)
        for c in range(C):                                                                 # a block's pieces: fewest, cut evenly
            mine = np.flatnonzero(L["tp_piece_c"] == c)
            if mine.size:
                sizes = np.diff(L["tp_piece_g"])[mine]
                groups = int(sizes.sum())
                assert mine.size == -(-groups // piece_groups)
                assert np.all(sizes[:-1] == -(-groups // mine.size)) and 0 < sizes[-1] <= -(-groups // mine.size)
        cblk = L["tp_piece_c"][piece_of_group][g_of_slot] if S else np.zeros(0, np.int64)
        assert np.array_equal(cblk[real].astype(np.int64) * (1 << shift) + col[real], p.colidx[src[real]])
        # tiles: the chunk of an entry, from its CSR position
        chunk = np.searchsorted(mp_nz, src[real], side="right") - 1
        key = cblk[real].astype(np.int64) * P + chunk
        assert np.all(np.diff(key) >= 0)                                                   # tiles in (c, p) order
        assert np.all((np.diff(src[real]) > 0) | (np.diff(key) > 0))                       # CSR order inside a tile
        # a group of four never straddles two tiles, and padding only closes a tile
        r4 = real.reshape(-1, 4)
        assert np.all(r4[:, 0]) and np.all(r4[:, :-1] >= r4[:, 1:])
        k4 = np.full(S, -1, np.int64)
        k4[real] = key
        k4 = k4.reshape(-1, 4)
        assert np.all((k4 == k4[:, :1]) | (k4 == -1))
        full = r4.all(axis=1)
        assert np.all(full[:-1] | (k4[:-1, 0] != k4[1:, 0]))                               # a padded group is its tile's last
        # reduce order: group for group the same entries, at their position within the chunk
        assert np.array_equal(np.sort(frm), np.arange(S // 4))                             # every group fetched exactly once
        pos4, src4 = pos.reshape(-1, 4), src.reshape(-1, 4)
        moved = src4[frm].astype(np.int64)                                                 # CSR position of every reduce-order slot
        chunk_of_group = np.searchsorted(L["tp_chunk_g"], np.arange(S // 4), side="right") - 1
        assert L["tp_chunk_g"][0] == 0 and L["tp_chunk_g"][-1] == S // 4
        want_pos = np.where(moved >= 0, moved - mp_nz[chunk_of_group][:, None], 0xFFFF)
        assert np.array_equal(pos4, want_pos)
        moved_c = cblk.reshape(-1, 4)[:, 0][frm].astype(np.int64) if S else np.zeros(0, np.int64)
        same_chunk = np.diff(chunk_of_group) == 0
        assert np.all(np.diff(moved_c)[same_chunk] >= 0)                                   # inside a chunk: by column block
        # the product taken through the layout is the product
        x = rng.uniform(-1, 1, p.n)
        a = rng.uniform(-1, 1, p.nnz)
        xs = np.concatenate((x, np.zeros(2 << shift)))
        prod1 = np.where(real, np.where(real, a[np.maximum(src, 0)], 0.0) * xs[np.where(real, cblk.astype(np.int64) * (1 << shift) + col, p.n)], 0.0)
        prod2 = prod1.reshape(-1, 4)[frm]                                                  # the reduce pass fetches group by group
        lds = np.zeros(p.nnz + 1)
        sel = pos4 != 0xFFFF
        lds[(mp_nz[chunk_of_group][:, None] + pos4)[sel]] = prod2[sel]
        y = np.add.reduceat(np.concatenate((lds[:p.nnz], [0.0])), np.minimum(p.rowptr[:-1], p.nnz))[: p.m] if p.m else np.zeros(0)
        y = np.where(np.diff(p.rowptr) > 0, y, 0.0)
        rows = np.repeat(np.arange(p.m), np.diff(p.rowptr))
        want = np.bincount(rows, weights=a * x[p.colidx], minlength=p.m)
        assert np.allclose(y, want, rtol=0, atol=1e-12)


def test_two_phase_piece_groups_worked_by_hand():
    f = oracle.two_phase_piece_groups
    # one block of 10 groups, 4 workgroups resident, 2 rounds wanted: 10 >= 2 * 4 * 1, so at most 8 pieces: t = 2 (5 pieces; t = 1: 10)
    assert f([10], 4, waves=2, cap=100, floor=1) == 2
    # pieces of 3 or more: 10 < 2 * 4 * 3, one round of 4: ceil(10 / 3) = 4 pieces, ceil(10 / 2) = 5
    assert f([10], 4, waves=2, cap=100, floor=3) == 3
    # 20 groups: fewer than 2 * 4 * 3, so one round of 4 although pieces of 3 would fill two: ceil(20 / 5) = 4, ceil(20 / 4) = 5
    assert f([20], 4, waves=2, cap=100, floor=3) == 5
    # the cap forces more rounds: three blocks of 5, cap 2: 9 pieces at best, 4 resident -> 3 rounds (12); t = 1 gives 15, t = 2 gives 9
    assert f([5, 5, 5], 4, waves=1, cap=2, floor=1) == 2
    # a small matrix: any t fills less than the device; the floor is the answer
    assert f([100], 512, waves=2, cap=16384, floor=2048) == 2048
    # thirty blocks of 130 000 groups and one of 64 000, 512 resident, two rounds (1024 pieces): 33 pieces per large block
    # need t >= 3940 (130000 / 3940 = 32.99..), the small one then takes 17: 1007; 34 per large block (t >= 3824) would
    # make 1020 + 17 = 1037
    assert f([130_000] * 30 + [64_000], 512) == 3940
    # empty blocks count for nothing
    assert f([0, 10, 0], 4, waves=2, cap=100, floor=1) == 2


@pytest.mark.parametrize("seed", range(6))
def test_two_phase_piece_groups_is_the_smallest_cap_that_fits(seed):
    rng = np.random.default_rng(seed)
    groups = rng.integers(0, 40_000, size=int(rng.integers(1, 40)))
    resident, waves, cap, floor = int(rng.integers(2, 64)), int(rng.integers(1, 4)), 4096, 16
    t = oracle.two_phase_piece_groups(groups, resident, waves, cap, floor)
    pieces = lambda c: int(np.sum(-(-groups // c)))
    k = waves if groups.sum() >= waves * resident * floor else 1
    while pieces(cap) > k * resident:
        k += 1
    assert floor <= t <= cap and pieces(t) <= k * resident
    assert t == floor or pieces(t - 1) > k * resident
    assert k == 1 or (k == waves and groups.sum() >= waves * resident * floor) or pieces(cap) > (k - 1) * resident


def test_grouped_two_phase_choice_boundaries():
    """Config 5 (1 M rows and columns, 16 M groups, bf16: x of 2.0 MB, 31 column blocks of 4096 groups, 2076 chunks) is
    taken; each condition is then moved across its threshold, the figures worked by hand."""
    m = n = 1_000_000
    nnz = 128_000_000
    E = nnz                                                               # all entries counted
    yes = lambda **k: oracle.grouped_two_phase_choice(**{**dict(m=m, n=n, nnz=nnz, dtype="bf16", plan=5, group_aligned=1,
                                                              vectors=15_970_000, entries=E), **k})
    assert yes() == 1 and yes(plan=4) == 1
    assert yes(plan=6) == 0 and yes(plan=1) == 0 and yes(group_aligned=0) == 0
    assert yes(vectors=-1) == 0
    assert yes(vectors=12_000_000) == 1 and yes(vectors=11_999_999) == 0   # 4 * 8 * v >= 3 * E  <=>  v >= 12 000 000
    assert yes(dtype="f32", vectors=24_000_000) == 1 and yes(dtype="f32", vectors=23_999_999) == 0   # vectors of four
    assert yes(n=524_288) == 1 and yes(n=524_287) == 0                    # x of exactly 1 MiB in bf16
    assert yes(dtype="f32", n=262_144, vectors=24_000_000) == 1 and yes(dtype="f32", n=262_143, vectors=24_000_000) == 0
    ng = 3 * 2 ** 21                                                       # 6 291 456 groups
    assert yes(nnz=8 * ng, entries=8 * ng, vectors=ng) == 1 and yes(nnz=8 * ng - 8, entries=8 * ng - 8, vectors=ng) == 0
    # tiles of eight groups: C = ceil(ceil(n / 8) / 4096), P = ceil((m + ng) / 8192); n = 64 M columns -> C = 1954,
    # m = 1 M, ng = 16 M -> P = 2076: C * P = 4 056 504 tiles, 8 * that = 32 452 032 > 16 M groups
    assert yes(n=64_000_000) == 0
    # n = 32 M -> C = 977: 8 * 977 * 2076 = 16 226 016 > 16 000 000; n = 31 M -> C = 947: 8 * 947 * 2076 = 15 727 776 <= 16 M
    assert yes(n=32_000_000) == 0 and yes(n=31_000_000) == 1


def test_two_phase_choice_rule():
    def f(m, n, nnz, dtype, plan, vectors=None, entries=None):       # scattered unless said otherwise: a vector per entry
        return oracle.two_phase_choice(m, n, nnz, dtype, plan, nnz if vectors is None else vectors, nnz if entries is None else entries)
    M = 4_000_000
    assert f(M, M, 31_913_584, "f32", 5)                       # 245 column blocks x 4384 chunks, 30 entries a tile
    assert f(M, M, 31_913_584, "f32", 4)
    assert not f(M, M, 31_913_584, "f32", 6)                   # only from the adaptive or the merge plan
    assert not f(M, (1 << 16) - 1, 31_913_584, "f32", 5)       # x smaller than 256 KiB: 2^16 floats ...
    assert f(M, 1 << 16, 31_913_584, "f32", 5)
    assert not f(M, (1 << 17) - 1, 31_913_584, "bf16", 5) and f(M, 1 << 17, 31_913_584, "bf16", 5)   # ... 2^17 bf16
    assert not f(M, M, 3 * (1 << 21) - 1, "f32", 5) and f(1 << 20, M, 3 * (1 << 21), "f32", 5)
    # tiles of fewer than eight entries on average: C = 245, P = ceil((m + nnz) / 8192)
    nnz = 8 * 245 * 4000
    assert f(8192 * 4000 - nnz, M, nnz, "f32", 5) and not f(8192 * 4000 - nnz + 1, M, nnz, "f32", 5)
    # more than 2^24 tiles: 512 column blocks x 2^15 chunks is the most
    assert f((1 << 27) - (1 << 20), 1 << 23, (1 << 27) + (1 << 20), "f32", 5)
    assert not f((1 << 27) - (1 << 20) + 1, 1 << 23, (1 << 27) + (1 << 20), "f32", 5)
    assert not f(1 << 27, 1 << 27, 1 << 30, "f32", 5)
    # scattered columns only: three distinct x vectors per four counted entries, or more
    assert f(M, M, 31_913_584, "f32", 5, vectors=3_000_000, entries=4_000_000)
    assert not f(M, M, 31_913_584, "f32", 5, vectors=2_999_999, entries=4_000_000)
    assert f(M, M, 31_913_584, "f32", 5, vectors=0, entries=0)            # nothing but over-long rows: no evidence of clustering
    assert not f(M, M, 31_913_584, "f32", 5, vectors=-1, entries=0)       # not counted: no,
    assert not f(M, M, 31_913_584, "f32", 5, vectors=-1, entries=-2)      # whatever the second figure says


def test_scatter_counts_handworked():
    """Three row blocks of a 6-row matrix, block_nnz 4: entries 3, 7 (one over-long row: not counted), 2."""
    rowptr = np.array([0, 1, 3, 10, 10, 11, 12], np.int32)
    row_blocks = np.array([0, 2, 3, 6], np.int32)
    assert oracle.scatter_counts(rowptr, row_blocks, 4, [2, 0, 1]) == (3, 5)
    assert oracle.scatter_counts(rowptr, row_blocks, 7, [2, 5, 1]) == (8, 12)
    assert oracle.scatter_counts(rowptr, np.array([0, 6], np.int32), 4, [0]) == (0, 0)


# ---- sliced ELL re-layout -------------------------------------------------------------------
def test_sell_handworked(golden_dir):
    h = json.loads((golden_dir / "sell_handworked.json").read_text())
    rp, ci = np.array(h["rowptr"], np.int32), np.array(h["colidx"], np.int32)
    for c in h["cases"]:
        got = oracle.sell_layout(h["m"], rp, ci, c["height"])
        for name in ("sell_ptr", "sell_col", "sell_src"):
            assert got[name].tolist() == c[name], (name, c["why"])
        assert got["S"] == c["sell_ptr"][-1] and got["ns"] == len(c["sell_ptr"]) - 1


def check_sell(p, height):
    """Pins the layout without restating the loops: every stored entry sits in exactly one slot, at the place the
    definition gives its (row, entry number); everything else is padding; the slices are as wide as their longest row
    and no wider; and the product taken slot by slot through the layout is the pinned CSR oracle's, bit for bit."""
    L = oracle.sell_layout(p.m, p.rowptr, p.colidx, height)
    ptr, col, src = L["sell_ptr"].astype(np.int64), L["sell_col"], L["sell_src"]
    lens = np.diff(p.rowptr).astype(np.int64)
    assert L["ns"] == -(-p.m // height) and ptr[0] == 0 and ptr[-1] == L["S"] == col.size == src.size
    live = src >= 0
    assert np.array_equal(np.sort(src[live]), np.arange(p.nnz))           # every entry once
    assert np.array_equal(col[live], p.colidx[src[live]]) and (col[~live] == -1).all()
    slot = np.flatnonzero(live)
    s = np.searchsorted(ptr, slot, side="right") - 1                        # the slot's slice
    off = slot - ptr[s]
    row, j = s * height + off % height, off // height
    assert (row < p.m).all() and np.array_equal(src[live], p.rowptr[row] + j) and (j < lens[row]).all()
    widths = np.diff(ptr) // height
    assert (np.diff(ptr) % height == 0).all()
    padded = np.concatenate([lens, np.zeros(L["ns"] * height - p.m, np.int64)]).reshape(L["ns"], height)
    assert np.array_equal(widths, padded.max(axis=1) if p.m else widths)
    # the product through the layout, entries of a row in their slot order (= storage order), in double
    y_ref, _ = oracle.spmv_problem(p)
    wide = (lambda a: a.astype(np.float64)) if p.dtype == "f32" else (lambda a: w.bf16_bits_to_f32(a).astype(np.float64))
    vals, x = wide(p.vals), wide(p.x)
    y = np.zeros(p.m)
    for k in range(int(widths.max()) if widths.size else 0):               # entry number k of every row, slice by slice
        for sl in np.flatnonzero(widths > k):
            base = ptr[sl] + k * height
            e = src[base:base + height]
            rows = sl * height + np.flatnonzero(e >= 0)
            y[rows] += vals[e[e >= 0]] * x[col[base:base + height][e >= 0]]
    y0 = p.y0.astype(np.float64) if p.y0 is not None else 0.0
    assert np.array_equal(np.float64(np.float32(p.alpha)) * y + (np.float64(np.float32(p.beta)) * y0 if p.beta != 0 else 0.0), y_ref)


@pytest.mark.parametrize("height", [1, 4, 64])
def test_sell_properties_on_random_and_degenerate_matrices(height):
    rng = np.random.default_rng(height)
    for lens, n in ((rng.integers(0, 9, 300), 50), (np.zeros(70, np.int64), 5), ([0, 0, 40, 0, 1], 64), ([3], 3), ([], 7),
                    (np.minimum(w.powerlaw_lengths(rng, 500, cap=300), 200), 200)):
        p = w.from_row_lengths(np.asarray(lens, np.int64), n, seed=3, dtype="f32", alpha=-1.5, beta=0.5)
        check_sell(p, height)
    check_sell(w.from_row_lengths(rng.integers(0, 20, 129), 100, seed=4, dtype="bf16"), height)


def test_sell_closed_forms():
    # rows of one length L: every slice is L wide, nothing is padded but the rows past m
    p = w.uniform_rows(1000, 1000, 7)
    L = oracle.sell_layout(p.m, p.rowptr, p.colidx, 64)
    assert L["ns"] == 16 and L["S"] == 16 * 64 * 7 and np.array_equal(L["sell_ptr"], np.arange(17) * 64 * 7)
    assert (L["sell_src"] >= 0).sum() == 7000 and (L["sell_src"][-64 * 7:].reshape(7, 64)[:, 40:] == -1).all()
    # height 1: the slices are the rows and the layout is CSR itself
    q = w.from_row_lengths(np.array([3, 0, 5, 1]), 9, seed=1)
    L1 = oracle.sell_layout(q.m, q.rowptr, q.colidx, 1)
    assert np.array_equal(L1["sell_ptr"], q.rowptr) and np.array_equal(L1["sell_col"], q.colidx)
    assert np.array_equal(L1["sell_src"], np.arange(q.nnz))
    # one slice as tall as the matrix: the ELL layout of App. C task 14, transposed (ELL is stored row by row)
    width = int(np.diff(q.rowptr).max())
    ell = w.to_ell(q)[1].reshape(q.m, width)
    Lm = oracle.sell_layout(q.m, q.rowptr, q.colidx, q.m)
    assert np.array_equal(Lm["sell_col"].reshape(width, q.m), ell.T)


# ---- group-aligned matrices and the two-pass plan on groups --------------------------------------
def test_csr_groups_handworked():
    """Worked by hand from the definition (width 4 for readability): rows of 4 and 8 entries, groups (8..11), (0..3), (4..7)."""
    rp = np.array([0, 4, 12], np.int32)
    good = np.array([8, 9, 10, 11, 0, 1, 2, 3, 4, 5, 6, 7], np.int32)
    assert oracle.csr_groups(2, rp, good, 4) == 1
    rg, cg = oracle.group_matrix(2, rp, good, 4)
    assert rg.tolist() == [0, 1, 3] and cg.tolist() == [2, 0, 1]
    assert oracle.csr_groups(2, rp, good, 2) == 1                         # pairs (8,9) (10,11) (0,1) .. are aligned runs of two as well
    assert oracle.csr_groups(2, rp, good, 8) == 0                         # the first row holds half a group of eight
    for k, c, why in ((0, 9, "a group that does not start at a multiple of four"), (2, 11, "a repeated column"),
                      (11, 8, "last column of the last group off"), (5, 2, "a gap inside a group")):
        bad = good.copy()
        bad[k] = c
        if k == 0:
            bad[:4] = [9, 10, 11, 12]                                     # consecutive, but starting at 9
        assert oracle.csr_groups(2, rp, bad, 4) == 0, why
    assert oracle.csr_groups(2, np.array([0, 6, 12], np.int32), good, 4) == 0   # a row starting inside a group
    assert oracle.csr_groups(2, np.array([0, 0, 0], np.int32), np.zeros(0, np.int32), 4) == 0  # no entries: nothing to group
    assert oracle.csr_groups(3, np.array([0, 4, 4, 12], np.int32), good, 4) == 1              # an empty row between


def test_csr_groups_on_the_generators():
    p = w.block_clustered(m=500, n=4096)
    assert oracle.csr_groups(p.m, p.rowptr, p.colidx) == 1
    rg, cg = oracle.group_matrix(p.m, p.rowptr, p.colidx)
    assert np.array_equal(rg, p.rowptr // 8) and np.array_equal(np.repeat(cg, 8) * 8 + np.tile(np.arange(8), cg.size), p.colidx)
    for q in (w.uniform_rows(64, 64, 8), w.laplace2d(16), w.from_row_lengths(np.full(10, 8), 100, seed=1)):
        assert oracle.csr_groups(q.m, q.rowptr, q.colidx) == 0
