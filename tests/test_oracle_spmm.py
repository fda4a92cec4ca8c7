"""Pins of the SpMM oracle (oracle/spmm_oracle.cpp): values fixed by a hand-worked example, by a
dense matrix product, by the already pinned SpMV oracle (K = 1) and by algebraic identities."""
import json

import numpy as np
import pytest

import oracle
import workloads as w


def dense_of(p):
    A = np.zeros((p.m, p.n), dtype=np.float64)
    for i in range(p.m):
        for e in range(p.rowptr[i], p.rowptr[i + 1]):
            A[i, p.colidx[e]] += np.float64(p.vals[e])   # repeated columns add up
    return A


def rand_B(n, K, seed=0):
    return np.random.default_rng(seed).uniform(-1, 1, (n, K)).astype(np.float32)


def test_handworked(golden_dir):
    h = json.loads((golden_dir / "spmm_3x4x2_handworked.json").read_text())
    rp, ci = np.array(h["rowptr"], np.int32), np.array(h["colidx"], np.int32)
    va, B, C0 = np.array(h["vals"], np.float32), np.array(h["B"], np.float32), np.array(h["C0"], np.float32)
    C, S = oracle.spmm_csr(h["m"], h["n"], rp, ci, va, B)
    assert np.array_equal(C, np.array(h["AB"])) and np.array_equal(S, np.array(h["S"]))
    C, S = oracle.spmm_csr(h["m"], h["n"], rp, ci, va, B, C0, h["alpha"], h["beta"])
    assert np.array_equal(C, np.array(h["C"])) and np.array_equal(S, np.array(h["S"]))
    # beta == 0 must not read C0: NaN there does not propagate
    C, _ = oracle.spmm_csr(h["m"], h["n"], rp, ci, va, B, np.full((3, 2), np.nan, np.float32), 1.0, 0.0)
    assert np.array_equal(C, np.array(h["AB"]))


@pytest.mark.parametrize("K", [1, 3, 16, 37])
def test_against_dense_product(K):
    for p in [w.uniform_rows(40, 30, 5), w.powerlaw(60), w.laplace2d(6)] + w.tiny_adversarial()[:5]:
        B = rand_B(p.n, K, seed=K)
        C0 = rand_B(p.m, K, seed=K + 100)
        C, S = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, B, C0, 1.5, -0.25)
        A = dense_of(p)
        want = 1.5 * (A @ B.astype(np.float64)) - 0.25 * C0.astype(np.float64)
        assert np.allclose(C, want, rtol=0, atol=1e-12 * (1 + np.abs(want).max())), p.name
        assert np.all(S + 1e-300 >= np.abs(A @ B.astype(np.float64)) - 1e-12)   # triangle inequality


def test_single_column_is_the_spmv_oracle():
    p = w.powerlaw(300)
    B = p.x.reshape(-1, 1).copy()
    y0 = p.y0 if p.y0 is not None else np.zeros(p.m, np.float32)
    C, S = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, B, y0.reshape(-1, 1).copy(), 0.75, 2.0)
    y, Sy = oracle.spmv_csr("f32", p.m, p.n, p.rowptr, p.colidx, p.vals, p.x, y0, 0.75, 2.0)
    assert np.array_equal(C[:, 0], y) and np.array_equal(S[:, 0], Sy)


def test_identity_matrix_copies_B_and_slices_use_ldb():
    n, K = 17, 9
    rp = np.arange(n + 1, dtype=np.int32)
    ci = np.arange(n, dtype=np.int32)
    va = np.ones(n, np.float32)
    wide = rand_B(n, 3 * K, seed=5)
    B = wide[:, K:2 * K]                       # a column slice: leading dimension 3K
    C, S = oracle.spmm_csr(n, n, rp, ci, va, B)
    assert np.array_equal(C, B.astype(np.float64)) and np.array_equal(S, np.abs(B.astype(np.float64)))
    # a permutation matrix permutes the rows of B
    perm = np.random.default_rng(2).permutation(n).astype(np.int32)
    C, _ = oracle.spmm_csr(n, n, rp, perm, va, B)
    assert np.array_equal(C, B[perm].astype(np.float64))


def test_linearity_in_B_and_rejects_bad_columns():
    p = w.uniform_rows(50, 64, 7)
    B1, B2 = rand_B(p.n, 5, 1), rand_B(p.n, 5, 2)
    # exactly representable combination: B1 + 2*B2 computed in float64 then checked on the double results
    C1, _ = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, B1)
    C2, _ = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, B2)
    B3 = (B1.astype(np.float64) + 2 * B2.astype(np.float64)).astype(np.float32)
    exact = B3.astype(np.float64) == B1.astype(np.float64) + 2 * B2.astype(np.float64)
    C3, _ = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, B3)
    cols_exact = exact.all(axis=0)
    assert np.allclose(C3[:, cols_exact], (C1 + 2 * C2)[:, cols_exact], rtol=0, atol=1e-12)
    bad = p.colidx.copy()
    bad[3] = p.n
    with pytest.raises(ValueError):
        oracle.spmm_csr(p.m, p.n, p.rowptr, bad, p.vals, B1)


def rowptr_from(lens):
    return np.concatenate(([0], np.cumsum(np.asarray(lens, dtype=np.int64)))).astype(np.int32)


def test_row_order_handworked(golden_dir):
    h = json.loads((golden_dir / "spmm_row_order_handworked.json").read_text())
    assert np.array_equal(oracle.spmm_row_order(rowptr_from(h["lens"])), np.array(h["one_window"], np.int32))
    assert np.array_equal(oracle.spmm_row_order(rowptr_from(h["lens"]), 11), np.array(h["one_window"], np.int32))
    assert np.array_equal(oracle.spmm_row_order(rowptr_from(h["lens"]), 4), np.array(h["windows_of_4"], np.int32))
    assert np.array_equal(oracle.spmm_row_order(rowptr_from(h["lens"]), 1), np.arange(11))
    assert oracle.spmm_row_order(rowptr_from([])).size == 0
    assert np.array_equal(oracle.spmm_row_order(rowptr_from([7])), [0])


@pytest.mark.parametrize("seed", range(6))
def test_row_order_defining_properties(seed):
    """A permutation of the rows; keys never increase along it; equal keys keep ascending row ids."""
    rng = np.random.default_rng(seed)
    m = int(rng.integers(1, 3000))
    lens = np.where(rng.random(m) < 0.05, rng.integers(200, 400, m), rng.poisson(rng.choice([1.5, 6, 20]), m))
    window = int(rng.choice([1, 7, 64, 4096]))
    rows = oracle.spmm_row_order(rowptr_from(lens), window)
    assert np.array_equal(np.sort(rows), np.arange(m))
    key = np.minimum(-(-lens[rows] // 4), 64)
    assert set(np.unique(key)) <= set(range(65)) and (key.max() == 64) == bool((lens > 252).any())
    for w0 in range(0, m, window):                     # every window holds its own rows, sorted
        part, kpart = rows[w0:w0 + window], key[w0:w0 + window]
        assert np.array_equal(np.sort(part), np.arange(w0, min(w0 + window, m)))
        assert np.all(np.diff(kpart) <= 0)
        assert np.all(np.diff(part)[np.diff(kpart) == 0] > 0)


def test_packed_copy_handworked(golden_dir):
    h = json.loads((golden_dir / "spmm_packed_handworked.json").read_text())
    rp = rowptr_from(h["lens"])
    nnz = int(rp[-1])
    colidx = ((7 * np.arange(nnz)) % 50).astype(np.int32)
    vals = (np.arange(nnz) + 1).astype(np.float32)
    rows = oracle.spmm_row_order(rp)
    assert rows.tolist() == h["rows"]
    desc, blocks = oracle.spmm_packed_layout(rp, rows)
    assert desc.tolist() == h["desc"] and blocks == h["blocks"]
    pcol, pval = oracle.spmm_pack(rp, colidx, vals, rows, desc)
    want_col, want_val = np.full(512, -1, np.int32), np.zeros(512, np.float32)
    for slot, k in h["live"]:
        want_col[slot], want_val[slot] = colidx[k], vals[k]
    assert np.array_equal(pcol, want_col) and np.array_equal(pval, want_val)
    assert not oracle.spmm_packed_choice(nnz, blocks)            # 512 slots for 23 entries
    assert oracle.spmm_packed_choice(256, 2) and not oracle.spmm_packed_choice(255, 2)
    assert not oracle.spmm_packed_choice(0, 0) and not oracle.spmm_packed_choice(2 ** 31, 2 ** 22 + 1)


@pytest.mark.parametrize("seed", range(5))
def test_packed_copy_holds_every_entry_once(seed):
    rng = np.random.default_rng(100 + seed)
    m = int(rng.integers(1, 400))
    lens = rng.poisson(rng.choice([2, 20.5, 70]), m)
    lens[rng.integers(0, m, 3)] = 0
    p = w.from_row_lengths(lens, 300, seed=seed, allow_dup=True)
    rows = oracle.spmm_row_order(p.rowptr, int(rng.choice([16, 64, 4096])))
    desc, blocks = oracle.spmm_packed_layout(p.rowptr, rows)
    pcol, pval = oracle.spmm_pack(p.rowptr, p.colidx, p.vals, rows, desc)
    assert pcol.size == blocks * 256 and desc[-2] == blocks and desc[-1] == 0
    live = pcol >= 0
    assert np.all(pval[~live] == 0) and np.all(pcol[~live] == -1) and live.sum() == p.nnz
    slot = np.flatnonzero(live)
    block, i = slot // 256, (slot % 256) // 16
    group = np.searchsorted(desc[0::2], block, side="right") - 1          # the group a block belongs to
    row = rows[16 * group + i]
    got = sorted(zip(row.tolist(), pcol[live].tolist(), pval[live].tolist()))
    want = sorted(zip(np.repeat(np.arange(m), lens).tolist(), p.colidx.tolist(), p.vals.tolist()))
    assert got == want
    # a group's steps: the quarter-rounded length of its longest row
    longest = np.array([lens[rows[16 * g:16 * g + 16]].max() for g in range((m + 15) // 16)])
    assert np.array_equal(desc[1:-2:2], -(-longest // 4)) and np.array_equal(np.diff(desc[0::2]), -(-longest // 16))


def test_packed_copy_entry_order_on_rows_with_every_residue_equally_often():
    """Rows that hold equally many columns of each residue modulo 4 (here: c consecutive quadruples of columns, in a
    shuffled storage order): the row at position p of the order then shows, at rank t, a column with
    (column - p) mod 4 == t mod 4 - so the 16 rows of a group ask for the four quarters of the banks in turn at every
    rank - and columns of one residue keep their storage order."""
    rng = np.random.default_rng(5)
    m, c = 40, 3
    rowptr = (np.arange(m + 1) * 4 * c).astype(np.int32)
    colidx = np.concatenate([rng.permutation(4 * c) + 4 * int(rng.integers(0, 10)) for _ in range(m)]).astype(np.int32)
    vals = np.arange(colidx.size, dtype=np.float32)                     # the value names the storage position
    rows = oracle.spmm_row_order(rowptr)
    assert rows.tolist() == list(range(m))                              # equal lengths: the order is the natural one
    desc, blocks = oracle.spmm_packed_layout(rowptr, rows)
    pcol, pval = oracle.spmm_pack(rowptr, colidx, vals, rows, desc)
    for p in range(m):
        g, i = divmod(p, 16)
        t = np.arange(4 * c)
        slot = ((desc[2 * g] + t // 16) * 64 + 4 * i + (t % 16) // 4) * 4 + t % 4
        assert np.array_equal((pcol[slot] - p) % 4, t % 4), p
        for r in range(4):                                              # one residue: storage order kept
            pos = pval[slot][pcol[slot] % 4 == r]
            assert np.all(np.diff(pos) > 0), (p, r)


# ---- bf16 storage --------------------------------------------------------------------------------
def test_bf16_handworked_and_against_the_pinned_oracles():
    """Values that bf16 holds exactly, worked by hand: A = [[1.5, 0, -2], [0, 0.25, 0]], B = [[2, -1], [4, 8], [0.5, 3]]
    gives A B = [[3 - 1, -1.5 - 6], [1, 2]] and S = [[3 + 1, 1.5 + 6], [1, 2]].  Then: one column against the pinned
    bf16 SpMV oracle, and any K against the pinned FP32 product on the widened numbers (widening is exact, so the two
    must agree bit for bit)."""
    bits = lambda a: w.f32_to_bf16_bits(np.asarray(a, np.float32))
    rp, ci = np.array([0, 2, 3], np.int32), np.array([0, 2, 1], np.int32)
    va, B = bits([1.5, -2.0, 0.25]), bits([[2, -1], [4, 8], [0.5, 3]])
    C, S = oracle.spmm_csr(2, 3, rp, ci, va, B)
    assert C.tolist() == [[2.0, -7.5], [1.0, 2.0]] and S.tolist() == [[4.0, 7.5], [1.0, 2.0]]
    C0 = np.array([[1, 2], [3, 4]], np.float32)
    C, _ = oracle.spmm_csr(2, 3, rp, ci, va, B, C0, 2.0, -0.5)
    assert C.tolist() == [[3.5, -16.0], [0.5, 2.0]]
    assert va.dtype == np.uint16 and va.tolist() == [0x3FC0, 0xC000, 0x3E80]      # 1.5, -2, 0.25 as bf16 bit patterns
    p = w.powerlaw(300, dtype="bf16")
    y0 = np.linspace(-1, 1, p.m, dtype=np.float32)
    C, S = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, p.x.reshape(-1, 1).copy(), y0.reshape(-1, 1).copy(), 0.75, 2.0)
    y, Sy = oracle.spmv_csr("bf16", p.m, p.n, p.rowptr, p.colidx, p.vals, p.x, y0, 0.75, 2.0)
    assert np.array_equal(C[:, 0], y) and np.array_equal(S[:, 0], Sy)
    Bb = bits(rand_B(p.n, 7, seed=3))
    wide = np.zeros((p.n, 20), np.uint16)
    wide[:, 5:12] = Bb                                                              # a column slice: ldb = 20
    C0 = rand_B(p.m, 7, seed=4)
    C16, S16 = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, p.vals, wide[:, 5:12], C0, -1.25, 0.5)
    C32, S32 = oracle.spmm_csr(p.m, p.n, p.rowptr, p.colidx, w.bf16_bits_to_f32(p.vals), w.bf16_bits_to_f32(Bb), C0, -1.25, 0.5)
    assert np.array_equal(C16, C32) and np.array_equal(S16, S32)
