"""Properties of the seeded input generators (shapes, counts, distributions of the five configs)."""
import hashlib

import numpy as np
import pytest

import workloads as w


def check_structure(p, sorted_distinct=True):
    assert p.rowptr.dtype == np.int32 and p.colidx.dtype == np.int32
    assert p.rowptr[0] == 0 and np.all(np.diff(p.rowptr) >= 0) and p.rowptr[-1] == p.colidx.size == p.vals.size
    assert p.colidx.min(initial=0) >= 0 and p.colidx.max(initial=0) < p.n
    assert p.vals.dtype == (np.float32 if p.dtype == "f32" else np.uint16) == p.x.dtype
    assert p.x.size == p.n
    if sorted_distinct and p.nnz:
        d = np.diff(p.colidx.astype(np.int64))
        starts = np.zeros(p.nnz, bool)
        lens = np.diff(p.rowptr)
        starts[p.rowptr[:-1][lens > 0]] = True
        assert np.all((d > 0) | starts[1:])


def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -2.5, 0.0, 3.140625], dtype=np.float32)
    b = w.f32_to_bf16_bits(f)
    back = w.bf16_bits_to_f32(b)
    # ties: 1+2^-8 is halfway between 1 and 1+2^-7 -> even mantissa (1.0); 1+3*2^-8 -> 1+2^-6
    assert back.tolist() == [1.0, 1.0, 1.015625, 1.0, 1.015625, -2.5, 0.0, 3.140625]
    r = np.random.default_rng(0).uniform(-4, 4, 10000).astype(np.float32)
    rb = w.bf16_bits_to_f32(w.f32_to_bf16_bits(r))
    assert np.all(np.abs(rb - r) <= np.abs(r) * 2.0 ** -8)


def test_cfg1_full():
    p = w.config(1)
    check_structure(p)
    assert (p.m, p.n, p.nnz) == (4096, 4096, 65536) and np.all(np.diff(p.rowptr) == 16)
    assert p.algorithmic_bytes() == 573444 and (p.alpha, p.beta) == (1.0, 0.0)
    assert -1 <= p.vals.min() and p.vals.max() < 1 and abs(p.vals.mean()) < 0.02


def test_cfg2_full():
    p = w.config(2)
    check_structure(p)
    assert (p.m, p.nnz) == (1048576, 5238784) and p.algorithmic_bytes() == 58687492
    assert np.bincount(np.diff(p.rowptr)).tolist() == [0, 0, 0, 4, 4088, 1044484]
    assert (p.alpha, p.beta) == (1.0, 0.5) and p.y0 is not None
    r = 5 * 1024 + 17
    s = p.rowptr[r]
    assert p.colidx[s:s + 5].tolist() == [r - 1024, r - 1, r, r + 1, r + 1024]
    assert p.vals[s:s + 5].tolist() == [-1, -1, 4, -1, -1]


def test_cfg3_scaled():
    g = 16
    p = w.stencil27(g)
    check_structure(p)
    assert p.nnz == (3 * g - 2) ** 3 and p.dtype == "bf16"
    lens = np.diff(p.rowptr)
    assert np.bincount(lens)[[8, 12, 18, 27]].tolist() == [8, 12 * (g - 2), 6 * (g - 2) ** 2, (g - 2) ** 3]
    rows = np.repeat(np.arange(p.m), lens)
    diag = p.colidx == rows
    assert diag.sum() == p.m and np.all(p.vals[diag] == 0x41D0)       # 26.0 in bf16
    off = w.bf16_bits_to_f32(p.vals[~diag])
    assert np.all(np.abs(off) <= 1.0)


def test_cfg4_scaled_distribution():
    p = w.powerlaw(400_000)
    check_structure(p)
    lens = np.diff(p.rowptr)
    assert lens.min() == 1 and lens.max() <= 200_000
    assert abs(np.minimum(lens, 20000).mean() - 7.9) < 0.25          # mean 8.0005 with a heavy tail
    frac = [(lens <= t).mean() for t in (4, 8, 16, 64)]
    assert np.allclose(frac, [0.66, 0.82, 0.92, 0.987], atol=0.01)
    q = w.powerlaw(200_000, literal=True)
    assert abs(np.minimum(np.diff(q.rowptr), 5000).mean() - 2.6) < 0.1


def test_cfg4_capped_row_is_distinct():
    # a row at the cap inside a much narrower matrix forces many redraws
    rng_lens = np.array([3, 20000, 1, 0, 7])
    p = w.from_row_lengths(rng_lens, 25000, seed=4)
    check_structure(p)


def test_cfg5_scaled():
    p = w.block_clustered(4096)
    check_structure(p)
    assert p.nnz == 4096 * 128 and np.all(np.diff(p.rowptr) == 128)
    c = p.colidx.reshape(4096, 16, 8)
    assert np.all(c[:, :, 0] % 8 == 0) and np.all(np.diff(c, axis=2) == 1)


def test_density_random_shape():
    p = w.density_random(1024, 2048, 0.01)
    check_structure(p)
    assert p.nnz == int(1024 * 2048 * 0.01)


def test_tiny_adversarial_structures():
    for p in w.tiny_adversarial():
        check_structure(p, sorted_distinct=p.name != "dup_unsorted")


def test_same_seed_same_bits():
    def h(p):
        s = hashlib.sha256()
        for a in (p.rowptr, p.colidx, p.vals, p.x):
            s.update(a.tobytes())
        return s.hexdigest()
    assert h(w.config(4, 1 / 100)) == h(w.config(4, 1 / 100))
    assert h(w.powerlaw(1000, seed=1)) != h(w.powerlaw(1000, seed=2))
