"""Generator checks: determinism, shapes, sortedness, the distributions' basic facts."""
import numpy as np

from paper_2404_04541_amd import workloads as W


def _canonical(c):
    assert c.rowptr.dtype == np.int64 and c.colidx.dtype == np.int32
    assert c.rowptr[0] == 0 and c.rowptr[-1] == c.colidx.size == c.values.size
    assert np.all(np.diff(c.rowptr) >= 0)
    if c.colidx.size:
        assert c.colidx.min() >= 0 and c.colidx.max() < c.cols
    r = np.repeat(np.arange(c.rows), np.diff(c.rowptr))
    key = r * c.cols + c.colidx
    assert np.all(np.diff(key) > 0), "columns ascending and unique in each row"


def test_counter_based_draws_are_pure_functions():
    i = np.arange(1000, dtype=np.uint64)
    a = W.rand_u64(3, 5, i)
    assert np.array_equal(a[::-1], W.rand_u64(3, 5, i[::-1]))
    assert not np.array_equal(a, W.rand_u64(3, 6, i)) and not np.array_equal(a, W.rand_u64(4, 5, i))
    u = W.rand_unit(0, 0, np.arange(200000, dtype=np.uint64))
    assert 0 <= u.min() and u.max() < 1 and abs(u.mean() - 0.5) < 5e-3
    b = W.rand_below(0, 1, np.arange(100000, dtype=np.uint64), 10)
    assert b.min() == 0 and b.max() == 9 and np.all(np.abs(np.bincount(b) - 10000) < 500)


def test_uniform_rows():
    a = W.uniform_rows(1000, 1000, 10, 0, 1)
    _canonical(a)
    assert np.all(np.diff(a.rowptr) == 10)
    assert -1 <= a.values.min() and a.values.max() < 1
    b = W.uniform_rows(1000, 1000, 10, 0, 1)
    assert np.array_equal(a.colidx, b.colidx) and np.array_equal(a.values, b.values)
    c = W.uniform_rows(50, 12, 12, 2, 3)  # dense rows force many redraws
    _canonical(c)


def test_stencil():
    for g in (3, 6):
        a = W.stencil27(g)
        _canonical(a)
        assert a.nnz == (3 * g - 2) ** 3
        p = W.stencil27(g, periodic=True)
        _canonical(p)
        assert p.nnz == 27 * g ** 3
    a = W.stencil27(6)
    # banded: |col - row| <= 1 + g + g*g
    r = np.repeat(np.arange(a.rows), np.diff(a.rowptr))
    assert np.abs(a.colidx - r).max() == 1 + 6 + 36
    assert (3 * 128 - 2) ** 3 == 55742968


def test_rmat_small():
    a = W.rmat(12, 16)
    _canonical(a)
    assert a.rows == 4096 and a.values.dtype == np.float32
    assert 0 <= a.values.min() and a.values.max() < 1
    assert 0.8 * 16 * 4096 < a.nnz <= 16 * 4096
    lens = np.diff(a.rowptr)
    # power law: heavy head at the low-index vertices, many empty rows
    assert lens[0] == lens.max() and lens.max() > 20 * lens.mean() and (lens == 0).sum() > 0.2 * a.rows
    colc = np.bincount(a.colidx, minlength=a.cols)
    assert colc[0] == colc.max()
    # quadrant probabilities: top row bit is 1 with probability c + d = 0.24
    top = (np.repeat(np.arange(a.rows), lens) >> 11) & 1
    assert abs(top.mean() - 0.24) < 0.03


def test_ttm_unfolding():
    x = W.coo3_uniform((16, 16, 16), 1000, 0)
    lin = (x.i.astype(np.int64) * 16 + x.j) * 16 + x.k
    assert np.unique(lin).size == 1000
    u = W.unfold_mode3(x)
    _canonical(u)
    assert (u.rows, u.cols, u.nnz) == (256, 16, 1000)
    d = np.zeros((16, 16, 16)); d[x.i, x.j, x.k] = x.values
    assert np.array_equal(u.to_dense(), d.reshape(256, 16))


def test_random_csr_variants():
    a = W.random_csr(100, 50, 5, 1)
    _canonical(a)
    assert (np.diff(a.rowptr) == 0).any()
    b = W.random_csr(100, 50, 5, 1, sort_rows=False, allow_duplicates=True)
    assert b.rowptr[-1] == b.colidx.size
    r = np.repeat(np.arange(b.rows), np.diff(b.rowptr))
    assert np.unique(r * 50 + b.colidx).size < b.nnz  # duplicates present


def test_small_instances_of_the_configs():
    a, b = W.config4(rows=4096, bcols=512)
    _canonical(a); _canonical(b)
    assert a.nnz == 8 * 4096 and b.nnz == 4 * 4096 and b.cols == 512
    a, m = W.config5(dim=32, nnz=5000)
    _canonical(a); _canonical(m)
    assert (a.rows, a.cols, a.nnz) == (1024, 32, 5000) and m.nnz == 16 * 32


def test_dedup_sweep_operands_follow_the_recipe():
    B, C = W.dedup_sweep(500, dense_elements=100_000, per_column=50)
    assert (B.rows, B.cols, C.rows, C.cols) == (200, 500, 500, 200)
    per_col = np.bincount(B.colidx, minlength=500)
    assert (per_col > 0).sum() == 50 and set(per_col[per_col > 0]) == {50}      # a tenth of the columns, 50 entries each
    assert np.array_equal(np.roll(B.to_dense().T, 1, axis=1), C.to_dense())       # second operand: B^T, columns rotated by one
    for M in (B, C):
        for i in range(M.rows):
            c = M.colidx[M.rowptr[i]:M.rowptr[i + 1]]
            assert np.all(np.diff(c) > 0)
