"""Pins for the checker's sparse tensor-times-matrix route (mode-3 unfolding + row-wise product):
dense einsum on tiny tensors, with unordered and repeated coordinates."""
import numpy as np
import pytest

import oracle
from paper_2404_04541_amd import workloads as W


def tiny_tensor(shape, nnz, seed, duplicates):
    I, J, K = shape
    idx = np.arange(nnz, dtype=np.uint64)
    xi = W.rand_below(seed, 1, idx, I).astype(np.int32)
    xj = W.rand_below(seed, 2, idx, J).astype(np.int32)
    xk = W.rand_below(seed, 3, idx, K).astype(np.int32)
    if not duplicates:
        lin = (xi.astype(np.int64) * J + xj) * K + xk
        _, first = np.unique(lin, return_index=True)
        first.sort()
        xi, xj, xk = xi[first], xj[first], xk[first]
    vals = W.draw_values(xi.size, -1.0, 1.0, np.float64, seed, 4)
    return xi, xj, xk, vals


@pytest.mark.parametrize("shape,nnz,seed,dup", [((3, 4, 5), 20, 1, False), ((6, 2, 7), 60, 2, True), ((1, 1, 9), 5, 3, False),
                                                ((5, 5, 5), 0, 4, False), ((4, 6, 3), 200, 5, True)])
def test_ttm_against_dense_einsum(shape, nnz, seed, dup):
    I, J, K = shape
    L = 6
    xi, xj, xk, vals = tiny_tensor(shape, nnz, seed, dup)
    M = W.random_csr(K, L, 3, seed + 10)
    r = oracle.spttm_mode3(shape, xi, xj, xk, vals, M)
    X = np.zeros(shape); Xp = np.zeros(shape, dtype=np.int64)
    np.add.at(X, (xi, xj, xk), vals); np.add.at(Xp, (xi, xj, xk), 1)
    Md = M.to_dense(); Mp = (M.to_dense() != 0)
    Mp = np.zeros((K, L), dtype=np.int64)
    for k in range(K):
        Mp[k, M.colidx[M.rowptr[k]:M.rowptr[k + 1]]] += 1
    Y = np.einsum("ijk,kl->ijl", X, Md)
    Yp = np.einsum("ijk,kl->ijl", Xp, Mp)
    assert r.rowptr.size == I * J + 1 and int(r.ip.sum()) == int(Yp.sum())
    for i in range(I):
        for j in range(J):
            row = i * J + j
            cols = r.colidx[r.rowptr[row]:r.rowptr[row + 1]]
            assert np.array_equal(cols, np.nonzero(Yp[i, j])[0].astype(np.int32))
            got = r.values[r.rowptr[row]:r.rowptr[row + 1]]
            scale = r.absum[r.rowptr[row]:r.rowptr[row + 1]]
            assert np.all(np.abs(got - Y[i, j, cols]) <= 1e-13 * np.maximum(scale, 1e-300))


def test_unfolding_orders_by_row_then_column_and_keeps_repeats():
    rowptr, col, val = oracle.unfold_mode3((2, 2, 4), [1, 0, 1, 0, 1], [1, 0, 1, 1, 1], [3, 2, 0, 1, 3], [1.0, 2.0, 3.0, 4.0, 5.0])
    # rows: (0,0)->0, (0,1)->1, (1,0)->2, (1,1)->3
    assert rowptr.tolist() == [0, 1, 2, 2, 5]
    assert col.tolist() == [2, 1, 0, 3, 3]
    assert val.tolist() == [2.0, 4.0, 3.0, 1.0, 5.0]   # the two (1,1,3) entries stay in input order
    with pytest.raises(ValueError):
        oracle.unfold_mode3((2, 2, 4), [2], [0], [0], [1.0])


def test_unfolding_agrees_with_the_generator_on_distinct_coordinates():
    x = W.coo3_uniform((8, 8, 8), 100, 0, 40)
    a = W.unfold_mode3(x)
    rowptr, col, val = oracle.unfold_mode3(x.shape, x.i, x.j, x.k, x.values)
    assert np.array_equal(rowptr, a.rowptr) and np.array_equal(col, a.colidx) and np.array_equal(val, a.values)


# ---- every mode: X x_m M with the kept coordinates folded into the row (paper section 7.4) ----

EINSUM = {1: "ijk,il->ljk", 2: "ijk,jl->ilk", 3: "ijk,kl->ijl"}


@pytest.mark.parametrize("mode", [1, 2, 3])
@pytest.mark.parametrize("shape,nnz,seed,dup", [((3, 4, 5), 25, 11, False), ((6, 2, 7), 70, 12, True), ((2, 5, 1), 9, 13, True)])
def test_ttm_every_mode_against_dense_einsum(mode, shape, nnz, seed, dup):
    L = 4
    xi, xj, xk, vals = tiny_tensor(shape, nnz, seed, dup)
    M = W.random_csr(shape[mode - 1], L, 2, seed + 20)
    r = oracle.spttm(shape, mode, xi, xj, xk, vals, M)
    X = np.zeros(shape); Xp = np.zeros(shape, dtype=np.int64)
    np.add.at(X, (xi, xj, xk), vals); np.add.at(Xp, (xi, xj, xk), 1)
    Mp = np.zeros((M.rows, L), dtype=np.int64)
    for k in range(M.rows):
        Mp[k, M.colidx[M.rowptr[k]:M.rowptr[k + 1]]] += 1
    Y = np.einsum(EINSUM[mode], X, M.to_dense())
    Yp = np.einsum(EINSUM[mode], Xp, Mp)     # products landing on each output coordinate
    out_shape = list(shape); out_shape[mode - 1] = L
    yi, yj, yk = oracle.fold(out_shape, mode, r.rowptr, r.colidx)
    # structure: exactly the coordinates that receive at least one product, each once
    got = np.zeros(out_shape, dtype=np.int64)
    np.add.at(got, (yi, yj, yk), 1)
    assert np.array_equal(got, (Yp > 0).astype(np.int64))
    assert int(r.ip.sum()) == int(Yp.sum())
    assert np.all(np.abs(r.values - Y[yi, yj, yk]) <= 1e-13 * np.maximum(r.absum, 1e-300))
    # rows ascending in the fold of the kept coordinates, columns ascending inside a row
    rows = np.repeat(np.arange(r.rowptr.size - 1), np.diff(r.rowptr))
    key = rows.astype(np.int64) * L + r.colidx
    assert np.all(np.diff(key) > 0)


def test_unfolding_over_modes_one_and_two_by_hand():
    # X in 2 x 3 x 2 with entries (i,j,k): (1,2,0)=1, (0,0,1)=2, (1,0,1)=3, (0,2,0)=4, (1,2,0)=5 (a repeat)
    xi, xj, xk, v = [1, 0, 1, 0, 1], [2, 0, 0, 2, 2], [0, 1, 1, 0, 0], [1.0, 2.0, 3.0, 4.0, 5.0]
    # mode 1: row j*K + k (6 rows), column i
    rp, col, val = oracle.unfold((2, 3, 2), 1, xi, xj, xk, v)
    assert rp.tolist() == [0, 0, 2, 2, 2, 5, 5]
    assert col.tolist() == [0, 1, 0, 1, 1] and val.tolist() == [2.0, 3.0, 4.0, 1.0, 5.0]
    # mode 2: row i*K + k (4 rows), column j
    rp, col, val = oracle.unfold((2, 3, 2), 2, xi, xj, xk, v)
    assert rp.tolist() == [0, 1, 2, 4, 5]
    assert col.tolist() == [2, 0, 2, 2, 0] and val.tolist() == [4.0, 2.0, 1.0, 5.0, 3.0]
    # folding gives the coordinates back (in unfolded order)
    yi, yj, yk = oracle.fold((2, 3, 2), 2, rp, col)
    assert yi.tolist() == [0, 0, 1, 1, 1] and yj.tolist() == [2, 0, 2, 2, 0] and yk.tolist() == [0, 1, 0, 0, 1]
    with pytest.raises(ValueError):
        oracle.unfold((2, 3, 2), 4, xi, xj, xk, v)
