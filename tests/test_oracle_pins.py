"""Pins for the CPU checker: each test fixes it against something other than itself
(dense brute force, exact special products, closed forms, invariants, the paper's
printed dedup example, scipy as an unrelated implementation)."""
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2404_04541_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_force(A, B):
    """Dense triple loop; structure from the union of patterns (not from value != 0)."""
    m, k, n = A.rows, A.cols, B.cols
    Ad = np.zeros((m, k)); Ap = np.zeros((m, k), dtype=np.int64)
    Bd = np.zeros((k, n)); Bp = np.zeros((k, n), dtype=np.int64)
    for i in range(m):
        for p in range(A.rowptr[i], A.rowptr[i + 1]):
            Ad[i, A.colidx[p]] += float(A.values[p]); Ap[i, A.colidx[p]] += 1
    for i in range(k):
        for p in range(B.rowptr[i], B.rowptr[i + 1]):
            Bd[i, B.colidx[p]] += float(B.values[p]); Bp[i, B.colidx[p]] += 1
    Cd = np.zeros((m, n)); Cp = np.zeros((m, n), dtype=np.int64)
    for i in range(m):
        for kk in range(k):
            if Ap[i, kk]:
                for j in range(n):
                    if Bp[kk, j]:
                        Cd[i, j] += Ad[i, kk] * Bd[kk, j]
                        Cp[i, kk * 0 + j] += Ap[i, kk] * Bp[kk, j]
    return Cd, Cp


def check_against_dense(A, B, rtol=1e-13):
    r = oracle.spgemm(A, B)
    Cd, Cp = brute_force(A, B)
    assert r.rowptr[0] == 0 and r.rowptr.size == A.rows + 1
    assert int(r.ip.sum()) == int(Cp.sum())
    for i in range(A.rows):
        cols = r.colidx[r.rowptr[i]:r.rowptr[i + 1]]
        vals = r.values[r.rowptr[i]:r.rowptr[i + 1]]
        want = np.nonzero(Cp[i])[0]
        assert np.array_equal(cols, want.astype(np.int32)), f"row {i} structure"
        assert np.all(np.diff(cols) > 0)
        scale = r.absum[r.rowptr[i]:r.rowptr[i + 1]]
        assert np.all(np.abs(vals - Cd[i, want]) <= rtol * np.maximum(scale, 1e-300))


@pytest.mark.parametrize("m,k,n,da,db,seed", [
    (1, 1, 1, 1, 1, 0), (7, 5, 9, 2, 3, 1), (16, 16, 16, 4, 4, 2), (33, 64, 20, 6, 2, 3),
    (64, 64, 64, 8, 8, 4), (20, 40, 3, 10, 1, 5), (40, 3, 50, 1, 12, 6)])
def test_brute_force_sorted_unique(m, k, n, da, db, seed):
    A = W.random_csr(m, k, da, seed, 60)
    B = W.random_csr(k, n, db, seed, 70)
    check_against_dense(A, B)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_unsorted_and_duplicate_inputs(seed):
    A = W.random_csr(24, 18, 5, seed, 60, sort_rows=False, allow_duplicates=True)
    B = W.random_csr(18, 30, 6, seed, 70, sort_rows=False, allow_duplicates=True)
    # duplicates really occur in these operands
    assert A.nnz > np.unique(np.repeat(np.arange(A.rows), np.diff(A.rowptr)) * 1000 + A.colidx).size or seed != 0
    check_against_dense(A, B)


def test_explicit_zero_is_kept():
    # C[0,0] = 1*1 + 1*(-1) = 0 exactly: the coordinate must still be stored
    A = W.CSR(1, 2, np.array([0, 2]), np.array([0, 1], np.int32), np.array([1.0, 1.0]))
    B = W.CSR(2, 2, np.array([0, 1, 3]), np.array([0, 0, 1], np.int32), np.array([1.0, -1.0, 5.0]))
    r = oracle.spgemm(A, B)
    assert r.colidx.tolist() == [0, 1] and r.values.tolist() == [0.0, 5.0] and r.absum.tolist() == [2.0, 5.0]


def test_empty_operands_and_rows():
    Z = W.CSR(5, 4, np.zeros(6, np.int64), np.zeros(0, np.int32), np.zeros(0))
    B = W.random_csr(4, 6, 2, 0)
    r = oracle.spgemm(Z, B)
    assert r.rowptr.tolist() == [0] * 6 and r.colidx.size == 0
    A = W.random_csr(5, 4, 2, 1)
    Zb = W.CSR(4, 6, np.zeros(5, np.int64), np.zeros(0, np.int32), np.zeros(0))
    r = oracle.spgemm(A, Zb)
    assert r.rowptr.tolist() == [0] * 6 and int(r.ip.sum()) == 0
    E = W.CSR(0, 4, np.zeros(1, np.int64), np.zeros(0, np.int32), np.zeros(0))
    r = oracle.spgemm(E, B)
    assert r.rowptr.tolist() == [0]


def test_paper_dedup_example():
    ins, exp = [], None
    for line in open(os.path.join(GOLDEN, "dedup_example.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "insert":
            ins.append((int(t[1]), int(t[2]), float(t[3])))
        else:
            exp = (int(t[1]), int(t[2]), float(t[3]))
    # two products landing on (2,2): A[2,0]=A[2,1]=1, B[0,2]=3, B[1,2]=8
    assert [(i, j) for i, j, _ in ins] == [(2, 2), (2, 2)]
    A = W.CSR(3, 2, np.array([0, 0, 0, 2]), np.array([0, 1], np.int32), np.array([1.0, 1.0]))
    B = W.CSR(2, 3, np.array([0, 1, 2]), np.array([2, 2], np.int32), np.array([ins[0][2], ins[1][2]]))
    r = oracle.spgemm(A, B)
    assert r.rowptr.tolist() == [0, 0, 0, 1]
    assert (2, int(r.colidx[0]), float(r.values[0])) == exp


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_identity_products_bit_identical(dtype):
    A = W.random_csr(200, 200, 7, 3, dtype=dtype)
    I = W.identity(200, dtype)
    for r in (oracle.spgemm(I, A), oracle.spgemm(A, I)):
        assert np.array_equal(r.rowptr, A.rowptr)
        assert np.array_equal(r.colidx, A.colidx)
        assert np.array_equal(r.values, A.values.astype(np.float64))


def test_permutation_and_diagonal_products_exact():
    n = 150
    A = W.random_csr(n, n, 6, 9)
    P = W.permutation(n, 4)
    perm = P.colidx.astype(np.int64)
    Ad = A.to_dense()
    # (P A)[i,:] = A[perm[i],:]
    r = oracle.spgemm(P, A)
    for i in range(n):
        s = slice(A.rowptr[perm[i]], A.rowptr[perm[i] + 1])
        assert np.array_equal(r.colidx[r.rowptr[i]:r.rowptr[i + 1]], A.colidx[s])
        assert np.array_equal(r.values[r.rowptr[i]:r.rowptr[i + 1]], A.values[s])
    # (A P)[i, perm[k]] = A[i,k]: columns are relabelled and must come out re-sorted
    r = oracle.spgemm(A, P)
    for i in range(n):
        s = slice(A.rowptr[i], A.rowptr[i + 1])
        newc = perm[A.colidx[s]]
        o = np.argsort(newc)
        assert np.array_equal(r.colidx[r.rowptr[i]:r.rowptr[i + 1]], newc[o].astype(np.int32))
        assert np.array_equal(r.values[r.rowptr[i]:r.rowptr[i + 1]], A.values[s][o])
    # diagonal scalings: one product per entry, so exact
    d = W.draw_values(n, 0.5, 2.0, np.float64, 7, 99)
    D = W.CSR(n, n, np.arange(n + 1, dtype=np.int64), np.arange(n, dtype=np.int32), d)
    r = oracle.spgemm(D, A)
    assert np.array_equal(r.colidx, A.colidx)
    assert np.array_equal(r.values, np.repeat(d, np.diff(A.rowptr)) * A.values)
    r = oracle.spgemm(A, D)
    assert np.array_equal(r.colidx, A.colidx)
    assert np.array_equal(r.values, A.values * d[A.colidx])
    assert np.allclose(Ad @ np.diag(d), W.CSR(n, n, r.rowptr, r.colidx, r.values).to_dense(), rtol=0, atol=0)


def test_count_invariants():
    A = W.random_csr(300, 120, 8, 11)
    B = W.random_csr(120, 90, 10, 12)
    r = oracle.spgemm(A, B)
    blen = np.diff(B.rowptr)
    ip = np.zeros(A.rows, np.int64)
    np.add.at(ip, np.repeat(np.arange(A.rows), np.diff(A.rowptr)), blen[A.colidx])
    assert np.array_equal(r.ip, ip)
    assert np.all(r.cnt <= np.minimum(ip, B.cols))
    assert r.cnt.sum() <= ip.sum()
    # disjoint column blocks per B row => no two products share a column => equality
    k, w = 40, 5
    Bd = W.CSR(k, k * w, np.arange(k + 1, dtype=np.int64) * w, np.arange(k * w, dtype=np.int32), np.ones(k * w))
    A2 = W.random_csr(100, k, 6, 13)
    r2 = oracle.spgemm(A2, Bd)
    assert np.array_equal(r2.cnt, r2.ip) and np.array_equal(r2.cnt, np.diff(A2.rowptr) * w)


def _conv_count(g):
    """1-D count of paths i -> k -> j with |i-k|<=1, |k-j|<=1 on a clipped line of g points."""
    c = np.zeros((g, g), dtype=np.int64)
    for i in range(g):
        for k in range(max(0, i - 1), min(g, i + 2)):
            for j in range(max(0, k - 1), min(g, k + 2)):
                c[i, j] += 1
    return c


@pytest.mark.parametrize("g", [2, 3, 4, 5, 7, 10])
def test_stencil_closed_form_exhaustive(g):
    A = W.stencil27(g, ones=True)
    assert A.nnz == (3 * g - 2) ** 3
    r = oracle.spgemm(A, A)
    assert int(r.ip.sum()) == (9 * g - 10) ** 3
    assert int(r.cnt.sum()) == (5 * g - 6) ** 3
    c1 = _conv_count(g)
    # C[(x,y,z),(x',y',z')] = c1[x,x'] * c1[y,y'] * c1[z,z'] (row = x + g*(y + g*z))
    full = np.einsum("zw,yv,xu->zyxwvu", c1, c1, c1).reshape(g ** 3, g ** 3)
    got = W.CSR(g ** 3, g ** 3, r.rowptr, r.colidx, r.values).to_dense()
    assert np.array_equal(got, full.astype(np.float64))
    for i in range(g ** 3):
        assert np.array_equal(r.colidx[r.rowptr[i]:r.rowptr[i + 1]], np.nonzero(full[i])[0])


def test_stencil_closed_form_totals_larger_grids():
    for g, periodic in ((24, False), (16, True)):
        A = W.stencil27(g, ones=True, periodic=periodic)
        r = oracle.spgemm(A, A)
        n = g ** 3
        if periodic:
            assert (A.nnz, int(r.ip.sum()), int(r.cnt.sum())) == (27 * n, 729 * n, 125 * n)
            assert np.all(r.values[r.rowptr[0]:r.rowptr[1]] >= 1)
        else:
            assert (A.nnz, int(r.ip.sum()), int(r.cnt.sum())) == ((3 * g - 2) ** 3, (9 * g - 10) ** 3, (5 * g - 6) ** 3)
        assert float(r.values.sum()) == float(r.ip.sum())  # all-ones: every product is 1


@pytest.mark.parametrize("dtype,seed", [(np.float64, 0), (np.float32, 1)])
def test_against_scipy(dtype, seed):
    A = W.random_csr(500, 400, 9, seed, dtype=dtype)
    B = W.random_csr(400, 300, 7, seed + 10, dtype=dtype)
    r = oracle.spgemm(A, B)
    Sa = sp.csr_matrix((A.values.astype(np.float64), A.colidx, A.rowptr), shape=(A.rows, A.cols))
    Sb = sp.csr_matrix((B.values.astype(np.float64), B.colidx, B.rowptr), shape=(B.rows, B.cols))
    # structure from all-ones operands so that scipy cannot drop cancelled entries
    Pa = sp.csr_matrix((np.ones(A.nnz), A.colidx, A.rowptr), shape=(A.rows, A.cols))
    Pb = sp.csr_matrix((np.ones(B.nnz), B.colidx, B.rowptr), shape=(B.rows, B.cols))
    Pc = (Pa @ Pb).tocsr(); Pc.sort_indices()
    assert np.array_equal(r.rowptr, Pc.indptr.astype(np.int64))
    assert np.array_equal(r.colidx, Pc.indices.astype(np.int32))
    Sc = (Sa @ Sb).toarray()
    rows = np.repeat(np.arange(A.rows), r.cnt)
    assert np.all(np.abs(r.values - Sc[rows, r.colidx]) <= 1e-13 * r.absum)
    Sabs = (abs(Sa) @ abs(Sb)).toarray()
    assert np.allclose(r.absum, Sabs[rows, r.colidx], rtol=1e-13, atol=0)


def test_row_list_and_range_agree_with_whole():
    A = W.random_csr(120, 80, 6, 21)
    B = W.random_csr(80, 70, 5, 22)
    whole = oracle.spgemm(A, B)
    part = oracle.spgemm_rows(A.rowptr, A.colidx, A.values, B.rowptr, B.colidx, B.values, row_lo=30, row_hi=50)
    assert np.array_equal(part.colidx, whole.colidx[whole.rowptr[30]:whole.rowptr[50]])
    pick = np.array([5, 99, 5, 0], dtype=np.int64)
    lst = oracle.spgemm_rows(A.rowptr, A.colidx, A.values, B.rowptr, B.colidx, B.values, rows=pick)
    for t, i in enumerate(pick):
        assert np.array_equal(lst.values[lst.rowptr[t]:lst.rowptr[t + 1]], whole.values[whole.rowptr[i]:whole.rowptr[i + 1]])


def test_config1_sizes():
    a, b = W.config1()
    r = oracle.spgemm(a, b)
    assert int(r.ip.sum()) == 100000
    # expectation 1000*1000*(1-0.99**10) ~ 95618 (section "configs"): loose statistical window
    assert 95000 < int(r.cnt.sum()) < 96300
    assert r.cnt.max() <= 100
