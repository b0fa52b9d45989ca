"""Pins for the checker's outer-product route (k -> i -> j with a coordinate workspace, the paper's
sections 4.1 and 4.3): hand-written doubly compressed operands, dense brute force, agreement in
structure with the row-wise route, every accumulation capacity."""
import numpy as np
import pytest

import oracle
from oracle import outer
from paper_2404_04541_amd import workloads as W


def test_doubly_compressed_builders_by_hand():
    # A (3 x 4): row 0: (0,1)=1 (0,3)=2 ; row 1: empty ; row 2: (2,1)=3 (2,1)=4 (a repeat)
    A = W.CSR(3, 4, np.array([0, 2, 2, 4]), np.array([1, 3, 1, 1], np.int32), np.array([1.0, 2.0, 3.0, 4.0]))
    cols, ptr, rows, vals = outer.dcsc_from_csr(A)
    assert cols.tolist() == [1, 3] and ptr.tolist() == [0, 3, 4]
    assert rows.tolist() == [0, 2, 2, 0] and vals.tolist() == [1.0, 3.0, 4.0, 2.0]
    r, rp, c, v = outer.dcsr_from_csr(A)
    assert r.tolist() == [0, 2] and rp.tolist() == [0, 2, 4] and c.tolist() == [1, 3, 1, 1] and v.tolist() == [1.0, 2.0, 3.0, 4.0]


def test_insert_sort_merge_example_of_the_paper():
    # two components on coordinate (2,2) with values 3 and 8 are merged into 11 (section 4.2)
    A = W.CSR(3, 2, np.array([0, 0, 0, 2]), np.array([0, 1], np.int32), np.array([3.0, 8.0]))
    B = W.CSR(2, 3, np.array([0, 1, 2]), np.array([2, 2], np.int32), np.array([1.0, 1.0]))
    rp, col, val, _, n = outer.spgemm_outer(A, B)
    assert rp.tolist() == [0, 0, 0, 1] and col.tolist() == [2] and val.tolist() == [11.0] and n == 2


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("capacity", [1, 7, 1 << 16])
def test_outer_product_against_dense_and_rowwise(seed, capacity):
    u = W.rand_unit(seed, 950, np.arange(4, dtype=np.uint64))
    m, k, n = (1 + int(v * 40) for v in u[:3])
    A = W.random_csr(m, k, 1 + u[3] * 4, seed, 951, sort_rows=seed % 2 == 0, allow_duplicates=seed % 3 == 0)
    B = W.random_csr(k, n, 3, seed, 952, sort_rows=seed % 2 == 1, allow_duplicates=seed % 3 == 1)
    rp, col, val, absum, nprod = outer.spgemm_outer(A, B, capacity)
    # dense brute force: structure from the pattern product, values from the triple loop
    Ad, Bd = A.to_dense(), B.to_dense()
    Ap = np.zeros((m, k), np.int64); Bp = np.zeros((k, n), np.int64)
    np.add.at(Ap, (np.repeat(np.arange(m), np.diff(A.rowptr)), A.colidx), 1)
    np.add.at(Bp, (np.repeat(np.arange(k), np.diff(B.rowptr)), B.colidx), 1)
    Cp = Ap @ Bp
    assert nprod == int(Cp.sum())
    rows = np.repeat(np.arange(m), np.diff(rp))
    got = np.zeros((m, n), np.int64); np.add.at(got, (rows, col), 1)
    assert np.array_equal(got, (Cp > 0).astype(np.int64))
    assert np.all(np.diff(rows.astype(np.int64) * n + col) > 0)
    assert np.all(np.abs(val - (Ad @ Bd)[rows, col]) <= 1e-13 * np.maximum(absum, 1e-300))
    # the row-wise route gives the same structure
    ref = oracle.spgemm(A, B)
    assert np.array_equal(rp, ref.rowptr) and np.array_equal(col, ref.colidx)
    assert np.all(np.abs(val - ref.values) <= 1e-13 * np.maximum(ref.absum, 1e-300))


def test_outer_product_empty_rows_and_columns():
    # rows of A without entries, columns of A that meet empty rows of B, and the reverse
    A = W.CSR(4, 5, np.array([0, 2, 2, 3, 3]), np.array([0, 4, 2], np.int32), np.array([1.0, 2.0, 3.0]))
    B = W.CSR(5, 3, np.array([0, 1, 1, 1, 2, 2]), np.array([1, 0], np.int32), np.array([5.0, 7.0]))
    rp, col, val, _, n = outer.spgemm_outer(A, B)
    assert rp.tolist() == [0, 1, 1, 1, 1] and col.tolist() == [1] and val.tolist() == [5.0] and n == 1
    Z = W.CSR(4, 5, np.zeros(5, np.int64), np.zeros(0, np.int32), np.zeros(0))
    rp, col, val, _, n = outer.spgemm_outer(Z, B)
    assert rp.tolist() == [0] * 5 and col.size == 0 and n == 0
