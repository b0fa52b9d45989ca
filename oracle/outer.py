"""Outer-product sparse x sparse product with a second-order sparse workspace (test infrastructure only).

The paper's leading example: C = A * B in the loop order k -> i -> j, A stored by columns with
only its non-empty columns kept (doubly compressed sparse columns), B by rows with only its
non-empty rows kept (doubly compressed sparse rows), the result in compressed sparse rows.
Because consecutive products land on unrelated coordinates (i, j), they pass through a workspace
that holds whole coordinates (section 4.1), run by the four stages of the algorithm template
(section 4.3): insert a component (i, j, value) into the accumulation array; when it is full, sort
it into result order and merge it, adding up equal coordinates, into the all array; at the end
compress the all array into the result's row pointer / column / value arrays.

Plain numpy, written for readability, sized for small operands.
"""
from __future__ import annotations

import numpy as np


def dcsc_from_csr(A):
    """Doubly compressed sparse columns of a CSR matrix: (cols, colptr, rowidx, values) where cols lists
    the non-empty columns ascending and entries of a column keep the order of their rows (and, for a
    repeated coordinate, of their appearance)."""
    rows = np.repeat(np.arange(A.rows, dtype=np.int64), np.diff(A.rowptr))
    order = np.lexsort((np.arange(rows.size), rows, A.colidx))   # by column, then row, then position
    c = np.asarray(A.colidx, dtype=np.int64)[order]
    cols, counts = np.unique(c, return_counts=True)
    colptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    return cols.astype(np.int32), colptr, rows[order].astype(np.int32), np.asarray(A.values)[order]


def dcsr_from_csr(B):
    """Doubly compressed sparse rows: (rows, rowptr, colidx, values) with only the non-empty rows listed."""
    lens = np.diff(B.rowptr)
    keep = np.nonzero(lens > 0)[0]
    rowptr = np.concatenate([[0], np.cumsum(lens[keep])]).astype(np.int64)
    return keep.astype(np.int32), rowptr, np.asarray(B.colidx, dtype=np.int32).copy(), np.asarray(B.values).copy()


def _sort_and_merge(acc_i, acc_j, acc_v, acc_s, all_i, all_j, all_v, all_s):
    """Sort stage + merge stage: the accumulation array goes into result order (row, then column; equal
    coordinates keep their order of insertion), joins the all array (older sums first), and equal
    coordinates are added up."""
    i = np.concatenate([all_i, acc_i]); j = np.concatenate([all_j, acc_j])
    v = np.concatenate([all_v, acc_v]); s = np.concatenate([all_s, acc_s])
    order = np.lexsort((np.arange(i.size), j, i))
    i, j, v, s = i[order], j[order], v[order], s[order]
    if i.size == 0:
        return i, j, v, s
    head = np.ones(i.size, dtype=bool)
    head[1:] = (i[1:] != i[:-1]) | (j[1:] != j[:-1])
    starts = np.nonzero(head)[0]
    return i[starts], j[starts], np.add.reduceat(v, starts), np.add.reduceat(s, starts)


def spgemm_outer(A, B, capacity: int = 1 << 16):
    """C = A * B by outer products through the insert / sort / merge / compress stages.
    Returns (rowptr int64, colidx int32, values float64, absum float64, products)."""
    if A.cols != B.rows:
        raise ValueError("A.cols != B.rows")
    a_cols, a_ptr, a_row, a_val = dcsc_from_csr(A)
    b_rows, b_ptr, b_col, b_val = dcsr_from_csr(B)
    a_val = a_val.astype(np.float64); b_val = b_val.astype(np.float64)
    e64, e32 = np.zeros(0, np.int64), np.zeros(0, np.float64)
    all_i, all_j, all_v, all_s = e64, e64, e32, e32
    acc_i, acc_j, acc_v, acc_s = [], [], [], []
    filled = 0
    products = 0
    pb = 0
    for pa, k in enumerate(a_cols):                      # k: co-iteration of A's columns and B's rows
        while pb < b_rows.size and b_rows[pb] < k:
            pb += 1
        if pb == b_rows.size or b_rows[pb] != k:
            continue
        for p in range(a_ptr[pa], a_ptr[pa + 1]):        # i
            lo, hi = b_ptr[pb], b_ptr[pb + 1]            # j
            n = int(hi - lo)
            pos = 0
            while pos < n:                               # insert; a full accumulation array is sorted and merged first
                take = min(n - pos, capacity - filled)
                if take == 0:
                    all_i, all_j, all_v, all_s = _sort_and_merge(np.concatenate(acc_i), np.concatenate(acc_j), np.concatenate(acc_v),
                                                                 np.concatenate(acc_s), all_i, all_j, all_v, all_s)
                    acc_i, acc_j, acc_v, acc_s, filled = [], [], [], [], 0
                    continue
                sl = slice(lo + pos, lo + pos + take)
                prod = a_val[p] * b_val[sl]
                acc_i.append(np.full(take, a_row[p], dtype=np.int64)); acc_j.append(b_col[sl].astype(np.int64))
                acc_v.append(prod); acc_s.append(np.abs(prod))
                filled += take; pos += take; products += take
    if filled:
        all_i, all_j, all_v, all_s = _sort_and_merge(np.concatenate(acc_i), np.concatenate(acc_j), np.concatenate(acc_v),
                                                     np.concatenate(acc_s), all_i, all_j, all_v, all_s)
    # compress: count the components of every row, prefix sum, copy columns and values
    rowptr = np.zeros(A.rows + 1, dtype=np.int64)
    np.cumsum(np.bincount(all_i, minlength=A.rows), out=rowptr[1:])
    return rowptr, all_j.astype(np.int32), all_v, all_s, products
