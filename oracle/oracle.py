"""ctypes wrapper of the CPU checker in spgemm_oracle.cpp (test infrastructure only).

The product path never imports this module.  Operands are plain numpy arrays
(rowptr int64, colidx int32, values float32/float64).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spgemm_oracle.cpp")
_LIB = os.path.join(_HERE, "libspgemm_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the checker with g++ (-O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_spgemm_rows.restype = C.c_int
        _lib.oracle_spgemm_rows.argtypes = [
            C.c_int64, C.c_int64, C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_void_p,
            C.c_int, C.c_int,
            C.c_void_p, C.c_void_p,
            C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]
        _lib.oracle_free.argtypes = [C.c_void_p]
        _lib.oracle_free.restype = None
        _lib.oracle_max_threads.restype = C.c_int
    return _lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


@dataclass
class OracleResult:
    cnt: np.ndarray      # int64 per requested row: entries of that row of C
    ip: np.ndarray       # int64 per requested row: intermediate products
    rowptr: np.ndarray   # int64, len(cnt)+1, offsets into colidx/values
    colidx: np.ndarray   # int32, ascending inside each row
    values: np.ndarray   # float64 sums (round to float32 yourself for float32 operands)
    absum: np.ndarray    # float64, sum of |a*b| per entry


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def spgemm_rows(a_rowptr, a_col, a_val, b_rowptr, b_col, b_val, rows=None, row_lo=0, row_hi=None,
                threads: int = 0) -> OracleResult:
    """Rows of C = A*B: either the index list `rows` or the range [row_lo, row_hi)."""
    lib = _load()
    a_rowptr = np.ascontiguousarray(a_rowptr, dtype=np.int64)
    b_rowptr = np.ascontiguousarray(b_rowptr, dtype=np.int64)
    a_col = np.ascontiguousarray(a_col, dtype=np.int32)
    b_col = np.ascontiguousarray(b_col, dtype=np.int32)
    if a_val is not None:
        a_val = np.ascontiguousarray(a_val)
    if b_val is not None:
        b_val = np.ascontiguousarray(b_val)
    dts = {v.dtype for v in (a_val, b_val) if v is not None}
    if len(dts) > 1 or (dts and next(iter(dts)) not in (np.dtype(np.float32), np.dtype(np.float64))):
        raise TypeError("values must both be float32 or both float64")
    is_f32 = int(bool(dts) and next(iter(dts)) == np.dtype(np.float32))
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        nr = rows.size
    else:
        if row_hi is None:
            row_hi = a_rowptr.size - 1
        nr = int(row_hi) - int(row_lo)
    cnt = np.zeros(max(nr, 0), dtype=np.int64)
    ip = np.zeros(max(nr, 0), dtype=np.int64)
    pc, pv, ps = C.c_void_p(), C.c_void_p(), C.c_void_p()
    rc = lib.oracle_spgemm_rows(nr, int(row_lo), _ptr(rows), _ptr(a_rowptr), _ptr(a_col), _ptr(a_val),
                                _ptr(b_rowptr), _ptr(b_col), _ptr(b_val), is_f32, int(threads),
                                _ptr(cnt), _ptr(ip), C.byref(pc), C.byref(pv), C.byref(ps))
    if rc != 0:
        raise RuntimeError("oracle_spgemm_rows failed")
    total = int(cnt.sum())
    try:
        col = np.ctypeslib.as_array(C.cast(pc, C.POINTER(C.c_int32)), shape=(max(total, 1),))[:total].copy()
        val = np.ctypeslib.as_array(C.cast(pv, C.POINTER(C.c_double)), shape=(max(total, 1),))[:total].copy()
        ab = np.ctypeslib.as_array(C.cast(ps, C.POINTER(C.c_double)), shape=(max(total, 1),))[:total].copy()
    finally:
        lib.oracle_free(pc); lib.oracle_free(pv); lib.oracle_free(ps)
    rowptr = np.zeros(nr + 1, dtype=np.int64)
    np.cumsum(cnt, out=rowptr[1:])
    return OracleResult(cnt, ip, rowptr, col, val, ab)


def spgemm(A, B, threads: int = 0) -> OracleResult:
    """Whole product for operands with .rowptr/.colidx/.values attributes."""
    return spgemm_rows(A.rowptr, A.colidx, A.values, B.rowptr, B.colidx, B.values, threads=threads)


def _mode_axes(mode: int):
    """Unfolding over `mode` (1, 2 or 3): the two kept modes form the row (earlier mode major), the
    unfolded mode is the column.  Returns the positions (a, b, c) in (i, j, k) of row-major, row-minor, column."""
    if mode not in (1, 2, 3):
        raise ValueError("mode must be 1, 2 or 3")
    return {1: (1, 2, 0), 2: (0, 2, 1), 3: (0, 1, 2)}[mode]


def unfold(shape, mode, xi, xj, xk, xval):
    """Mode-`mode` unfolding of a coordinate tensor X(i,j,k) (the index folding of the paper's section 7.4):
    the two other coordinates fold into the row (mode 3: i*J + j; mode 2: i*K + k; mode 1: j*K + k), the
    coordinate of `mode` is the column; entries ordered by (row, column), repeated coordinates kept as
    separate entries in their order of appearance.  Returns (rowptr int64, colidx int32, values)."""
    dims = tuple(int(v) for v in shape)
    x = [np.asarray(xi, dtype=np.int64), np.asarray(xj, dtype=np.int64), np.asarray(xk, dtype=np.int64)]
    for c, d in zip(x, dims):
        if c.size and (c.min() < 0 or c.max() >= d):
            raise ValueError("coordinate out of range")
    a, b, c = _mode_axes(mode)
    row = x[a] * dims[b] + x[b]
    order = np.lexsort((np.arange(row.size), x[c], row))   # by row, then column, then input position
    nrows = dims[a] * dims[b]
    rowptr = np.zeros(nrows + 1, dtype=np.int64)
    np.cumsum(np.bincount(row, minlength=nrows), out=rowptr[1:])
    return rowptr, x[c][order].astype(np.int32), np.asarray(xval)[order]


def spttm(shape, mode, xi, xj, xk, xval, M, threads: int = 0) -> OracleResult:
    """Tensor times matrix over `mode`: the coordinate of that mode is replaced by l with
    Y(..l..) = sum_x X(..x..) M(x,l), computed as the row-wise product of the mode unfolding with M.
    Row r of the result is the same fold of the two kept coordinates as in unfold()."""
    rowptr, colidx, values = unfold(shape, mode, xi, xj, xk, xval)
    return spgemm_rows(rowptr, colidx, values, M.rowptr, M.colidx, M.values, threads=threads)


def fold(shape, mode, rowptr, colidx):
    """Coordinates (i, j, k) of the entries of a matrix that is the mode-`mode` unfolding of a tensor of
    the given shape (after a contraction, shape[mode-1] is the matrix's column count)."""
    dims = tuple(int(v) for v in shape)
    a, b, c = _mode_axes(mode)
    rowptr = np.asarray(rowptr, dtype=np.int64)
    rows = np.repeat(np.arange(rowptr.size - 1, dtype=np.int64), np.diff(rowptr))
    out = [None, None, None]
    out[a] = (rows // dims[b]).astype(np.int32)
    out[b] = (rows % dims[b]).astype(np.int32)
    out[c] = np.asarray(colidx, dtype=np.int32).copy()
    return tuple(out)


def unfold_mode3(shape, xi, xj, xk, xval):
    """unfold() over the third mode: row i*J + j, column k."""
    return unfold(shape, 3, xi, xj, xk, xval)


def spttm_mode3(shape, xi, xj, xk, xval, M, threads: int = 0) -> OracleResult:
    """spttm() over the third mode: row i*J + j of the result holds Y(i,j,:)."""
    return spttm(shape, 3, xi, xj, xk, xval, M, threads=threads)
