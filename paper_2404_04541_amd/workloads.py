"""Seeded synthetic sparse operands (numpy only).

This module serves both the GPU library's callers and the CPU checker, so it
holds no part of the product's arithmetic: it only draws structures and
values.  Everything is derived from one counter-based generator (a 64-bit
finalising mix of seed, stream id and element index), so a matrix does not
depend on thread count or on the order in which its pieces are produced.

The paper evaluates on SuiteSparse matrices and FROSTT tensors (section 7.1)
which are not available offline; the generators below are the stand-ins with
the shapes and distributions of the five benchmark configurations.

All CSR outputs: rowptr int64 (rows+1), colidx int32 ascending and unique
inside each row, values float32/float64 indexed by CSR position.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)
_S1 = np.uint64(0xD6E8FEB86659FD93)
_S2 = np.uint64(0xA0761D6478BD642F)


def _fin(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser (public-domain mixing function of Steele/Vigna)."""
    z = (z ^ (z >> np.uint64(30))) * _C1
    z = (z ^ (z >> np.uint64(27))) * _C2
    return z ^ (z >> np.uint64(31))


def rand_u64(seed: int, stream: int, index: np.ndarray) -> np.ndarray:
    """Counter-based 64-bit draw: a pure function of (seed, stream, index)."""
    with np.errstate(over="ignore"):
        idx = np.asarray(index).astype(np.uint64)
        key = _fin(np.uint64(seed) * _S1 + np.uint64(stream) * _S2 + _GOLD)
        return _fin(_fin(idx * _GOLD + key) ^ key)


def rand_unit(seed: int, stream: int, index: np.ndarray) -> np.ndarray:
    """Uniform double in [0, 1) with 53 random bits."""
    return (rand_u64(seed, stream, index) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def rand_below(seed: int, stream: int, index: np.ndarray, n: int) -> np.ndarray:
    """Uniform integer in [0, n) (multiply-shift on the top 32 bits; n < 2**32)."""
    hi = rand_u64(seed, stream, index) >> np.uint64(32)
    return ((hi * np.uint64(n)) >> np.uint64(32)).astype(np.int64)


@dataclass
class CSR:
    rows: int
    cols: int
    rowptr: np.ndarray  # int64, rows+1
    colidx: np.ndarray  # int32, nnz
    values: np.ndarray  # float32 or float64, nnz

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def to_dense(self) -> np.ndarray:
        """Densify (duplicates add). For tiny matrices only."""
        d = np.zeros((self.rows, self.cols), dtype=np.float64)
        r = np.repeat(np.arange(self.rows), np.diff(self.rowptr))
        np.add.at(d, (r, self.colidx), self.values.astype(np.float64))
        return d


def draw_values(nnz: int, lo: float, hi: float, dtype, seed: int, stream: int) -> np.ndarray:
    """Values uniform in [lo, hi), one per CSR position, drawn after the structure is final."""
    u = rand_unit(seed, stream, np.arange(nnz, dtype=np.uint64))
    return (lo + (hi - lo) * u).astype(dtype)


def _distinct_columns(rows: int, cols: int, per_row: int, seed: int, stream: int) -> np.ndarray:
    """rows x per_row array of distinct uniform columns per row, ascending (redraw on repeats)."""
    if per_row > cols:
        raise ValueError("per_row exceeds column count")
    idx = np.arange(rows * per_row, dtype=np.uint64).reshape(rows, per_row)
    c = rand_below(seed, stream, idx, cols)
    attempt = 0
    while True:
        c.sort(axis=1)
        dup = np.zeros(c.shape, dtype=bool)
        dup[:, 1:] = c[:, 1:] == c[:, :-1]
        if not dup.any():
            return c
        attempt += 1
        r, s = np.nonzero(dup)
        redraw_idx = (np.uint64(attempt) << np.uint64(40)) + idx[r, s]
        c[r, s] = rand_below(seed, stream, redraw_idx, cols)


def uniform_rows(rows: int, cols: int, per_row: int, seed: int, stream: int,
                 dtype=np.float64, lo: float = -1.0, hi: float = 1.0) -> CSR:
    """Exactly per_row nonzeros in every row at distinct uniform-random columns."""
    c = _distinct_columns(rows, cols, per_row, seed, stream)
    rowptr = np.arange(rows + 1, dtype=np.int64) * per_row
    colidx = c.reshape(-1).astype(np.int32)
    vals = draw_values(colidx.size, lo, hi, dtype, seed, stream + 1)
    return CSR(rows, cols, rowptr, colidx, vals)


def stencil27(g: int, seed: int = 0, stream: int = 10, dtype=np.float64, periodic: bool = False,
              ones: bool = False) -> CSR:
    """27-point stencil on a g^3 grid, row = x + g*(y + g*z); neighbours {-1,0,1}^3.

    periodic=False clips at the boundary (banded matrix, (3g-2)^3 nonzeros);
    periodic=True wraps (27 g^3 nonzeros).  Values uniform in [-1,1) (not symmetric),
    or all ones when ones=True (used by closed-form checks).
    """
    n = g * g * g
    ar = np.arange(g, dtype=np.int64)
    z, y, x = np.meshgrid(ar, ar, ar, indexing="ij")
    x = x.reshape(-1); y = y.reshape(-1); z = z.reshape(-1)
    cols = np.empty((n, 27), dtype=np.int64)
    ok = np.empty((n, 27), dtype=bool)
    s = 0
    for dz in (-1, 0, 1):
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                xx, yy, zz = x + dx, y + dy, z + dz
                if periodic:
                    xx %= g; yy %= g; zz %= g
                    ok[:, s] = True
                else:
                    ok[:, s] = (xx >= 0) & (xx < g) & (yy >= 0) & (yy < g) & (zz >= 0) & (zz < g)
                cols[:, s] = xx + g * (yy + g * zz)
                s += 1
    big = np.int64(n)
    cols[~ok] = big
    cols.sort(axis=1)
    if periodic and g < 3:
        # wrap-around makes neighbours coincide on tiny grids: keep one copy
        dupm = np.zeros(cols.shape, dtype=bool)
        dupm[:, 1:] = cols[:, 1:] == cols[:, :-1]
        cols[dupm] = big
        cols.sort(axis=1)
    keep = cols < big
    counts = keep.sum(axis=1)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    colidx = cols[keep].astype(np.int32)
    if ones:
        vals = np.ones(colidx.size, dtype=dtype)
    else:
        vals = draw_values(colidx.size, -1.0, 1.0, dtype, seed, stream)
    return CSR(n, n, rowptr, colidx, vals)


def rmat(scale: int, edge_factor: int = 16, a: float = 0.57, b: float = 0.19, c: float = 0.19,
         seed: int = 0, stream: int = 20, dtype=np.float32) -> CSR:
    """R-MAT power-law graph, 2^scale vertices, edge_factor * 2^scale directed edges drawn.

    Per bit level the quadrant is a (row bit 0, col bit 0), b (0,1), c (1,0), d (1,1);
    no noise, no vertex permutation, self loops kept, not symmetrised; duplicate
    edges collapse to one entry; then values uniform in [0,1).
    """
    n = 1 << scale
    ne = edge_factor * n
    eidx = np.arange(ne, dtype=np.uint64)
    r = np.zeros(ne, dtype=np.int64)
    cc = np.zeros(ne, dtype=np.int64)
    for level in range(scale):
        u = rand_unit(seed, stream + 1 + level, eidx)
        rb = (u >= a + b).astype(np.int64)
        cb = (((u >= a) & (u < a + b)) | (u >= a + b + c)).astype(np.int64)
        r = (r << 1) | rb
        cc = (cc << 1) | cb
    key = np.unique((r << scale) | cc)
    r = key >> scale
    cc = key & (n - 1)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(r, minlength=n), out=rowptr[1:])
    vals = draw_values(key.size, 0.0, 1.0, dtype, seed, stream)
    return CSR(n, n, rowptr, cc.astype(np.int32), vals)


@dataclass
class COO3:
    shape: tuple
    i: np.ndarray
    j: np.ndarray
    k: np.ndarray
    values: np.ndarray


def coo3_uniform(shape, nnz: int, seed: int = 0, stream: int = 40, dtype=np.float64) -> COO3:
    """nnz distinct uniform-random coordinates of a 3-tensor, sorted lexicographically, values in [-1,1)."""
    I, J, K = shape
    total = I * J * K
    if nnz > total:
        raise ValueError("more nonzeros than tensor elements")
    got = np.empty(0, dtype=np.int64)
    drawn = 0
    while got.size < nnz:
        need = nnz - got.size
        batch = need + need // 64 + 16
        idx = np.arange(drawn, drawn + batch, dtype=np.uint64)
        drawn += batch
        hi = rand_below(seed, stream, idx, I * J)
        lo = rand_below(seed, stream + 1, idx, K)
        lin = hi * K + lo
        # keep first occurrences in draw order so that the set is independent of batch size
        allk = np.concatenate([got, lin])
        _, first = np.unique(allk, return_index=True)
        first.sort()
        got = allk[first][:nnz]
    got.sort()
    vals = draw_values(nnz, -1.0, 1.0, dtype, seed, stream + 2)
    return COO3((I, J, K), (got // (J * K)).astype(np.int32), ((got // K) % J).astype(np.int32),
                (got % K).astype(np.int32), vals)


def unfold_mode3(x: COO3) -> CSR:
    """Mode-3 unfolding of X(i,j,k): row = i*J + j, column = k (coordinates assumed distinct)."""
    I, J, K = x.shape
    row = x.i.astype(np.int64) * J + x.j.astype(np.int64)
    order = np.lexsort((x.k, row))
    row = row[order]
    rowptr = np.zeros(I * J + 1, dtype=np.int64)
    np.cumsum(np.bincount(row, minlength=I * J), out=rowptr[1:])
    return CSR(I * J, K, rowptr, x.k[order].astype(np.int32), x.values[order])


def identity(n: int, dtype=np.float64) -> CSR:
    return CSR(n, n, np.arange(n + 1, dtype=np.int64), np.arange(n, dtype=np.int32), np.ones(n, dtype=dtype))


def permutation(n: int, seed: int, stream: int = 50, dtype=np.float64) -> CSR:
    """Permutation matrix: row i has a single 1 at column perm[i]."""
    perm = np.argsort(rand_u64(seed, stream, np.arange(n, dtype=np.uint64)), kind="stable")
    return CSR(n, n, np.arange(n + 1, dtype=np.int64), perm.astype(np.int32), np.ones(n, dtype=dtype))


def random_csr(rows: int, cols: int, mean_per_row: float, seed: int, stream: int = 60, dtype=np.float64,
               sort_rows: bool = True, allow_duplicates: bool = False, lo: float = -1.0, hi: float = 1.0) -> CSR:
    """Ragged random matrix for tests: row lengths vary (many rows empty), columns uniform.

    sort_rows=False leaves each row's columns in draw order; allow_duplicates=True keeps
    repeated (row, column) entries.  Both are legal operands.
    """
    u = rand_unit(seed, stream, np.arange(rows, dtype=np.uint64))
    # geometric-ish spread of lengths with the requested mean, capped at 4x the mean (+1)
    lens = np.minimum(np.floor(-np.log1p(-u) * mean_per_row), 4 * mean_per_row + 1).astype(np.int64)
    if not allow_duplicates:
        lens = np.minimum(lens, cols)
    rowptr = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(lens, out=rowptr[1:])
    nnz = int(rowptr[-1])
    col = rand_below(seed, stream + 1, np.arange(nnz, dtype=np.uint64), max(cols, 1)) if nnz else np.zeros(0, np.int64)
    r = np.repeat(np.arange(rows, dtype=np.int64), lens)
    if not allow_duplicates and nnz:
        key = np.unique(r * cols + col)
        r = key // cols
        col_sorted = key % cols
        rowptr = np.zeros(rows + 1, dtype=np.int64)
        np.cumsum(np.bincount(r, minlength=rows), out=rowptr[1:])
        col = col_sorted
        nnz = key.size
        if not sort_rows:
            # deterministic shuffle inside each row
            sk = rand_u64(seed, stream + 2, np.arange(nnz, dtype=np.uint64))
            order = np.lexsort((sk, r))
            col = col[order]
    elif sort_rows and nnz:
        order = np.lexsort((col, r))
        col = col[order]
    vals = draw_values(nnz, lo, hi, dtype, seed, stream + 3)
    return CSR(rows, cols, rowptr, col.astype(np.int32), vals)


def dedup_sweep(K: int, dense_elements: int = 100_000_000, column_fraction: float = 0.1, per_column: int = 1000,
                seed: int = 0, stream: int = 80, dtype=np.float64):
    """Operands of the paper's synthetic first-order sweep (section 7.2): B is I x K with I*K = dense_elements;
    a tenth of its columns are non-empty, each with per_column nonzeros at distinct uniform rows; the second
    operand is the transpose of B with its columns rotated by one (section 7.1).  Growing K shrinks I, so
    more products of a row land on the same output column (more deduplication).
    Returns (B, C) with C of shape K x I; the product B*C is I x I."""
    I = dense_elements // K
    nc = max(1, int(round(K * column_fraction)))
    per_column = min(per_column, I)
    cols = np.sort(np.argsort(rand_u64(seed, stream, np.arange(K, dtype=np.uint64)), kind="stable")[:nc])
    # per non-empty column: the per_column rows with the smallest random keys
    keys = rand_u64(seed, stream + 1, np.arange(nc * I, dtype=np.uint64)).reshape(nc, I)
    rows = np.argpartition(keys, per_column - 1, axis=1)[:, :per_column]
    r = rows.reshape(-1).astype(np.int64)
    c = np.repeat(cols, per_column).astype(np.int64)
    vals = draw_values(r.size, -1.0, 1.0, dtype, seed, stream + 2)
    def to_csr(nrows, ncols, rr, cc, vv):
        order = np.lexsort((cc, rr))
        rowptr = np.zeros(nrows + 1, dtype=np.int64)
        np.cumsum(np.bincount(rr, minlength=nrows), out=rowptr[1:])
        return CSR(nrows, ncols, rowptr, cc[order].astype(np.int32), vv[order])
    B = to_csr(I, K, r, c, vals)
    C = to_csr(K, I, c, (r + 1) % I, vals)
    return B, C


# ---------------------------------------------------------------------------
# The five benchmark configurations (seed 0 for all).
# ---------------------------------------------------------------------------

def config1(seed: int = 0):
    """C = A*A, A 1000x1000 fp64, exactly 10 nonzeros per row, values in [-1,1)."""
    a = uniform_rows(1000, 1000, 10, seed, 1, np.float64)
    return a, a


def config2(g: int = 128, seed: int = 0, periodic: bool = False):
    """C = A*A, A the 27-point stencil on a g^3 grid (default 128), fp64 values in [-1,1)."""
    a = stencil27(g, seed, 10, np.float64, periodic)
    return a, a


def config3(scale: int = 20, seed: int = 0):
    """C = A*A, A R-MAT (a=.57, b=c=.19, d=.05), 2^scale rows, average degree 16 drawn, fp32 values in [0,1)."""
    a = rmat(scale, 16, 0.57, 0.19, 0.19, seed, 20, np.float32)
    return a, a


def config4(rows: int = 4194304, bcols: int = 65536, seed: int = 0):
    """C = A*B, A rows x rows with 8 per row, B rows x bcols with 4 per row, fp64."""
    a = uniform_rows(rows, rows, 8, seed, 30, np.float64)
    b = uniform_rows(rows, bcols, 4, seed, 32, np.float64)
    return a, b


def config5(dim: int = 2048, nnz: int = 10_000_000, per_row: int = 16, seed: int = 0):
    """Sparse TTM over mode 3: unfold X (dim^3, nnz distinct entries) to (dim*dim) x dim CSR, times sparse M (dim x dim)."""
    x = coo3_uniform((dim, dim, dim), nnz, seed, 40, np.float64)
    a = unfold_mode3(x)
    m = uniform_rows(dim, dim, per_row, seed, 44, np.float64)
    return a, m
