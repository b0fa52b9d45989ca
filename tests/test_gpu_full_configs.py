"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The CPU checker cannot finish whole products of this size in test time (config 3 has
2.1e10 intermediate products), so every configuration is checked by
  - properties that hold for the whole result (row pointer monotone and consistent with
    nnz, every row's size bounded by its product count and the column count, columns
    strictly ascending inside every row, totals against closed forms where they exist), and
  - rows sampled by a seeded draw (the heaviest rows always included), compared with the
    checker element by element: structure bit-exact, values within the tolerance.
"""
import numpy as np
import pytest

import oracle
from paper_2404_04541_amd import workloads as W
from helpers import RTOL

pytestmark = pytest.mark.gpu


def product_counts(A, B):
    lens = np.diff(B.rowptr)
    run = np.concatenate([[0], np.cumsum(lens[A.colidx], dtype=np.int64)])
    return run[A.rowptr[1:]] - run[A.rowptr[:-1]]


def pick_rows(ip_rows, budget, n_random, seed, n_heavy=3):
    """The n_heavy rows with most products, then seeded random non-empty rows while the product budget lasts."""
    order = np.argsort(ip_rows, kind="stable")
    heavy = order[::-1][:n_heavy]
    nonempty = np.nonzero(ip_rows > 0)[0]
    draw = nonempty[W.rand_below(seed, 700, np.arange(4 * n_random, dtype=np.uint64), nonempty.size)]
    draw = draw[np.sort(np.unique(draw, return_index=True)[1])][:n_random]
    keep = np.cumsum(ip_rows[draw]) <= budget
    rows = np.unique(np.concatenate([heavy, draw[keep]]))
    return rows.astype(np.int64)


def columns_ascending_everywhere(rowptr_dev, col_dev, n_cols, chunk=1 << 27):
    """True when every row's columns are strictly ascending and inside [0, n_cols) (device-side, chunked)."""
    import torch
    nnz = col_dev.numel()
    if nnz == 0:
        return True
    starts = rowptr_dev[1:-1]   # positions where a new row begins
    for lo in range(0, nnz, chunk):
        hi = min(nnz, lo + chunk)
        c = col_dev[lo:hi]
        if int(c.min()) < 0 or int(c.max()) >= n_cols:
            return False
        nxt = col_dev[lo + 1:min(nnz, hi + 1)]
        bad = nxt <= c[:nxt.numel()]     # bad[j]: entry lo+j+1 does not ascend over entry lo+j
        a = int(torch.searchsorted(starts, lo + 1))
        b = int(torch.searchsorted(starts, lo + nxt.numel(), right=True))
        bad[(starts[a:b] - (lo + 1))] = False   # ... unless lo+j+1 starts a row
        if bool(bad.any()):
            return False
    return True


def check_full(A, B, budget=1.2e8, n_random=1500, seed=0, totals=None):
    import torch
    from paper_2404_04541_amd import binding as sg
    h = sg.Handle()
    dA = sg.to_device(A)
    dB = dA if B is A else sg.to_device(B)
    rp, nnz, plan = sg.spgemm_symbolic(h, dA, dB)
    col, val = sg.spgemm_numeric(h, plan, dA, dB, rp)
    torch.cuda.synchronize()
    st = plan.stats()
    plan.destroy()
    ip_rows = product_counts(A, B)
    assert st["ip_total"] == int(ip_rows.sum())
    if totals is not None:
        assert (st["ip_total"], nnz) == totals
    rph = rp.cpu().numpy()
    cnt = np.diff(rph)
    assert rph[0] == 0 and rph[-1] == nnz and nnz <= st["ip_total"]
    assert np.all(cnt >= 0) and np.all(cnt <= np.minimum(ip_rows, B.cols))
    assert np.all((cnt > 0) == (ip_rows > 0))
    assert columns_ascending_everywhere(rp, col, B.cols)
    rows = pick_rows(ip_rows, budget, n_random, seed)
    ref = oracle.spgemm_rows(A.rowptr, A.colidx, A.values, B.rowptr, B.colidx, B.values, rows=rows)
    assert np.array_equal(ref.cnt, cnt[rows]), "sampled row sizes differ"
    assert np.array_equal(ref.ip, ip_rows[rows])
    # gather the sampled rows of the GPU result
    idx = np.concatenate([np.arange(rph[r], rph[r + 1]) for r in rows]) if rows.size else np.zeros(0, np.int64)
    didx = torch.from_numpy(idx).cuda()
    gcol = col[didx].cpu().numpy()
    gval = val[didx].cpu().numpy()
    assert np.array_equal(gcol, ref.colidx), "sampled column indices differ"
    rtol = RTOL[np.dtype(A.values.dtype)]
    want = ref.values.astype(A.values.dtype).astype(np.float64)
    err = np.abs(gval.astype(np.float64) - want)
    assert np.all(err <= rtol * ref.absum), f"worst ratio {float((err / np.maximum(ref.absum, 1e-300)).max()):.3e}"
    return st, rows.size, int(ref.ip.sum())


def test_config2_stencil_128():
    g = 128
    a, b = W.config2(g)
    check_full(a, b, totals=((9 * g - 10) ** 3, (5 * g - 6) ** 3))


def test_config3_rmat_scale20():
    a, b = W.config3()
    st, _, _ = check_full(a, b, budget=1.5e8)
    assert st["nnz_c"] > 2 ** 32      # the row pointer must be 64-bit
    assert st["num_bin_rows"][5] > 0 and st["num_bin_rows"][6] > 0
    assert st["dense_search_tiles"] > 0 and st["dense_tiles"] > st["dense_search_tiles"]


def test_config4_rectangular():
    a, b = W.config4()
    st, _, _ = check_full(a, b)
    assert st["ip_total"] == 4194304 * 8 * 4


def test_config5_ttm_unfolded():
    a, m = W.config5()
    st, _, _ = check_full(a, m)
    assert st["ip_total"] == 10_000_000 * 16
