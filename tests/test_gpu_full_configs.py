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


def strict_failures(err, want, rtol):
    """How many values miss the plain element-wise test |gpu - ref| <= rtol * |ref| (reported, not asserted:
    a nearly cancelled sum can miss it for any change of summation order although nothing is wrong)."""
    return int(np.count_nonzero(err > rtol * np.abs(want)))


def check_whole(A, B, block_rows=1 << 18, totals=None, gpu=None):
    """Whole-result comparison with the checker, in blocks of rows so that only one block of the
    reference is on the host at a time: structure bit-exact, values within the tolerance."""
    import torch
    from paper_2404_04541_amd import binding as sg
    if gpu is None:
        h = sg.Handle()
        dA = sg.to_device(A)
        dB = dA if B is A else sg.to_device(B)
        rp, nnz, plan = sg.spgemm_symbolic(h, dA, dB)
        col, val = sg.spgemm_numeric(h, plan, dA, dB, rp)
        torch.cuda.synchronize()
        st = plan.stats()
        plan.destroy()
    else:
        rp, col, val, nnz, st = gpu
    if totals is not None:
        assert (st["ip_total"], nnz) == totals
    rph = rp.cpu().numpy()
    rtol = RTOL[np.dtype(A.values.dtype)]
    strict = 0
    ip_sum = 0
    for lo in range(0, A.rows, block_rows):
        hi = min(A.rows, lo + block_rows)
        ref = oracle.spgemm_rows(A.rowptr, A.colidx, A.values, B.rowptr, B.colidx, B.values, row_lo=lo, row_hi=hi)
        ip_sum += int(ref.ip.sum())
        assert np.array_equal(ref.rowptr + rph[lo], rph[lo:hi + 1]), f"row pointer differs in rows [{lo}, {hi})"
        a, b = int(rph[lo]), int(rph[hi])
        assert np.array_equal(col[a:b].cpu().numpy(), ref.colidx), f"column indices differ in rows [{lo}, {hi})"
        want = ref.values.astype(A.values.dtype).astype(np.float64)
        err = np.abs(val[a:b].cpu().numpy().astype(np.float64) - want)
        bad = err > rtol * ref.absum
        assert not bad.any(), f"{int(bad.sum())} values off in rows [{lo}, {hi})"
        strict += strict_failures(err, want, rtol)
    assert ip_sum == st["ip_total"]
    print(f"whole result compared: {nnz} entries, {strict} of them miss the plain rtol*|ref| test (cancellation)")
    return st


def numeric_class(ip, cnt):
    """The numeric row classes of the library, recomputed on the host (0/1 sorted list, 2/3 hash, 5/6 dense)."""
    c = np.full(ip.shape, 7, dtype=np.int64)
    live = cnt > 0
    c[live] = np.where(ip[live] <= 1 << 20, 5, 6)
    c[live & (cnt <= 1536)] = 3
    c[live & (cnt <= 192)] = 2
    c[live & (ip <= 128)] = 1
    c[live & (ip <= 32)] = 0
    return c


def test_config2_stencil_128():
    g = 128
    a, b = W.config2(g)
    check_whole(a, b, totals=((9 * g - 10) ** 3, (5 * g - 6) ** 3))


def test_config3_rmat_scale20_every_class_and_tile_kind():
    """Config 3 cannot be compared whole in test time (2.1e10 products); rows are drawn from every numeric
    class and, inside the dense classes, from every kind of tile the planner makes: rows that become one
    searched tile, rows whose structure is kept as columns (ranked tiles from a column list), rows kept as
    flag words (ranked tiles from flag words), and the heaviest rows (direct tiles in their first blocks)."""
    import torch
    from paper_2404_04541_amd import binding as sg
    a, b = W.config3()
    h = sg.Handle()
    dA = sg.to_device(a)
    rp, nnz, plan = sg.spgemm_symbolic(h, dA, dA)
    col, val = sg.spgemm_numeric(h, plan, dA, dA, rp)
    torch.cuda.synchronize()
    st = plan.stats()
    plan.destroy()
    assert nnz > 2 ** 32 and st["nnz_c"] == nnz
    assert st["dense_search_tiles"] > 0 and st["dense_direct_tiles"] > 0 and st["dense_tiles"] > st["dense_search_tiles"]
    assert st["plan_bytes"] > st["plan_list_bytes"] >= st["plan_list_used"] > 0
    ip_rows = product_counts(a, b)
    rph = rp.cpu().numpy()
    cnt = np.diff(rph)
    assert rph[0] == 0 and rph[-1] == nnz and np.all(cnt <= np.minimum(ip_rows, b.cols)) and np.all((cnt > 0) == (ip_rows > 0))
    assert columns_ascending_everywhere(rp, col, b.cols)
    cls = numeric_class(ip_rows, cnt)
    for c in (0, 1, 2, 3, 5, 6):
        assert st["num_bin_rows"][c] == int(np.count_nonzero(cls == c)), f"class {c}"
    dense = cls >= 5
    dense = dense & (cls < 7)
    words = b.cols // 32
    strata = {
        "class 0": cls == 0, "class 1": cls == 1, "class 2": cls == 2, "class 3": cls == 3, "class 6": cls == 6,
        "searched tile": dense & (cnt <= 10000) & (ip_rows <= 4 * cnt),
        "ranked from columns": dense & (cnt > 12000) & (cnt < words),
        "ranked from flag words": dense & (cnt >= words) & (cnt < 200000),
    }
    picked = [np.argsort(ip_rows, kind="stable")[::-1][:3]]      # the heaviest rows: direct tiles in their dense blocks
    for k, (name, mask) in enumerate(strata.items()):
        rows = np.nonzero(mask)[0]
        assert rows.size > 0, f"no row in stratum '{name}'"
        draw = rows[W.rand_below(0, 710 + k, np.arange(400, dtype=np.uint64), rows.size)]
        draw = draw[np.sort(np.unique(draw, return_index=True)[1])]
        keep = np.cumsum(ip_rows[draw]) <= 1.5e7
        keep[0] = True
        picked.append(draw[keep])
        print(f"stratum '{name}': {rows.size} rows, {int(keep.sum())} compared")
    rows = np.unique(np.concatenate(picked)).astype(np.int64)
    ref = oracle.spgemm_rows(a.rowptr, a.colidx, a.values, b.rowptr, b.colidx, b.values, rows=rows)
    assert np.array_equal(ref.cnt, cnt[rows]) and np.array_equal(ref.ip, ip_rows[rows])
    idx = np.concatenate([np.arange(rph[r], rph[r + 1]) for r in rows])
    didx = torch.from_numpy(idx).cuda()
    assert np.array_equal(col[didx].cpu().numpy(), ref.colidx), "sampled column indices differ"
    want = ref.values.astype(np.float32).astype(np.float64)
    err = np.abs(val[didx].cpu().numpy().astype(np.float64) - want)
    assert np.all(err <= 1e-5 * ref.absum), f"worst ratio {float((err / np.maximum(ref.absum, 1e-300)).max()):.3e}"
    print(f"{rows.size} rows, {idx.size} entries compared; {strict_failures(err, want, 1e-5)} miss the plain rtol*|ref| test")


def test_config4_rectangular():
    a, b = W.config4()
    st = check_whole(a, b)
    assert st["ip_total"] == 4194304 * 8 * 4


def test_config5_ttm_unfolded():
    a, m = W.config5()
    st = check_whole(a, m)
    assert st["ip_total"] == 10_000_000 * 16
