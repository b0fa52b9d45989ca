"""Rows placed exactly on the library's class boundaries, on both sides of each: product counts of
32/33, 128/129, 768/769, 1536/1537 (symbolic classes), output sizes of 192/193 and 1536/1537 (numeric
classes), a row of exactly as many entries as a searched tile holds and one more, a block of 8192
columns with exactly the direct-tile threshold of entries and one less; unsorted and repeated B rows
over more than one block; an unsorted B with a row too long for the dense workspaces."""
import numpy as np
import pytest

from paper_2404_04541_amd import workloads as W
from helpers import gpu_product, assert_matches_oracle

pytestmark = pytest.mark.gpu

SEARCH_CAP = 11264
DIRECT_MIN = 6144


def csr_from_rows(rows, cols, dtype=np.float64, seed=5):
    lens = np.array([len(r) for r in rows], dtype=np.int64)
    rowptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    colidx = np.concatenate([np.asarray(r, dtype=np.int32) for r in rows]) if lens.sum() else np.zeros(0, np.int32)
    return W.CSR(len(rows), cols, rowptr, colidx, W.draw_values(int(lens.sum()), -1.0, 1.0, dtype, seed, 1))


def spread(n, cols, offset=0):
    """n ascending distinct columns spread evenly over [0, cols)."""
    return (np.arange(n, dtype=np.int64) * cols // n + offset).astype(np.int32)


def boundary_operands(dtype):
    n = 1 << 20
    b_rows, a_rows, want = [], [], []

    def add(b_lists):
        """One row of A that multiplies the given new rows of B."""
        ks = []
        for cols in b_lists:
            ks.append(len(b_rows))
            b_rows.append(cols)
        a_rows.append(ks)

    for ip in (32, 33, 128, 129, 768, 769, 1536, 1537):          # one B row: ip = cnt = its length
        add([spread(ip, n)])
    for ip in (32, 33, 128, 129):                                # two B rows, the second inside the first: cnt = ip / 2 (rounded up)
        first = spread((ip + 1) // 2, n)
        add([first, first[:ip // 2]])
    for cnt in (192, 193, 1536, 1537):                           # three products per column: the numeric classes by output size
        base = spread(cnt, n)
        add([base, base, base[:cnt - 1]])
    for cnt in (SEARCH_CAP, SEARCH_CAP + 1, SEARCH_CAP - 1):     # two B rows, disjoint, over the whole width
        base = spread(cnt, n)
        add([base[0::2], base[1::2]])
    for e in (DIRECT_MIN, DIRECT_MIN - 1):                       # a block of 8192 columns with exactly / just under the threshold
        first = np.sort(W.rand_below(3, e, np.arange(20000, dtype=np.uint64), 8192))
        first = np.unique(first)[:e]
        while first.size < e:
            first = np.unique(np.concatenate([first, np.arange(8192)]))[:e]
        add([first.astype(np.int32), spread(8000, n - 8192, 8192)])
    a_rows.append([])                                            # an empty row between
    add([spread(40000, n), spread(40000, n, 3), spread(300, n, 7)])   # a long row: several ranked tiles
    return csr_from_rows(a_rows, len(b_rows), dtype, 6), csr_from_rows(b_rows, n, dtype, 7)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_rows_on_every_class_boundary(dtype):
    A, B = boundary_operands(dtype)
    got = gpu_product(A, B)
    ref = assert_matches_oracle(A, B, got, what="boundary rows")
    st = got[3]
    ip, cnt = ref.ip, ref.cnt
    assert ip[:8].tolist() == [32, 33, 128, 129, 768, 769, 1536, 1537] and np.array_equal(cnt[:8], ip[:8])
    assert cnt[12:16].tolist() == [192, 193, 1536, 1537]
    assert cnt[16:19].tolist() == [SEARCH_CAP, SEARCH_CAP + 1, SEARCH_CAP - 1]
    assert st["sym_bin_rows"][0] >= 1 and st["sym_bin_rows"][1] >= 2 and st["sym_bin_rows"][2] >= 2 and st["sym_bin_rows"][3] >= 2
    assert ip[8:12].tolist() == [32, 33, 128, 129] and cnt[8:12].tolist() == [16, 17, 64, 65]
    # searched tiles are planned by the dense symbolic kernel (rows of more than 1536 products) for rows of at most
    # SEARCH_CAP entries and at most 4 products per entry (all of these rows are spread over the whole width,
    # which one ranked tile cannot hold); the count includes the row that the hash workspace takes in the end
    searched = (ip > 1536) & (cnt <= SEARCH_CAP) & (ip <= 4 * cnt)
    assert searched[16] and not searched[17] and searched[18]
    assert st["dense_search_tiles"] == int(searched.sum())
    assert st["dense_direct_tiles"] == 1       # exactly the block at the threshold


@pytest.mark.parametrize("column_list", [1, 0])
def test_unsorted_and_repeated_b_rows_over_several_blocks(column_list):
    # B rows in arbitrary order with repeats, 20000 columns (three blocks), rows of more products than the
    # hash workspaces take: the dense workspace walks whole B rows per tile and filters by column
    from paper_2404_04541_amd import binding as sg
    A = W.random_csr(60, 900, 40, 91)
    B = W.random_csr(900, 20000, 120, 92, sort_rows=False, allow_duplicates=True)
    for force in (0, 3):
        got = gpu_product(A, B, force, options={sg.OPT_COLUMN_LIST: column_list})
        ref = assert_matches_oracle(A, B, got, what=f"unsorted wide force={force} list={column_list}")
        assert int(ref.ip.max()) > 1536 and got[3]["dense_tiles"] > 0


def test_unsorted_b_with_a_row_too_long_is_refused():
    from paper_2404_04541_amd import binding as sg
    n = 1 << 21
    long_row = np.arange(n, dtype=np.int32)[::-1].copy()      # descending: not sorted, 2^21 entries
    B = W.CSR(2, n, np.array([0, n, n + 1]), np.concatenate([long_row, np.array([5], np.int32)]), np.ones(n + 1))
    A = W.CSR(1, 2, np.array([0, 2]), np.array([0, 1], np.int32), np.ones(2))
    h = sg.Handle()
    with pytest.raises(sg.SpgemmError) as e:
        sg.spgemm_symbolic(h, sg.to_device(A), sg.to_device(B))
    assert e.value.status == -4
    # the same row ascending is fine
    B2 = W.CSR(2, n, B.rowptr, np.concatenate([long_row[::-1], np.array([5], np.int32)]), B.values)
    got = gpu_product(A, B2, handle=h)
    assert_matches_oracle(A, B2, got, what="long ascending row")
