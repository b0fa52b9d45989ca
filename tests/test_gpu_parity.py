"""GPU parity: the HIP library (through the C ABI) against the CPU checker, element by element."""
import numpy as np
import pytest

import oracle
from paper_2404_04541_amd import workloads as W
from helpers import gpu_product, assert_matches_oracle

pytestmark = pytest.mark.gpu

AUTO, LIST, HASH, DENSE, STAGED = 0, 1, 2, 3, 4


def run(A, B, force=AUTO, what="", via="phases", options=None):
    got = gpu_product(A, B, force, via=via, options=options)
    ref = assert_matches_oracle(A, B, got, what=what)
    st = got[3]
    if st is not None:
        assert st["ip_total"] == int(ref.ip.sum())
        assert st["nnz_c"] == int(ref.cnt.sum())
    return st


def test_config1_random_1000():
    a, b = W.config1()
    st = run(a, b, what="config1")
    assert st["sym_bin_rows"][1] == 1000  # ip = 100 per row: the one-wave sorted-list bin


@pytest.mark.parametrize("force", [AUTO, LIST, HASH, DENSE, STAGED])
def test_every_workspace_computes_the_same_function(force):
    # ragged rows from empty to a few thousand products: crosses every bin boundary
    A = W.random_csr(3000, 2500, 12, 5)
    B = W.random_csr(2500, 4000, 30, 6)
    run(A, B, force, what=f"ragged force={force}")


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_ragged_tail_and_many_tiles(dtype):
    A = W.random_csr(5003, 3001, 40, 7, dtype=dtype)
    B = W.random_csr(3001, 7777, 25, 8, dtype=dtype)
    run(A, B, what="ragged tails")


@pytest.mark.parametrize("seed", range(12))
def test_randomized_shapes_every_route(seed):
    # seeded shapes and densities from tiny to a few thousand products per row, rectangular, both value
    # types, every forced route: the same C from all of them
    u = W.rand_unit(seed, 900, np.arange(8, dtype=np.uint64))
    m, k, n = (1 + int(v * 1500) for v in u[:3])
    da, db = 1 + u[3] * 30, 1 + u[4] * 60
    dtype = np.float32 if seed % 2 else np.float64
    A = W.random_csr(m, k, da, seed, 910, dtype=dtype, sort_rows=seed % 3 != 0, allow_duplicates=seed % 4 == 0)
    B = W.random_csr(k, n * (40 if seed % 5 == 0 else 1), db, seed, 920, dtype=dtype, sort_rows=seed % 3 != 1,
                     allow_duplicates=seed % 4 == 1)
    ref = None
    for force in (AUTO, LIST, HASH, DENSE, STAGED):
        got = gpu_product(A, B, force)
        ref = assert_matches_oracle(A, B, got, ref=ref, what=f"seed {seed} force={force} {m}x{k}x{B.cols}")


def test_hash_retrieval_with_columns_too_wide_to_pack():
    # beyond 2^20 (large class) and 2^23 (small class) columns the hash workspace sorts (column, sum)
    # pairs instead of packed (column, slot) words
    A = W.random_csr(500, 400, 8, 81)
    run(A, W.random_csr(400, 3_000_000, 40, 82), HASH, what="hash, 3M columns")
    run(A, W.random_csr(400, 9_000_000, 10, 83), HASH, what="hash, 9M columns")


def test_sorted_list_keys_too_wide_to_pack():
    # beyond 2^25 (short list) and 2^23 (long list) columns a key of the sorted-list workspace cannot
    # carry its list position; equal columns are then ordered by position while they are counted.
    # Few distinct columns spread over a wide range: nearly every product has partners to merge with.
    stretch = 700_001
    for a_mean, b_mean, seed in ((3, 5, 84), (6, 12, 86)):   # products per row mostly <= 32, resp. mostly 33..128
        A = W.random_csr(600, 400, a_mean, seed)
        B0 = W.random_csr(400, 60, b_mean, seed + 1)
        B = W.CSR(400, 60 * stretch, B0.rowptr, (B0.colidx.astype(np.int64) * stretch).astype(np.int32), B0.values)
        for force in (AUTO, LIST):
            st = run(A, B, force, what=f"wide sorted-list keys, means {a_mean}/{b_mean}, force={force}")
            assert st["num_bin_rows"][0] + st["num_bin_rows"][1] > 300
        # the same structure with narrow columns takes the packed route
        run(A, B0, LIST, what="narrow sorted-list keys")


def test_sorted_list_rows_with_many_a_entries():
    # rows of up to 128 products made of many A entries with B rows of one or two entries: the one-wave class
    # takes its A entries 64 at a time, and a batch of at most 16 entries deals products instead of entries
    # to the lanes; 70 = a full batch and a short one, 16 / 17 = both sides of that limit
    k = 300
    degs = [70, 100, 17, 16, 15, 64, 65, 128, 1, 40] * 12
    rowptr = np.zeros(len(degs) + 1, dtype=np.int64)
    np.cumsum(degs, out=rowptr[1:])
    nnz = int(rowptr[-1])
    cols = np.concatenate([np.sort(W.rand_below(87, 1, np.arange(i * 1000, i * 1000 + 4 * d, dtype=np.uint64), k)[:d])
                           for i, d in enumerate(degs)]).astype(np.int32)
    A = W.CSR(len(degs), k, rowptr, cols, W.draw_values(nnz, -1.0, 1.0, np.float64, 87, 2))
    lens = 1 + (np.arange(k) % 7 == 0)   # one entry per B row, two in every seventh
    bp = np.zeros(k + 1, dtype=np.int64)
    np.cumsum(lens, out=bp[1:])
    bcol = W.rand_below(87, 3, np.arange(int(bp[-1]), dtype=np.uint64), 50).astype(np.int32)
    B = W.CSR(k, 50, bp, bcol, W.draw_values(int(bp[-1]), -1.0, 1.0, np.float64, 87, 4))
    for force in (AUTO, LIST):
        st = run(A, B, force, what=f"many A entries, force={force}")
    assert st["num_bin_rows"][1] >= 60


def test_stencil_small_grid():
    a, b = W.config2(g=12)
    st = run(a, b, what="stencil 12^3")
    assert st["ip_total"] == (9 * 12 - 10) ** 3 and st["nnz_c"] == (5 * 12 - 6) ** 3


@pytest.mark.parametrize("force", [AUTO, DENSE, STAGED])
def test_rmat_small_scale_power_law(force):
    a, b = W.config3(scale=13)
    st = run(a, b, force, what=f"rmat scale 13 force={force}")
    if force == AUTO:
        assert sum(st["num_bin_rows"][5:7]) > 0, "long rows must reach the dense workspace"
    if force == STAGED:
        assert st["num_bin_rows"][4] > 0, "rows of few products must reach the staged coordinate list"


def test_rectangular_and_ttm_small():
    a, b = W.config4(rows=20000, bcols=512)
    run(a, b, what="config4 small")
    a, m = W.config5(dim=64, nnz=40000)
    run(a, m, what="config5 small")


@pytest.mark.parametrize("column_list", [1, 0])
@pytest.mark.parametrize("direct_min", [6144, 256, 1 << 20])
def test_dense_tiles_direct_ranked_with_and_without_column_list(column_list, direct_min):
    # power-law rows: dense heads (direct tiles) and sparse tails (ranked tiles) in the same rows;
    # the ranked tiles take their structure from the plan's column list or rebuild it themselves
    from paper_2404_04541_amd import binding as sg
    a, b = W.config3(scale=15)
    st = run(a, b, DENSE, what=f"rmat 15 dense list={column_list} direct_min={direct_min}",
             options={sg.OPT_COLUMN_LIST: column_list, sg.OPT_DIRECT_MIN: direct_min})
    ranked = st["dense_tiles"] - st["dense_search_tiles"] - st["dense_direct_tiles"]
    assert ranked > 0 or direct_min == 256, "hub rows need ranked tiles unless every block counts as dense"
    if column_list == 0:
        assert st["dense_search_tiles"] == 0   # searched tiles need the list
    if direct_min == 256:
        assert st["dense_direct_tiles"] > 0
    if direct_min == 1 << 20:
        assert st["dense_direct_tiles"] == 0


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_short_rows_over_many_columns_become_searched_tiles(dtype):
    # a few thousand entries per row of C spread over a million columns: several ranked tiles by width,
    # one searched tile by entry count (ranks by bisection of the plan's column list)
    from paper_2404_04541_amd import binding as sg
    A = W.random_csr(300, 3000, 6, 71, dtype=dtype)
    B = W.random_csr(3000, 1_000_000, 500, 72, dtype=dtype)
    st = run(A, B, AUTO, what="searched tiles")
    assert st["dense_search_tiles"] > 0
    st = run(A, B, AUTO, what="searched tiles off", options={sg.OPT_SEARCH_RATIO: 0})
    assert st["dense_search_tiles"] == 0 and st["dense_tiles"] > 0
    # a list too small for all rows: some searched, the others through the staged or ranked routes
    st = run(A, B, AUTO, what="searched tiles, small list", options={sg.OPT_COLUMN_LIST: 1 << 18})
    assert 0 < st["dense_search_tiles"] < 300


def test_column_list_too_small_for_all_rows():
    # a list of 256 KB holds the columns of some rows only: the others take the routes that need no list
    from paper_2404_04541_amd import binding as sg
    a, b = W.config3(scale=14)
    for force in (AUTO, DENSE):
        st = run(a, b, force, what=f"small list force={force}", options={sg.OPT_COLUMN_LIST: 1 << 18})
        assert st["dense_tiles"] > 0


@pytest.mark.parametrize("column_list", [1, 0])
def test_without_block_table_pieces_are_bisected(column_list):
    from paper_2404_04541_amd import binding as sg
    a, b = W.config3(scale=14)
    run(a, b, DENSE, what="no block table", options={sg.OPT_BLOCK_TABLE: 0, sg.OPT_COLUMN_LIST: column_list})
    A = W.random_csr(24, 6000, 1500, 61)
    B = W.random_csr(6000, 2_500_000, 40, 62)
    run(A, B, DENSE, what="no block table, wide", options={sg.OPT_BLOCK_TABLE: 0, sg.OPT_COLUMN_LIST: column_list})


def test_wide_matrix_several_flag_list_spans_and_long_a_rows():
    # more than 2^20 columns (the symbolic flag list covers the row in several spans) and rows of A
    # with more entries than the numeric kernel keeps in registers
    from paper_2404_04541_amd import binding as sg
    A = W.random_csr(24, 6000, 1500, 61)
    B = W.random_csr(6000, 2_500_000, 40, 62)
    for force in (AUTO, DENSE):
        st = run(A, B, force, what=f"wide force={force}")
        assert st["dense_tiles"] > 0
    # shorter rows: every span of a row has few enough entries for one searched tile of its own
    A2 = W.random_csr(40, 6000, 300, 63)
    st = run(A2, B, DENSE, what="wide, searched tiles per span")
    assert st["dense_search_tiles"] > 40, "more searched tiles than rows: they are per span"
    # the same without the block-offset table (piece bounds by bisection) and with unordered B rows (whole
    # rows are walked for every span; no searched tiles then, a tile would see products of other spans)
    run(A2, B, DENSE, what="wide, no block table", options={sg.OPT_BLOCK_TABLE: 0})
    Bu = W.random_csr(6000, 2_500_000, 40, 62, sort_rows=False)
    st = run(A2, Bu, DENSE, what="wide, unordered B")
    assert st["dense_search_tiles"] == 0


@pytest.mark.parametrize("direct_min", [256, 1 << 20])
def test_dedup_sweep_operands_dense_and_sparse_routes(direct_min):
    # the paper's synthetic sweep at a reduced size
    from paper_2404_04541_amd import binding as sg
    B, C = W.dedup_sweep(4000, dense_elements=40_000_000, per_column=400)
    for force, ratio in ((AUTO, 4), (DENSE, 0), (DENSE, 1000000)):
        st = run(B, C, force, what=f"dedup sweep force={force} direct_min={direct_min} search_ratio={ratio}",
                 options={sg.OPT_DIRECT_MIN: direct_min, sg.OPT_SEARCH_RATIO: ratio})
        if ratio == 0:
            assert st["dense_search_tiles"] == 0


def test_dense_workspace_many_windows_and_tiles():
    # wide column space (several windows) and rows with more entries than one tile holds
    A = W.random_csr(40, 3000, 900, 11)
    B = W.random_csr(3000, 600000, 60, 12)
    run(A, B, DENSE, what="dense windows")
    B2 = W.random_csr(3000, 40000, 400, 13)
    st = run(A, B2, AUTO, what="dense tiles")
    assert sum(st["num_bin_rows"][5:7]) > 0


def test_unsorted_and_duplicate_inputs():
    A = W.random_csr(400, 300, 9, 21, sort_rows=False, allow_duplicates=True)
    B = W.random_csr(300, 500, 14, 22, sort_rows=False, allow_duplicates=True)
    for force in (AUTO, HASH, DENSE, STAGED):
        run(A, B, force, what=f"unsorted/duplicates force={force}")


def test_identity_and_permutation_exact():
    A = W.random_csr(700, 700, 15, 31)
    I = W.identity(700)
    P = W.permutation(700, 3)
    for X, Y in ((I, A), (A, I), (P, A), (A, P)):
        got = gpu_product(X, Y)
        ref = assert_matches_oracle(X, Y, got)
        assert np.array_equal(got[2], ref.values)  # one product per entry: bit-identical values


def test_explicit_zero_kept_and_empty_cases():
    A = W.CSR(1, 2, np.array([0, 2]), np.array([0, 1], np.int32), np.array([1.0, 1.0]))
    B = W.CSR(2, 2, np.array([0, 1, 3]), np.array([0, 0, 1], np.int32), np.array([1.0, -1.0, 5.0]))
    rp, col, val, _ = gpu_product(A, B)
    assert rp.tolist() == [0, 2] and col.tolist() == [0, 1] and val.tolist() == [0.0, 5.0]
    Z = W.CSR(5, 4, np.zeros(6, np.int64), np.zeros(0, np.int32), np.zeros(0))
    Bn = W.random_csr(4, 6, 2, 0)
    for X, Y in ((Z, Bn), (W.random_csr(5, 4, 2, 1), W.CSR(4, 6, np.zeros(5, np.int64), np.zeros(0, np.int32), np.zeros(0))),
                 (W.CSR(0, 4, np.zeros(1, np.int64), np.zeros(0, np.int32), np.zeros(0)), Bn)):
        rp, col, val, _ = gpu_product(X, Y)
        assert rp.tolist() == [0] * (X.rows + 1) and col.size == 0 and val.size == 0


def test_single_call_entry_point_and_plan_reuse():
    import torch
    from paper_2404_04541_amd import binding as sg
    A = W.random_csr(1500, 1200, 10, 41)
    B = W.random_csr(1200, 1800, 12, 42)
    run(A, B, via="single", what="spgemm()")
    h = sg.Handle()
    dA, dB = sg.to_device(A), sg.to_device(B)
    rp, nnz, plan = sg.spgemm_symbolic(h, dA, dB)
    col1, val1 = sg.spgemm_numeric(h, plan, dA, dB, rp)
    dA2 = sg.DeviceCSR(dA.rows, dA.cols, dA.rowptr, dA.colidx, dA.values * 2.0)
    col2, val2 = sg.spgemm_numeric(h, plan, dA2, dB, rp)
    torch.cuda.synchronize()
    # sums are accumulated with LDS atomics, so their order (not their structure) may change from run to run
    assert torch.equal(col1, col2) and torch.allclose(val2, val1 * 2.0, rtol=1e-12, atol=1e-14)


def test_invalid_input_is_reported_not_executed():
    import torch
    from paper_2404_04541_amd import binding as sg
    A = W.random_csr(100, 80, 5, 51)
    B = W.random_csr(80, 90, 5, 52)
    h = sg.Handle()
    dA, dB = sg.to_device(A), sg.to_device(B)
    bad = dB.colidx.clone(); bad[3] = 90  # column == cols
    with pytest.raises(sg.SpgemmError) as e:
        sg.spgemm_symbolic(h, dA, sg.DeviceCSR(dB.rows, dB.cols, dB.rowptr, bad, dB.values))
    assert e.value.status == -8
    badrp = dA.rowptr.clone(); badrp[10] = badrp[11] + 1
    with pytest.raises(sg.SpgemmError) as e:
        sg.spgemm_symbolic(h, sg.DeviceCSR(dA.rows, dA.cols, badrp, dA.colidx, dA.values), dB)
    assert e.value.status == -8
    # the handle stays usable
    rp, nnz, plan = sg.spgemm_symbolic(h, dA, dB)
    assert nnz == int(oracle.spgemm(A, B).cnt.sum())
