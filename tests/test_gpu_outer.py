"""GPU parity of the outer-product route (k -> i -> j through the accumulation / all arrays) against the
CPU checker's outer-product route and its row-wise route; the doubly compressed conversions against the
checker's builders."""
import numpy as np
import pytest

import oracle
from oracle import outer
from paper_2404_04541_amd import workloads as W
from helpers import RTOL

pytestmark = pytest.mark.gpu


def run_outer(A, B, capacity=0, handle=None):
    import torch
    from paper_2404_04541_amd import binding as sg
    h = handle or sg.Handle()
    dA, dB = sg.to_device(A), sg.to_device(B)
    Ac = sg.dcsc_from_csr(h, dA)
    Br = sg.dcsr_from_csr(h, dB)
    C = sg.spgemm_outer(h, Ac, Br, capacity)
    torch.cuda.synchronize()
    return Ac, Br, C


def check_against_oracles(A, B, C, what):
    ref = oracle.spgemm(A, B)
    assert np.array_equal(C.rowptr.cpu().numpy(), ref.rowptr), f"{what}: rowptr differs"
    assert np.array_equal(C.colidx.cpu().numpy(), ref.colidx), f"{what}: colidx differs"
    want = ref.values.astype(A.values.dtype).astype(np.float64)
    err = np.abs(C.values.cpu().numpy().astype(np.float64) - want)
    assert np.all(err <= RTOL[np.dtype(A.values.dtype)] * ref.absum), f"{what}: values off"
    return ref


@pytest.mark.parametrize("seed", range(8))
def test_outer_route_small_every_capacity(seed):
    u = W.rand_unit(seed, 960, np.arange(4, dtype=np.uint64))
    m, k, n = (1 + int(v * 300) for v in u[:3])
    dtype = np.float32 if seed % 2 else np.float64
    A = W.random_csr(m, k, 1 + u[3] * 6, seed, 961, dtype=dtype, sort_rows=seed % 3 != 0, allow_duplicates=seed % 4 == 0)
    B = W.random_csr(k, n, 4, seed, 962, dtype=dtype, sort_rows=seed % 3 != 1, allow_duplicates=seed % 4 == 1)
    for cap in (0, 1, 37, 1000):
        Ac, Br, C = run_outer(A, B, cap)
        check_against_oracles(A, B, C, f"seed {seed} capacity {cap}")
    # the conversions against the checker's builders
    cols, ptr, rows, vals = outer.dcsc_from_csr(A)
    assert np.array_equal(Ac.vec.cpu().numpy(), cols) and np.array_equal(Ac.ptr.cpu().numpy(), ptr)
    assert np.array_equal(Ac.idx.cpu().numpy(), rows) and np.array_equal(Ac.values.cpu().numpy(), vals)
    r, rp, c, v = outer.dcsr_from_csr(B)
    assert np.array_equal(Br.vec.cpu().numpy(), r) and np.array_equal(Br.ptr.cpu().numpy(), rp)
    assert np.array_equal(Br.idx.cpu().numpy(), c) and np.array_equal(Br.values.cpu().numpy(), v)
    # and the checker's own outer-product route gives the same structure
    orp, ocol, oval, oabs, _ = outer.spgemm_outer(A, B, 1000)
    assert np.array_equal(C.rowptr.cpu().numpy(), orp) and np.array_equal(C.colidx.cpu().numpy(), ocol)


def test_outer_route_empty_rows_columns_and_operands():
    from paper_2404_04541_amd import binding as sg
    h = sg.Handle()
    # most rows of A and most rows of B empty; columns of A that meet no row of B and the reverse
    A = W.random_csr(5000, 4000, 0.05, 31)
    B = W.random_csr(4000, 3000, 0.08, 32)
    _, _, C = run_outer(A, B, handle=h)
    ref = check_against_oracles(A, B, C, "hypersparse")
    assert int(ref.cnt.sum()) < 100
    Z = W.CSR(7, 5, np.zeros(8, np.int64), np.zeros(0, np.int32), np.zeros(0))
    Bn = W.random_csr(5, 6, 2, 0)
    for X, Y in ((Z, Bn), (W.random_csr(7, 5, 2, 1), W.CSR(5, 6, np.zeros(6, np.int64), np.zeros(0, np.int32), np.zeros(0)))):
        Ac, Br, C = run_outer(X, Y, handle=h)
        assert C.rowptr.cpu().tolist() == [0] * 8 and C.nnz == 0 and (Ac.vec.numel() == 0 or Br.vec.numel() == 0)
    with pytest.raises(sg.SpgemmError) as e:
        sg.spgemm_outer(h, sg.dcsc_from_csr(h, sg.to_device(Bn)), sg.dcsr_from_csr(h, sg.to_device(Bn)))   # 6 columns against 5 rows
    assert e.value.status == -2


def test_outer_route_config1_and_a_rectangular_case_with_several_batches():
    a, b = W.config1()
    _, _, C = run_outer(a, b)
    check_against_oracles(a, b, C, "config 1")
    a, b = W.config4(rows=200000, bcols=4096)     # 6.4e6 products, rectangular result; batches of 2^20
    _, _, C = run_outer(a, b, 1 << 20)
    check_against_oracles(a, b, C, "rectangular, 7 batches")
    a, b = W.config3(scale=12)                    # power-law: long runs of equal coordinates in a batch
    _, _, C = run_outer(a, b, 1 << 18)
    check_against_oracles(a, b, C, "power law")
