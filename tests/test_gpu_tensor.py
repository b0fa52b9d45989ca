"""GPU parity of the sparse tensor-times-matrix entry points (mode-3 unfolding on the GPU, the
row-wise product, folding back) against the CPU checker."""
import numpy as np
import pytest

import oracle
from paper_2404_04541_amd import workloads as W
from helpers import RTOL

pytestmark = pytest.mark.gpu


def to_dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def coords(shape, nnz, seed, distinct):
    I, J, K = shape
    idx = np.arange(nnz, dtype=np.uint64)
    xi = W.rand_below(seed, 1, idx, I).astype(np.int32)
    xj = W.rand_below(seed, 2, idx, J).astype(np.int32)
    xk = W.rand_below(seed, 3, idx, K).astype(np.int32)
    if distinct:
        lin = (xi.astype(np.int64) * J + xj) * K + xk
        _, first = np.unique(lin, return_index=True)
        first.sort()
        xi, xj, xk = xi[first], xj[first], xk[first]
    return xi, xj, xk


@pytest.mark.parametrize("shape,nnz,distinct,dtype", [((7, 5, 11), 150, True, np.float64), ((40, 33, 300), 50000, False, np.float64),
                                                      ((300, 200, 70000), 400000, True, np.float32), ((3, 3, 3), 0, True, np.float64)])
def test_unfold_ttm_fold(shape, nnz, distinct, dtype):
    import torch
    from paper_2404_04541_amd import binding as sg
    I, J, K = shape
    xi, xj, xk = coords(shape, nnz, 7, distinct)
    vals = W.draw_values(xi.size, -1.0, 1.0, dtype, 7, 4)
    M = W.random_csr(K, 500, 6, 9, dtype=dtype)
    h = sg.Handle()
    dxi, dxj, dxk, dv = to_dev(xi), to_dev(xj), to_dev(xk), to_dev(vals)
    U = sg.sptensor_unfold_mode3(h, shape, dxi, dxj, dxk, dv)
    rp, col, val = oracle.unfold_mode3(shape, xi, xj, xk, vals)
    assert (U.rows, U.cols) == (I * J, K)
    assert np.array_equal(U.rowptr.cpu().numpy(), rp) and np.array_equal(U.colidx.cpu().numpy(), col)
    assert np.array_equal(U.values.cpu().numpy(), val)   # a stable sort: repeated coordinates keep their input order
    Y = sg.spttm_mode3(h, shape, dxi, dxj, dxk, dv, sg.to_device(M))
    torch.cuda.synchronize()
    ref = oracle.spttm_mode3(shape, xi, xj, xk, vals, M)
    assert np.array_equal(Y.rowptr.cpu().numpy(), ref.rowptr) and np.array_equal(Y.colidx.cpu().numpy(), ref.colidx)
    want = ref.values.astype(dtype).astype(np.float64)
    err = np.abs(Y.values.cpu().numpy().astype(np.float64) - want)
    assert np.all(err <= RTOL[np.dtype(dtype)] * ref.absum)
    yi, yj = sg.sptensor_fold_mode3(h, J, Y)
    torch.cuda.synchronize()
    rows = np.repeat(np.arange(I * J), np.diff(ref.rowptr))
    assert np.array_equal(yi.cpu().numpy(), (rows // J).astype(np.int32)) and np.array_equal(yj.cpu().numpy(), (rows % J).astype(np.int32))


def test_coordinate_out_of_range_is_reported():
    from paper_2404_04541_amd import binding as sg
    h = sg.Handle()
    xi, xj, xk = (to_dev(np.array(v, dtype=np.int32)) for v in ([0, 1], [0, 5], [1, 1]))
    with pytest.raises(sg.SpgemmError) as e:
        sg.sptensor_unfold_mode3(h, (2, 5, 3), xi, xj, xk, to_dev(np.array([1.0, 2.0])))
    assert e.value.status == -8


def test_config5_through_the_tensor_entry_point():
    # the full-size tensor of configuration 5 from its unordered coordinates: the unfolding and the product
    # against the CPU checker (its own unfolding of the same coordinates, then its row-wise product), whole
    import torch
    from paper_2404_04541_amd import binding as sg
    from test_gpu_full_configs import check_whole
    x = W.coo3_uniform((2048, 2048, 2048), 10_000_000, 0, 40, np.float64)
    m = W.uniform_rows(2048, 2048, 16, 0, 44, np.float64)
    order = np.argsort(W.rand_u64(0, 77, np.arange(x.values.size, dtype=np.uint64)), kind="stable")   # hand the entries over unordered
    xi, xj, xk, xv = (v[order] for v in (x.i, x.j, x.k, x.values))
    h = sg.Handle()
    dxi, dxj, dxk, dv = (to_dev(v) for v in (xi, xj, xk, xv))
    U = sg.sptensor_unfold_mode3(h, x.shape, dxi, dxj, dxk, dv)
    rp, col, val = oracle.unfold(x.shape, 3, xi, xj, xk, xv)
    assert np.array_equal(U.rowptr.cpu().numpy(), rp) and np.array_equal(U.colidx.cpu().numpy(), col)
    assert np.array_equal(U.values.cpu().numpy(), val)
    Y = sg.spttm_mode3(h, x.shape, dxi, dxj, dxk, dv, sg.to_device(m))
    torch.cuda.synchronize()
    assert Y.nnz > 150_000_000
    a = W.CSR(2048 * 2048, 2048, rp, col, val)
    check_whole(a, m, gpu=(Y.rowptr, Y.colidx, Y.values, Y.nnz, {"ip_total": 10_000_000 * 16}))

@pytest.mark.parametrize("mode", [1, 2, 3])
@pytest.mark.parametrize("shape,nnz,distinct,dtype", [((9, 6, 13), 300, False, np.float64), ((120, 90, 4000), 200000, True, np.float32),
                                                      ((4, 4, 4), 0, True, np.float64), ((1, 700, 33), 5000, False, np.float64)])
def test_unfold_ttm_fold_every_mode(mode, shape, nnz, distinct, dtype):
    import torch
    from paper_2404_04541_amd import binding as sg
    xi, xj, xk = coords(shape, nnz, 17 + mode, distinct)
    vals = W.draw_values(xi.size, -1.0, 1.0, dtype, 17, 4)
    L = 37
    M = W.random_csr(shape[mode - 1], L, 5, 19, dtype=dtype)
    h = sg.Handle()
    dxi, dxj, dxk, dv = to_dev(xi), to_dev(xj), to_dev(xk), to_dev(vals)
    U = sg.sptensor_unfold(h, mode, shape, dxi, dxj, dxk, dv)
    rp, col, val = oracle.unfold(shape, mode, xi, xj, xk, vals)
    assert (U.rows, U.cols) == (rp.size - 1, shape[mode - 1])
    assert np.array_equal(U.rowptr.cpu().numpy(), rp) and np.array_equal(U.colidx.cpu().numpy(), col)
    assert np.array_equal(U.values.cpu().numpy(), val)
    Y = sg.spttm(h, mode, shape, dxi, dxj, dxk, dv, sg.to_device(M))
    torch.cuda.synchronize()
    ref = oracle.spttm(shape, mode, xi, xj, xk, vals, M)
    assert np.array_equal(Y.rowptr.cpu().numpy(), ref.rowptr) and np.array_equal(Y.colidx.cpu().numpy(), ref.colidx)
    want = ref.values.astype(dtype).astype(np.float64)
    err = np.abs(Y.values.cpu().numpy().astype(np.float64) - want)
    assert np.all(err <= RTOL[np.dtype(dtype)] * ref.absum)
    out_shape = list(shape); out_shape[mode - 1] = L
    got = sg.sptensor_fold(h, mode, out_shape, Y)
    torch.cuda.synchronize()
    for g, w in zip(got, oracle.fold(out_shape, mode, ref.rowptr, ref.colidx)):
        assert np.array_equal(g.cpu().numpy(), w)


def test_tensor_argument_errors():
    from paper_2404_04541_amd import binding as sg
    h = sg.Handle()
    xi, xj, xk = coords((5, 6, 7), 50, 3, True)
    vals = W.draw_values(xi.size, -1.0, 1.0, np.float64, 3, 4)
    d = [to_dev(x) for x in (xi, xj, xk, vals)]
    with pytest.raises(sg.SpgemmError) as e:
        sg.sptensor_unfold(h, 4, (5, 6, 7), *d)
    assert e.value.status == -1
    M = sg.to_device(W.random_csr(6, 9, 2, 1))     # rows match mode 2 only
    with pytest.raises(sg.SpgemmError) as e:
        sg.spttm(h, 3, (5, 6, 7), *d, M)
    assert e.value.status == -2
    Y = sg.spttm(h, 2, (5, 6, 7), *d, M)
    with pytest.raises(sg.SpgemmError) as e:
        sg.sptensor_fold(h, 1, (5, 9, 7), Y)        # Y is the mode-2 unfolding (35 x 9), not the mode-1 one
    assert e.value.status == -2
    bad = d[1].clone(); bad[0] = 6
    with pytest.raises(sg.SpgemmError) as e:
        sg.sptensor_unfold(h, 1, (5, 6, 7), d[0], bad, d[2], d[3])
    assert e.value.status == -8
