"""The entry point that allocates nothing (sptensor_unfold_noalloc) against sptensor_unfold, through
the C ABI: two calls in a row on one handle, the second with a smaller input, so that whatever the
first call left in the library's fixed scratch array is still there when the second one runs."""
import numpy as np
import pytest

from paper_2404_04541_amd import workloads as W

pytestmark = pytest.mark.gpu


def tensor(shape, nnz, seed):
    import torch
    idx = np.arange(nnz, dtype=np.uint64)
    c = [torch.from_numpy(W.rand_below(seed, 1 + a, idx, shape[a]).astype(np.int32)).cuda() for a in range(3)]
    v = torch.from_numpy(W.draw_values(nnz, -1.0, 1.0, np.float64, seed, 4)).cuda()
    return c, v


def test_no_alloc_unfolding_matches_the_allocating_one_twice():
    import torch
    from paper_2404_04541_amd import binding as sg
    h_ref = sg.Handle()
    h = sg.Handle(torch_allocator=False)   # no allocator callback: any allocation would have to be hipMalloc
    for shape, nnz, mode, seed in (((300, 200, 5000), 700_000, 3, 1), ((40, 50, 60), 9_000, 1, 2)):
        (xi, xj, xk), v = tensor(shape, nnz, seed)
        ref = sg.sptensor_unfold(h_ref, mode, shape, xi, xj, xk, v)
        rp = torch.full((ref.rows + 1,), -1, dtype=torch.int64, device="cuda")
        col = torch.full((nnz,), -1, dtype=torch.int32, device="cuda")
        val = torch.full((nnz,), float("nan"), dtype=torch.float64, device="cuda")
        before = torch.cuda.memory_allocated()
        sg.sptensor_unfold_noalloc(h, mode, shape, xi, xj, xk, v, rp, col, val)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(rp, ref.rowptr) and torch.equal(col, ref.colidx) and torch.equal(val, ref.values)
    # beyond the fixed scratch: a clear error, nothing run
    (xi, xj, xk), v = tensor((2000, 2000, 2000), sg.NOALLOC_MAX_NNZ + 1, 3)
    rp = torch.empty(2000 * 2000 + 1, dtype=torch.int64, device="cuda")
    col = torch.empty(v.numel(), dtype=torch.int32, device="cuda")
    val = torch.empty_like(v)
    with pytest.raises(sg.SpgemmError) as e:
        sg.sptensor_unfold_noalloc(h, 3, (2000, 2000, 2000), xi, xj, xk, v, rp, col, val)
    assert e.value.status == -4 and "at most" in str(e.value)
    # a coordinate out of range is still reported, and the next call is unaffected
    (xi, xj, xk), v = tensor((10, 10, 10), 100, 4)
    xi[5] = 10
    rp = torch.empty(101, dtype=torch.int64, device="cuda"); col = torch.empty(100, dtype=torch.int32, device="cuda"); val = torch.empty_like(v)
    with pytest.raises(sg.SpgemmError) as e:
        sg.sptensor_unfold_noalloc(h, 3, (10, 10, 10), xi, xj, xk, v, rp, col, val)
    assert e.value.status == -8
    xi[5] = 9
    ref = sg.sptensor_unfold(h_ref, 3, (10, 10, 10), xi, xj, xk, v)
    sg.sptensor_unfold_noalloc(h, 3, (10, 10, 10), xi, xj, xk, v, rp, col, val)
    torch.cuda.synchronize()
    assert torch.equal(rp, ref.rowptr) and torch.equal(col, ref.colidx) and torch.equal(val, ref.values)
