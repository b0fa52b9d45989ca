"""The row-block pipeline (symbolic of block t + 1 on a second stream while numeric of block t runs)
against the single-pass product and the CPU checker: stacked, the blocks are the same matrix."""
import numpy as np
import pytest

import oracle
from paper_2404_04541_amd import workloads as W
from helpers import RTOL

pytestmark = pytest.mark.gpu


def stacked(blocks, first):
    rp = [np.zeros(1, np.int64)]
    base = 0
    for b, lo, hi in zip(blocks, first[:-1], first[1:]):
        assert b.rows == hi - lo
        r = b.rowptr.cpu().numpy()
        assert r[0] == 0 and r[-1] == b.nnz
        rp.append(r[1:] + base)
        base += b.nnz
    col = np.concatenate([b.colidx.cpu().numpy() for b in blocks])
    val = np.concatenate([b.values.cpu().numpy() for b in blocks])
    return np.concatenate(rp), col, val


@pytest.mark.parametrize("case", ["ragged", "power law", "rectangular f32"])
def test_pipeline_blocks_stack_to_the_single_pass_result(case):
    import torch
    from paper_2404_04541_amd import binding as sg
    if case == "ragged":
        A, B = W.random_csr(3000, 2500, 12, 5), W.random_csr(2500, 4000, 30, 6)
    elif case == "power law":
        A, B = W.config3(scale=14)
    else:
        A, B = W.random_csr(5003, 3001, 40, 7, dtype=np.float32), W.random_csr(3001, 7777, 25, 8, dtype=np.float32)
    h = sg.Handle()
    dA = sg.to_device(A)
    dB = dA if B is A else sg.to_device(B)
    single = sg.spgemm(h, dA, dB)
    ref = oracle.spgemm(A, B)
    ip_prefix = np.concatenate([[0], np.cumsum(ref.ip + 1)])
    for nblocks in (1, 2, 5, 16):
        blocks, first = sg.spgemm_pipelined(h, dA, dB, nblocks)
        torch.cuda.synchronize()
        assert first[0] == 0 and first[-1] == A.rows and all(a <= b for a, b in zip(first, first[1:]))
        rp, col, val = stacked(blocks, first)
        # bit-identical structure to the single pass and to the checker
        assert np.array_equal(rp, single.rowptr.cpu().numpy()) and np.array_equal(col, single.colidx.cpu().numpy())
        assert np.array_equal(rp, ref.rowptr) and np.array_equal(col, ref.colidx)
        want = ref.values.astype(A.values.dtype).astype(np.float64)
        assert np.all(np.abs(val.astype(np.float64) - want) <= RTOL[np.dtype(A.values.dtype)] * ref.absum)
        # blocks of about equal work: no block holds much more than its share plus one row
        work = np.diff(ip_prefix[first])
        assert work.max() <= ip_prefix[-1] / nblocks + (ref.ip.max() + 1) + 1


def test_pipeline_more_blocks_than_rows_and_empty_operands():
    import torch
    from paper_2404_04541_amd import binding as sg
    h = sg.Handle()
    A, B = W.random_csr(5, 40, 3, 11), W.random_csr(40, 30, 4, 12)
    blocks, first = sg.spgemm_pipelined(h, sg.to_device(A), sg.to_device(B), 9)
    torch.cuda.synchronize()
    ref = oracle.spgemm(A, B)
    rp, col, val = stacked(blocks, first)
    assert np.array_equal(rp, ref.rowptr) and np.array_equal(col, ref.colidx)
    Z = W.CSR(6, 40, np.zeros(7, np.int64), np.zeros(0, np.int32), np.zeros(0))
    blocks, first = sg.spgemm_pipelined(h, sg.to_device(Z), sg.to_device(B), 3)
    assert sum(b.nnz for b in blocks) == 0 and first[-1] == 6
    with pytest.raises(sg.SpgemmError) as e:
        sg.spgemm_pipelined(h, sg.to_device(A), sg.to_device(B), 0)
    assert e.value.status == -1
