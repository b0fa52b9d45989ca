"""Shared pieces of the GPU parity tests: run the library through the C ABI binding, run the
CPU checker on the same operands, compare."""
import numpy as np

RTOL = {np.dtype(np.float64): 1e-12, np.dtype(np.float32): 1e-5}


def gpu_product(A, B, force=0, handle=None, via="phases", options=None):
    """C = A*B on the GPU through the binding. Returns (rowptr, colidx, values) numpy arrays and stats."""
    import torch
    from paper_2404_04541_amd import binding as sg
    h = handle or sg.Handle()
    h.set_option(sg.OPT_FORCE_WORKSPACE, force)
    for opt, value in (options or {}).items():
        h.set_option(opt, value)
    dA, dB = sg.to_device(A), sg.to_device(B)
    if via == "single":
        Cd = sg.spgemm(h, dA, dB)
        torch.cuda.synchronize()
        return Cd.rowptr.cpu().numpy(), Cd.colidx.cpu().numpy(), Cd.values.cpu().numpy(), None
    rp, nnz, plan = sg.spgemm_symbolic(h, dA, dB)
    col, val = sg.spgemm_numeric(h, plan, dA, dB, rp)
    torch.cuda.synchronize()
    st = plan.stats()
    plan.destroy()
    return rp.cpu().numpy(), col.cpu().numpy(), val.cpu().numpy(), st


def assert_matches_oracle(A, B, got, ref=None, what=""):
    """rowptr and colidx bit-exact; |value - ref| <= rtol * sum|a*b| (the componentwise bound of a
    recursive sum; equals rtol*|ref| when nothing cancels).  Reference values are the double sums
    rounded once to the operand type."""
    import oracle
    rp, col, val = got[:3]
    if ref is None:
        ref = oracle.spgemm(A, B)
    assert rp.dtype == np.int64 and col.dtype == np.int32 and val.dtype == A.values.dtype
    assert np.array_equal(rp, ref.rowptr), f"{what}: rowptr differs"
    assert np.array_equal(col, ref.colidx), f"{what}: colidx differs"
    rtol = RTOL[np.dtype(A.values.dtype)]
    want = ref.values.astype(A.values.dtype).astype(np.float64)
    err = np.abs(val.astype(np.float64) - want)
    bound = rtol * ref.absum
    bad = err > bound
    assert not bad.any(), f"{what}: {int(bad.sum())} values off, worst ratio {float((err / np.maximum(ref.absum, 1e-300)).max()):.3e}"
    return ref
