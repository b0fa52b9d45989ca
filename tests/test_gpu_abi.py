"""C-ABI paths on the GPU that the torch-backed binding does not take by itself: a handle without an
allocator (the library's own hipMalloc / hipFree), a stream other than the default one, an allocator
that fails part-way, a numeric call with operands that are not the plan's."""
import ctypes as C

import numpy as np
import pytest

import oracle
from paper_2404_04541_amd import workloads as W
from helpers import assert_matches_oracle

pytestmark = pytest.mark.gpu


def hip_runtime():
    hip = C.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
    hip.hipMemcpy.restype = C.c_int
    hip.hipMemGetInfo.argtypes = [C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    return hip


def test_handle_without_allocator_uses_the_librarys_own_allocation():
    import torch
    from paper_2404_04541_amd import binding as sg
    A = W.random_csr(900, 700, 9, 201)
    B = W.random_csr(700, 5000, 40, 202)     # long rows too: the dense workspace and its plan lists are allocated as well
    lib = sg.load_library()
    h = C.c_void_p()
    assert lib.spgemm_create(C.byref(h), None, None) == 0
    dA, dB = sg.to_device(A), sg.to_device(B)
    sa, sb, sc = dA.struct(), dB.struct(), sg.CsrStruct()
    hip = hip_runtime()
    want = oracle.spgemm(A, B)
    nnz = int(want.cnt.sum())
    rp = torch.empty(A.rows + 1, dtype=torch.int64, device="cuda")
    col = torch.empty(nnz, dtype=torch.int32, device="cuda")
    val = torch.empty(nnz, dtype=torch.float64, device="cuda")
    free_after = []
    for attempt in range(2):     # (the first product also loads the kernels; the second must leave the same memory free)
        sc = sg.CsrStruct()
        assert lib.spgemm(h, C.byref(sa), C.byref(sb), C.byref(sc)) == 0, lib.spgemm_last_error(h)
        assert sc.nnz == nnz and sc.rows == A.rows
        for dst, src in ((rp, sc.rowptr), (col, sc.colidx), (val, sc.values)):
            assert hip.hipMemcpy(dst.data_ptr(), src, dst.numel() * dst.element_size(), 3) == 0   # device to device
        assert_matches_oracle(A, B, (rp.cpu().numpy(), col.cpu().numpy(), val.cpu().numpy()), ref=want, what="no allocator")
        for ptr in (sc.rowptr, sc.colidx, sc.values):
            assert lib.spgemm_free_device(h, ptr) == 0
        torch.cuda.synchronize()
        free, total = C.c_size_t(), C.c_size_t()
        hip.hipMemGetInfo(C.byref(free), C.byref(total))
        free_after.append(free.value)
    assert free_after[1] >= free_after[0] - (1 << 20), "the library kept device memory after its results were freed"
    assert lib.spgemm_destroy(h) == 0


def test_stream_other_than_the_default_one():
    import torch
    from paper_2404_04541_amd import binding as sg
    A = W.random_csr(2000, 1500, 12, 203, dtype=np.float32)
    B = W.random_csr(1500, 3000, 30, 204, dtype=np.float32)
    stream = torch.cuda.Stream()
    h = sg.Handle(stream=stream)
    with torch.cuda.stream(stream):
        dA, dB = sg.to_device(A), sg.to_device(B)
        stream.synchronize()
        rp, nnz, plan = sg.spgemm_symbolic(h, dA, dB)
        col, val = sg.spgemm_numeric(h, plan, dA, dB, rp)
    stream.synchronize()
    plan.destroy()
    assert_matches_oracle(A, B, (rp.cpu().numpy(), col.cpu().numpy(), val.cpu().numpy()), what="own stream")


def test_allocator_that_fails_part_way_leaves_nothing_behind():
    import torch
    from paper_2404_04541_amd import binding as sg
    A = W.random_csr(800, 600, 9, 205)
    B = W.random_csr(600, 4000, 40, 206)
    dA, dB = sg.to_device(A), sg.to_device(B)
    lib = sg.load_library()
    want = oracle.spgemm(A, B)
    calls = 0
    optional = 0
    n_ok = None
    for fail_at in range(1, 12):
        live, state = {}, {"n": 0}

        def alloc(_ctx, nbytes):
            state["n"] += 1
            if state["n"] == fail_at:
                return None
            t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device="cuda")
            live[t.data_ptr()] = t
            return t.data_ptr()

        def free(_ctx, ptr):
            assert ptr in live, "free of a pointer the allocator never gave out"
            del live[ptr]

        cb = (sg.ALLOC_FN(alloc), sg.FREE_FN(free))
        st = sg.AllocatorStruct(cb[0], cb[1], None)
        h = C.c_void_p()
        assert lib.spgemm_create(C.byref(h), None, C.byref(st)) == 0
        sa, sb, sc = dA.struct(), dB.struct(), sg.CsrStruct()
        rc = lib.spgemm(h, C.byref(sa), C.byref(sb), C.byref(sc))
        torch.cuda.synchronize()
        if rc == 0:
            assert len(live) == 3 and sc.nnz == int(want.cnt.sum())    # C's three arrays, nothing else
            for ptr in (sc.rowptr, sc.colidx, sc.values):
                lib.spgemm_free_device(h, ptr)
            assert not live
            lib.spgemm_destroy(h)
            if state["n"] < fail_at:       # the failing call was never reached: the sweep is over
                n_ok = state["n"]
                break
            # the plan's structure list is optional (the product goes on without it), and a refused allocation of C
            # makes the library plan again without that list and ask once more
            optional += 1
            continue
        # the optional structure list may be refused without failing the product; every other refusal is an error
        assert rc == -5, (fail_at, rc, lib.spgemm_last_error(h))
        assert not live, f"allocation {fail_at} failed and {len(live)} buffers were left behind"
        # the handle is still usable: same product with the failure behind us
        sc = sg.CsrStruct()
        assert lib.spgemm(h, C.byref(sa), C.byref(sb), C.byref(sc)) == 0
        torch.cuda.synchronize()
        assert sc.nnz == int(want.cnt.sum())
        for ptr in (sc.rowptr, sc.colidx, sc.values):
            lib.spgemm_free_device(h, ptr)
        assert not live
        lib.spgemm_destroy(h)
        calls += 1
    assert n_ok is not None and calls >= 3 and optional <= 3, "the sweep never reached a run without a failing allocation"


def test_numeric_with_other_operands_than_the_plans():
    from paper_2404_04541_amd import binding as sg
    A = W.random_csr(300, 200, 5, 207)
    B = W.random_csr(200, 250, 6, 208)
    A2 = W.random_csr(300, 200, 6, 209)     # other structure, same shape
    B2 = W.random_csr(200, 260, 6, 210)     # other width
    h = sg.Handle()
    dA, dB = sg.to_device(A), sg.to_device(B)
    rp, nnz, plan = sg.spgemm_symbolic(h, dA, dB)
    for X, Y in ((sg.to_device(A2), dB), (dA, sg.to_device(B2))):
        with pytest.raises(sg.SpgemmError) as e:
            sg.spgemm_numeric(h, plan, X, Y, rp)
        assert e.value.status == -2
    other = sg.Handle()
    with pytest.raises(sg.SpgemmError) as e:
        sg.spgemm_numeric(other, plan, dA, dB, rp)
    assert e.value.status == -7
    col, val = sg.spgemm_numeric(h, plan, dA, dB, rp)     # the plan is still good
    import torch
    torch.cuda.synchronize()
    assert_matches_oracle(A, B, (rp.cpu().numpy(), col.cpu().numpy(), val.cpu().numpy()), what="after refused calls")
    plan.destroy()
