"""Thin Python binding of the C ABI in include/spgemm.h (argument marshalling only).

torch supplies device memory and the stream; every step of the product runs in the
HIP library.  There is no fallback: without the built library this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspgemm_gfx950.so")

SPGEMM_F32, SPGEMM_F64 = 0, 1
OPT_TIMING, OPT_FORCE_WORKSPACE, OPT_DIRECT_MIN, OPT_COLUMN_LIST, OPT_BLOCK_TABLE, OPT_SEARCH_RATIO = 1, 2, 3, 4, 5, 6
WORKSPACE_AUTO, WORKSPACE_SORTED_LIST, WORKSPACE_HASH, WORKSPACE_DENSE, WORKSPACE_STAGED = 0, 1, 2, 3, 4
NUM_KERNEL_CLASSES = 11
NUM_BINS = 8
KERNEL_CLASS_NAMES = ("count", "bin", "sym_esc", "sym_hash", "sym_dense", "scan", "num_esc", "num_hash", "num_dense", "num_staged", "block_ptr")

STATUS_NAMES = {0: "OK", -1: "INVALID_ARG", -2: "DIM_MISMATCH", -3: "DTYPE_MISMATCH", -4: "UNSUPPORTED",
                -5: "ALLOC_FAILED", -6: "HIP_ERROR", -7: "BAD_STATE", -8: "INVALID_INPUT"}

EXPORTED = ("spgemm_create", "spgemm_destroy", "spgemm_set_option", "spgemm_symbolic", "spgemm_numeric", "spgemm",
            "spgemm_free_device", "spgemm_plan_destroy", "spgemm_get_stats", "spgemm_last_error", "spgemm_version",
            "sptensor_unfold_mode3", "spttm_mode3", "sptensor_fold_mode3", "sptensor_unfold", "spttm", "sptensor_fold", "sptensor_unfold_noalloc",
            "spgemm_dcsr_from_csr", "spgemm_dcsc_from_csr", "spgemm_dcs_free", "spgemm_outer", "spgemm_pipelined")


class SpgemmError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


class CsrStruct(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("nnz", C.c_int64), ("rowptr", C.c_void_p),
                ("colidx", C.c_void_p), ("values", C.c_void_p), ("dtype", C.c_int32)]


ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_void_p, C.c_size_t)
FREE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class AllocatorStruct(C.Structure):
    _fields_ = [("alloc", ALLOC_FN), ("free", FREE_FN), ("ctx", C.c_void_p)]


class DcsStruct(C.Structure):
    _fields_ = [("major_dim", C.c_int64), ("minor_dim", C.c_int64), ("nvec", C.c_int64), ("nnz", C.c_int64), ("vec", C.c_void_p),
                ("ptr", C.c_void_p), ("idx", C.c_void_p), ("values", C.c_void_p), ("dtype", C.c_int32)]


class StatsStruct(C.Structure):
    _fields_ = [("ip_total", C.c_int64), ("nnz_c", C.c_int64), ("sym_bin_rows", C.c_int64 * NUM_BINS),
                ("num_bin_rows", C.c_int64 * NUM_BINS), ("sym_bin_ip", C.c_int64 * NUM_BINS),
                ("num_bin_ip", C.c_int64 * NUM_BINS), ("num_bin_nnz", C.c_int64 * NUM_BINS), ("kernel_ms", C.c_double * NUM_KERNEL_CLASSES),
                ("kernel_launches", C.c_int32 * NUM_KERNEL_CLASSES), ("dense_tiles", C.c_int64),
                ("dense_direct_tiles", C.c_int64), ("dense_runs", C.c_int64), ("dense_search_tiles", C.c_int64),
                ("plan_bytes", C.c_int64), ("plan_list_bytes", C.c_int64), ("plan_list_used", C.c_int64)]


_lib = None


def load_library():
    """Load the built library (raises if it has not been built: there is no other path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2404_04541_amd.build` "
                           "(or __graft_entry__.build()); this package has no CPU fallback")
    lib = C.CDLL(LIB_PATH)
    P = C.POINTER
    lib.spgemm_create.argtypes = [P(C.c_void_p), C.c_void_p, P(AllocatorStruct)]
    lib.spgemm_destroy.argtypes = [C.c_void_p]
    lib.spgemm_set_option.argtypes = [C.c_void_p, C.c_int, C.c_int64]
    lib.spgemm_symbolic.argtypes = [C.c_void_p, P(CsrStruct), P(CsrStruct), C.c_void_p, P(C.c_int64), P(C.c_void_p)]
    lib.spgemm_numeric.argtypes = [C.c_void_p, C.c_void_p, P(CsrStruct), P(CsrStruct), C.c_void_p, C.c_void_p, C.c_void_p]
    lib.spgemm.argtypes = [C.c_void_p, P(CsrStruct), P(CsrStruct), P(CsrStruct)]
    lib.spgemm_free_device.argtypes = [C.c_void_p, C.c_void_p]
    lib.spgemm_plan_destroy.argtypes = [C.c_void_p]
    lib.spgemm_get_stats.argtypes = [C.c_void_p, P(StatsStruct)]
    tensor_args = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
    lib.sptensor_unfold_mode3.argtypes = tensor_args + [P(CsrStruct)]
    lib.spttm_mode3.argtypes = tensor_args + [P(CsrStruct), P(CsrStruct)]
    lib.sptensor_fold_mode3.argtypes = [C.c_void_p, C.c_int64, P(CsrStruct), C.c_void_p, C.c_void_p]
    mode_args = [C.c_void_p, C.c_int] + tensor_args[1:]
    lib.sptensor_unfold.argtypes = mode_args + [P(CsrStruct)]
    lib.spttm.argtypes = mode_args + [P(CsrStruct), P(CsrStruct)]
    lib.sptensor_unfold_noalloc.argtypes = mode_args + [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.sptensor_fold.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, P(CsrStruct), C.c_void_p, C.c_void_p, C.c_void_p]
    lib.spgemm_dcsr_from_csr.argtypes = [C.c_void_p, P(CsrStruct), P(DcsStruct)]
    lib.spgemm_dcsc_from_csr.argtypes = [C.c_void_p, P(CsrStruct), P(DcsStruct)]
    lib.spgemm_dcs_free.argtypes = [C.c_void_p, P(DcsStruct)]
    lib.spgemm_outer.argtypes = [C.c_void_p, P(DcsStruct), P(DcsStruct), C.c_int64, P(CsrStruct)]
    lib.spgemm_pipelined.argtypes = [C.c_void_p, P(CsrStruct), P(CsrStruct), C.c_int, P(CsrStruct), P(C.c_int64)]
    lib.spgemm_last_error.argtypes = [C.c_void_p]
    lib.spgemm_last_error.restype = C.c_char_p
    for name in EXPORTED:
        if name != "spgemm_last_error":
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


@dataclass
class DeviceCSR:
    """CSR operand held in torch device tensors (rowptr int64, colidx int32, values f32/f64)."""
    rows: int
    cols: int
    rowptr: torch.Tensor
    colidx: torch.Tensor
    values: torch.Tensor

    @property
    def nnz(self) -> int:
        return int(self.colidx.numel())

    def struct(self) -> CsrStruct:
        dt = {torch.float32: SPGEMM_F32, torch.float64: SPGEMM_F64}[self.values.dtype]
        assert self.rowptr.dtype == torch.int64 and self.colidx.dtype == torch.int32
        assert self.rowptr.is_contiguous() and self.colidx.is_contiguous() and self.values.is_contiguous()
        n = self.nnz
        return CsrStruct(self.rows, self.cols, n, self.rowptr.data_ptr(), self.colidx.data_ptr() if n else None,
                         self.values.data_ptr() if n else None, dt)


def to_device(csr, device="cuda") -> DeviceCSR:
    """Copy a host CSR (attributes rows, cols, rowptr, colidx, values as numpy arrays) to the GPU."""
    return DeviceCSR(int(csr.rows), int(csr.cols),
                     torch.from_numpy(np.ascontiguousarray(csr.rowptr, dtype=np.int64)).to(device),
                     torch.from_numpy(np.ascontiguousarray(csr.colidx, dtype=np.int32)).to(device),
                     torch.from_numpy(np.ascontiguousarray(csr.values)).to(device))


class Plan:
    def __init__(self, handle: "Handle", ptr: int, nnz_c: int):
        self.handle, self.ptr, self.nnz_c = handle, ptr, nnz_c

    def stats(self) -> dict:
        st = StatsStruct()
        self.handle._check(self.handle.lib.spgemm_get_stats(self.ptr, C.byref(st)))
        return {"ip_total": int(st.ip_total), "nnz_c": int(st.nnz_c),
                "sym_bin_rows": list(st.sym_bin_rows), "num_bin_rows": list(st.num_bin_rows),
                "sym_bin_ip": list(st.sym_bin_ip), "num_bin_ip": list(st.num_bin_ip), "num_bin_nnz": list(st.num_bin_nnz),
                "kernel_ms": dict(zip(KERNEL_CLASS_NAMES, st.kernel_ms)),
                "kernel_launches": dict(zip(KERNEL_CLASS_NAMES, st.kernel_launches)),
                "dense_tiles": int(st.dense_tiles), "dense_direct_tiles": int(st.dense_direct_tiles),
                "dense_runs": int(st.dense_runs), "dense_search_tiles": int(st.dense_search_tiles),
                "plan_bytes": int(st.plan_bytes), "plan_list_bytes": int(st.plan_list_bytes), "plan_list_used": int(st.plan_list_used)}

    def destroy(self):
        if self.ptr:
            self.handle.lib.spgemm_plan_destroy(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Handle:
    """spgemm_create / spgemm_destroy.  Device memory for scratch and results comes from torch."""

    def __init__(self, stream: Optional[torch.cuda.Stream] = None, torch_allocator: bool = True):
        self.lib = load_library()
        self.stream = stream
        self._live = {}
        self._alloc_struct = None
        if torch_allocator:
            def _alloc(_ctx, nbytes):
                try:
                    with torch.cuda.stream(self.stream) if self.stream is not None else _nullctx():
                        t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device="cuda")
                except Exception:
                    return None
                self._live[t.data_ptr()] = t
                return t.data_ptr()

            def _free(_ctx, ptr):
                self._live.pop(ptr, None)

            self._cb = (ALLOC_FN(_alloc), FREE_FN(_free))
            self._alloc_struct = AllocatorStruct(self._cb[0], self._cb[1], None)
        h = C.c_void_p()
        sp = C.c_void_p(stream.cuda_stream) if stream is not None else None
        rc = self.lib.spgemm_create(C.byref(h), sp, C.byref(self._alloc_struct) if self._alloc_struct else None)
        if rc != 0:
            raise SpgemmError(rc, "spgemm_create failed")
        self.ptr = h

    def _check(self, rc: int):
        if rc != 0:
            raise SpgemmError(rc, self.lib.spgemm_last_error(self.ptr).decode())

    def set_option(self, option: int, value: int):
        self._check(self.lib.spgemm_set_option(self.ptr, option, value))

    def adopt(self, ptr: int, nbytes: int, dtype: torch.dtype) -> torch.Tensor:
        """Take over a buffer that the library obtained through the allocator callback."""
        t = self._live.pop(ptr)
        return t[:nbytes].view(dtype)

    def close(self):
        if self.ptr:
            self.lib.spgemm_destroy(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class _nullctx:
    def __enter__(self):
        return None

    def __exit__(self, *a):
        return False


def spgemm_symbolic(handle: Handle, A: DeviceCSR, B: DeviceCSR, c_rowptr: Optional[torch.Tensor] = None):
    """-> (c_rowptr int64 device tensor, nnz_c, Plan)."""
    if c_rowptr is None:
        c_rowptr = torch.empty(A.rows + 1, dtype=torch.int64, device=A.rowptr.device)
    sa, sb = A.struct(), B.struct()
    nnz = C.c_int64(0)
    plan = C.c_void_p()
    handle._check(handle.lib.spgemm_symbolic(handle.ptr, C.byref(sa), C.byref(sb), c_rowptr.data_ptr(), C.byref(nnz),
                                             C.byref(plan)))
    return c_rowptr, int(nnz.value), Plan(handle, plan, int(nnz.value))


def spgemm_numeric(handle: Handle, plan: Plan, A: DeviceCSR, B: DeviceCSR, c_rowptr: torch.Tensor,
                   c_colidx: Optional[torch.Tensor] = None, c_values: Optional[torch.Tensor] = None):
    """-> (c_colidx int32, c_values) device tensors of plan.nnz_c elements (allocated when not given)."""
    n = plan.nnz_c
    if c_colidx is None:
        c_colidx = torch.empty(n, dtype=torch.int32, device=A.rowptr.device)
    if c_values is None:
        c_values = torch.empty(n, dtype=A.values.dtype, device=A.rowptr.device)
    sa, sb = A.struct(), B.struct()
    handle._check(handle.lib.spgemm_numeric(handle.ptr, plan.ptr, C.byref(sa), C.byref(sb), c_rowptr.data_ptr(),
                                            c_colidx.data_ptr() if n else None, c_values.data_ptr() if n else None))
    return c_colidx, c_values


def spgemm(handle: Handle, A: DeviceCSR, B: DeviceCSR) -> DeviceCSR:
    """C = A * B through the library's single entry point; result buffers come from the handle's allocator."""
    if handle._alloc_struct is None:
        raise RuntimeError("spgemm() through this binding needs the torch allocator (results are adopted as tensors)")
    sa, sb, sc = A.struct(), B.struct(), CsrStruct()
    handle._check(handle.lib.spgemm(handle.ptr, C.byref(sa), C.byref(sb), C.byref(sc)))
    vdt = A.values.dtype
    vsz = 4 if vdt == torch.float32 else 8
    rowptr = handle.adopt(sc.rowptr, (sc.rows + 1) * 8, torch.int64)
    if sc.nnz:
        colidx = handle.adopt(sc.colidx, sc.nnz * 4, torch.int32)
        values = handle.adopt(sc.values, sc.nnz * vsz, vdt)
    else:
        colidx = torch.empty(0, dtype=torch.int32, device=rowptr.device)
        values = torch.empty(0, dtype=vdt, device=rowptr.device)
    return DeviceCSR(int(sc.rows), int(sc.cols), rowptr, colidx, values)


def _adopt_csr(handle: Handle, sc: CsrStruct, vdt: torch.dtype, device) -> DeviceCSR:
    vsz = 4 if vdt == torch.float32 else 8
    rowptr = handle.adopt(sc.rowptr, (sc.rows + 1) * 8, torch.int64)
    if sc.nnz:
        colidx = handle.adopt(sc.colidx, sc.nnz * 4, torch.int32)
        values = handle.adopt(sc.values, sc.nnz * vsz, vdt)
    else:
        colidx = torch.empty(0, dtype=torch.int32, device=device)
        values = torch.empty(0, dtype=vdt, device=device)
    return DeviceCSR(int(sc.rows), int(sc.cols), rowptr, colidx, values)


def _tensor_args(handle, shape, xi, xj, xk, xval):
    I, J, K = (int(v) for v in shape)
    n = int(xval.numel())
    for t in (xi, xj, xk):
        assert t.dtype == torch.int32 and t.is_contiguous() and t.numel() == n
    assert xval.is_contiguous()
    dt = {torch.float32: SPGEMM_F32, torch.float64: SPGEMM_F64}[xval.dtype]
    ptr = lambda t: t.data_ptr() if n else None
    return [handle.ptr, I, J, K, n, ptr(xi), ptr(xj), ptr(xk), ptr(xval), dt]


def sptensor_unfold_mode3(handle: Handle, shape, xi, xj, xk, xval) -> DeviceCSR:
    """Mode-3 unfolding of a coordinate tensor (device int32 coordinates, values): (I*J) x K CSR."""
    sc = CsrStruct()
    handle._check(handle.lib.sptensor_unfold_mode3(*_tensor_args(handle, shape, xi, xj, xk, xval), C.byref(sc)))
    return _adopt_csr(handle, sc, xval.dtype, xval.device)


def spttm_mode3(handle: Handle, shape, xi, xj, xk, xval, M: DeviceCSR) -> DeviceCSR:
    """Y = X x_3 M as the unfolded (I*J) x M.cols CSR (row i*J + j holds Y(i,j,:))."""
    sm, sc = M.struct(), CsrStruct()
    handle._check(handle.lib.spttm_mode3(*_tensor_args(handle, shape, xi, xj, xk, xval), C.byref(sm), C.byref(sc)))
    return _adopt_csr(handle, sc, xval.dtype, xval.device)


def sptensor_fold_mode3(handle: Handle, J: int, Y: DeviceCSR):
    """-> (yi, yj) int32 device tensors: first two coordinates of every entry of the unfolded Y."""
    yi = torch.empty(Y.nnz, dtype=torch.int32, device=Y.rowptr.device)
    yj = torch.empty(Y.nnz, dtype=torch.int32, device=Y.rowptr.device)
    sy = Y.struct()
    handle._check(handle.lib.sptensor_fold_mode3(handle.ptr, int(J), C.byref(sy), yi.data_ptr() if Y.nnz else None,
                                                 yj.data_ptr() if Y.nnz else None))
    return yi, yj


def _mode_args(handle, mode, shape, xi, xj, xk, xval):
    a = _tensor_args(handle, shape, xi, xj, xk, xval)
    return [a[0], int(mode)] + a[1:]


def sptensor_unfold(handle: Handle, mode: int, shape, xi, xj, xk, xval) -> DeviceCSR:
    """Unfolding of a coordinate tensor over `mode` (1, 2 or 3): the two kept coordinates fold into the row."""
    sc = CsrStruct()
    handle._check(handle.lib.sptensor_unfold(*_mode_args(handle, mode, shape, xi, xj, xk, xval), C.byref(sc)))
    return _adopt_csr(handle, sc, xval.dtype, xval.device)


def spttm(handle: Handle, mode: int, shape, xi, xj, xk, xval, M: DeviceCSR) -> DeviceCSR:
    """Y = X x_mode M as the unfolded CSR matrix."""
    sm, sc = M.struct(), CsrStruct()
    handle._check(handle.lib.spttm(*_mode_args(handle, mode, shape, xi, xj, xk, xval), C.byref(sm), C.byref(sc)))
    return _adopt_csr(handle, sc, xval.dtype, xval.device)


def sptensor_fold(handle: Handle, mode: int, shape, Y: DeviceCSR):
    """-> (yi, yj, yk) int32 device tensors: the coordinates of every entry of Y, the unfolding over `mode`
    of a tensor of extents `shape`."""
    out = [torch.empty(Y.nnz, dtype=torch.int32, device=Y.rowptr.device) for _ in range(3)]
    sy = Y.struct()
    I, J, K = (int(v) for v in shape)
    handle._check(handle.lib.sptensor_fold(handle.ptr, int(mode), I, J, K, C.byref(sy), *[t.data_ptr() if Y.nnz else None for t in out]))
    return tuple(out)


NOALLOC_MAX_NNZ = 1 << 20


def sptensor_unfold_noalloc(handle: Handle, mode: int, shape, xi, xj, xk, xval, out_rowptr, out_colidx, out_values):
    """sptensor_unfold into caller-owned device tensors, without any allocation inside the library."""
    n = int(xval.numel())
    assert out_rowptr.dtype == torch.int64 and out_colidx.dtype == torch.int32 and out_values.dtype == xval.dtype
    assert out_colidx.numel() >= n and out_values.numel() >= n
    handle._check(handle.lib.sptensor_unfold_noalloc(*_mode_args(handle, mode, shape, xi, xj, xk, xval), out_rowptr.data_ptr(),
                                                     out_colidx.data_ptr() if n else None, out_values.data_ptr() if n else None))


@dataclass
class DeviceDCS:
    """Doubly compressed sparse rows or columns held in torch device tensors."""
    major_dim: int
    minor_dim: int
    vec: torch.Tensor      # int32, the kept vectors' indices
    ptr: torch.Tensor      # int64, len(vec) + 1
    idx: torch.Tensor      # int32
    values: torch.Tensor

    def struct(self) -> DcsStruct:
        dt = {torch.float32: SPGEMM_F32, torch.float64: SPGEMM_F64}[self.values.dtype]
        nv, n = int(self.vec.numel()), int(self.idx.numel())
        return DcsStruct(self.major_dim, self.minor_dim, nv, n, self.vec.data_ptr() if nv else None, self.ptr.data_ptr(),
                         self.idx.data_ptr() if n else None, self.values.data_ptr() if n else None, dt)


def _adopt_dcs(handle: Handle, sd: DcsStruct, vdt: torch.dtype) -> DeviceDCS:
    vsz = 4 if vdt == torch.float32 else 8
    # (the library allocates nvec + 1 slots for vec so that an empty list still has a buffer)
    vec = handle.adopt(sd.vec, (sd.nvec + 1) * 4, torch.int32)[:sd.nvec]
    ptr = handle.adopt(sd.ptr, (sd.nvec + 1) * 8, torch.int64)
    idx = handle.adopt(sd.idx, max(sd.nnz, 0) * 4, torch.int32)
    val = handle.adopt(sd.values, max(sd.nnz, 0) * vsz, vdt)
    return DeviceDCS(int(sd.major_dim), int(sd.minor_dim), vec, ptr, idx, val)


def dcsr_from_csr(handle: Handle, M: DeviceCSR) -> DeviceDCS:
    sm, sd = M.struct(), DcsStruct()
    handle._check(handle.lib.spgemm_dcsr_from_csr(handle.ptr, C.byref(sm), C.byref(sd)))
    return _adopt_dcs(handle, sd, M.values.dtype)


def dcsc_from_csr(handle: Handle, M: DeviceCSR) -> DeviceDCS:
    sm, sd = M.struct(), DcsStruct()
    handle._check(handle.lib.spgemm_dcsc_from_csr(handle.ptr, C.byref(sm), C.byref(sd)))
    return _adopt_dcs(handle, sd, M.values.dtype)


def spgemm_outer(handle: Handle, A: DeviceDCS, B: DeviceDCS, acc_capacity: int = 0) -> DeviceCSR:
    """C = A * B by outer products through the insert / sort / merge / compress stages (A doubly compressed columns,
    B doubly compressed rows)."""
    sa, sb, sc = A.struct(), B.struct(), CsrStruct()
    handle._check(handle.lib.spgemm_outer(handle.ptr, C.byref(sa), C.byref(sb), int(acc_capacity), C.byref(sc)))
    return _adopt_csr(handle, sc, A.values.dtype, A.ptr.device)


def spgemm_pipelined(handle: Handle, A: DeviceCSR, B: DeviceCSR, nblocks: int):
    """C = A * B as row blocks, symbolic of block t + 1 overlapped with numeric of block t.
    -> (list of DeviceCSR blocks, list of nblocks + 1 first-row indices)."""
    sa, sb = A.struct(), B.struct()
    blocks = (CsrStruct * nblocks)()
    first = (C.c_int64 * (nblocks + 1))()
    handle._check(handle.lib.spgemm_pipelined(handle.ptr, C.byref(sa), C.byref(sb), int(nblocks), blocks, first))
    return [_adopt_csr(handle, blocks[t], A.values.dtype, A.rowptr.device) for t in range(nblocks)], list(first)
