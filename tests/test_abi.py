"""Host-side checks of the C ABI that need no GPU: the built library loads, exports every
symbol that include/spgemm.h declares, and rejects bad arguments before its first HIP call."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "spgemm.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:spgemm|sptensor|spttm)[a-z_0-9]*)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    from paper_2404_04541_amd import binding as sg
    if not os.path.exists(sg.LIB_PATH):
        from paper_2404_04541_amd.build import build_library
        build_library()
    return sg.load_library()


def test_every_declared_symbol_is_exported(lib):
    from paper_2404_04541_amd import binding as sg
    names = declared_functions()
    assert "spgemm_symbolic" in names and "spgemm_numeric" in names and "spgemm" in names
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in spgemm.h but not exported"
    assert sorted(sg.EXPORTED) == names, "binding.EXPORTED and the header disagree"
    assert lib.spgemm_version() >= 100


def test_struct_layouts_match_the_header():
    from paper_2404_04541_amd import binding as sg
    text = open(HEADER).read()
    classes = re.search(r"enum \{\s*SPGEMM_K_COUNT = 0,(.*?)SPGEMM_NUM_KERNEL_CLASSES", text, re.S).group(1)
    n_classes = 1 + len(re.findall(r"SPGEMM_K_[A-Z_]+,", classes))
    assert n_classes == sg.NUM_KERNEL_CLASSES == len(sg.KERNEL_CLASS_NAMES)
    assert int(re.search(r"#define SPGEMM_NUM_BINS (\d+)", text).group(1)) == sg.NUM_BINS
    assert C.sizeof(sg.CsrStruct) == 3 * 8 + 3 * 8 + 8  # three sizes, three pointers, dtype padded to 8
    want = 2 * 8 + 5 * 8 * sg.NUM_BINS + 8 * sg.NUM_KERNEL_CLASSES + 4 * sg.NUM_KERNEL_CLASSES
    want = (want + 7) // 8 * 8 + 7 * 8
    assert C.sizeof(sg.StatsStruct) == want


def _csr(rows, cols, nnz, dtype=1, rowptr=1, colidx=1, values=1):
    from paper_2404_04541_amd import binding as sg
    # argument checks never dereference the pointers: any non-null value will do
    return sg.CsrStruct(rows, cols, nnz, rowptr or None, colidx or None, values or None, dtype)


def test_argument_errors_come_before_any_gpu_work(lib):
    h = C.c_void_p()
    assert lib.spgemm_create(None, None, None) == -1
    assert lib.spgemm_create(C.byref(h), None, None) == 0
    plan, nnz = C.c_void_p(), C.c_int64()
    rp = C.c_void_p(8)

    def sym(a, b, rowptr=rp):
        return lib.spgemm_symbolic(h, C.byref(a) if a is not None else None, C.byref(b) if b is not None else None,
                                   rowptr, C.byref(nnz), C.byref(plan))

    good = _csr(4, 4, 3)
    assert sym(None, good) == -1                               # null operand
    assert sym(_csr(-1, 4, 0), good) == -1                     # negative size
    assert sym(_csr(4, 4, 3, dtype=7), good) == -1             # unknown value type
    assert sym(_csr(4, 4, 3, rowptr=0), good) == -1            # null rowptr
    assert sym(_csr(4, 4, 3, colidx=0), good) == -1            # null colidx with nnz > 0
    assert sym(_csr(4, 5, 3), good) == -2                      # A.cols != B.rows
    assert sym(_csr(4, 4, 3, dtype=0), good) == -3             # value types differ
    assert sym(_csr(2**31, 4, 0), _csr(4, 4, 0)) == -4         # too many rows
    assert sym(good, good, rowptr=None) == -1                  # null output
    assert b"null" in lib.spgemm_last_error(h)
    assert lib.spgemm_numeric(h, None, C.byref(good), C.byref(good), rp, rp, rp) == -1   # null plan
    assert lib.spgemm(h, C.byref(good), C.byref(good), None) == -1
    assert lib.spgemm_set_option(h, 99, 0) == -1
    assert lib.spgemm_set_option(h, 2, 5) == -1                # workspace kinds are 0..4
    assert lib.spgemm_set_option(h, 2, 4) == 0
    assert lib.spgemm_set_option(h, 1, 2) == -1                # timing takes 0 or 1
    assert lib.spgemm_set_option(h, 3, 255) == -1              # direct-tile threshold: 256 or more
    assert lib.spgemm_set_option(h, 4, 100) == -1              # column list: 0, 1 or a byte limit >= 4096
    assert lib.spgemm_set_option(h, 4, 1 << 20) == 0
    assert lib.spgemm_set_option(h, 6, -1) == -1               # products per entry for searched tiles: 0 or more
    assert lib.spgemm_get_stats(None, None) == -1
    assert lib.spgemm_plan_destroy(None) == -1
    assert lib.spgemm_destroy(h) == 0
    assert lib.spgemm_destroy(None) == -1


def test_missing_library_is_an_error_not_a_fallback(monkeypatch):
    from paper_2404_04541_amd import binding as sg
    monkeypatch.setattr(sg, "_lib", None)
    monkeypatch.setattr(sg, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libspgemm_gfx950.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        sg.load_library()
