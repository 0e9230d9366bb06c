"""The C-ABI library loads and exports every symbol the header declares; argument
checks that need no GPU answer with the documented codes (no compute calls)."""
import ctypes
import os
import re

import pytest

from paper_1903_01042_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _has_gpu():
    import torch
    return torch.cuda.is_available()


def _declared():
    text = open(os.path.join(ROOT, "include", "codenet.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(codenet_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_1903_01042_amd import build
        build.build_library(verbose=False)
    return B.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert set(names) == set(B.EXPORTS), (names, B.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_struct_layouts_match_the_header():
    # codenet_report: 2 ints + MAX_T ints + MAX_R floats + 1 float; codenet_fault: 4 ints, 2 u64, 3 floats, 1 int
    assert ctypes.sizeof(B.Report) == 4 * (2 + B.MAX_T + B.MAX_R + 1)
    assert ctypes.sizeof(B.Fault) == 48
    assert B.Fault.seed.offset == 16 and B.Fault.lo.offset == 32
    text = open(os.path.join(ROOT, "include", "codenet.h")).read()
    for name, val in (("CODENET_MAX_T", B.MAX_T), ("CODENET_MAX_R", B.MAX_R), ("CODENET_MAX_L", B.MAX_L),
                      ("CODENET_MAX_FAULTS", B.MAX_FAULTS)):
        assert re.search(r"#define\s+%s\s+%d\b" % (name, val), text), name
    # enumerators the binding restates
    for name, val in (("CODENET_CLEAN", B.CLEAN), ("CODENET_CORRECTED", B.CORRECTED),
                      ("CODENET_UNCORRECTABLE", B.UNCORRECTABLE), ("CODENET_DISAGREE", B.DISAGREE),
                      ("CODENET_FWD", B.FWD), ("CODENET_BWD", B.BWD), ("CODENET_WEIGHT", B.WEIGHT),
                      ("CODENET_CHECK", B.CHECK), ("CODENET_CHECK_EVALUATION", B.CHECK_EVALUATION),
                      ("CODENET_CHECK_LIST", B.CHECK_LIST), ("CODENET_EPI_MUL", B.EPI_MUL),
                      ("CODENET_E_ALLOC", B.E_ALLOC)):
        assert re.search(r"\b%s\s*=\s*%d\b" % (name, val), text), name


def test_argument_errors_without_a_gpu(lib):
    h = ctypes.c_void_p(0)
    assert lib.codenet_encode(None, None, None, ctypes.byref(h)) == B.E_NULL
    d = B.Desc(0, 8, 2, 2, 0, 0, None, None, B.F32, 4, 1e-3, 1e-2)
    fake = ctypes.c_void_p(16)          # never dereferenced: the shape check comes first
    assert lib.codenet_encode(ctypes.byref(d), fake, None, ctypes.byref(h)) == B.E_SHAPE
    d = B.Desc(8, 8, 2, 2, 0, 0, None, None, 7, 4, 1e-3, 1e-2)
    assert lib.codenet_encode(ctypes.byref(d), fake, None, ctypes.byref(h)) == B.E_DTYPE
    d = B.Desc(8, 8, 2, 2, 0, 0, None, None, B.F32, 0, 1e-3, 1e-2)
    assert lib.codenet_encode(ctypes.byref(d), fake, None, ctypes.byref(h)) == B.E_BATCH
    d = B.Desc(8, 8, 2, 2, 9, 0, None, None, B.F32, 4, 1e-3, 1e-2)
    assert lib.codenet_encode(ctypes.byref(d), fake, None, ctypes.byref(h)) == B.E_CODE
    # rows 0 and 1 of P are equal: a zero 2x2 minor, not MDS
    P = (ctypes.c_double * 6)(1.0, 2.0, 1.0, 2.0, 1.0, 3.0)
    d = B.Desc(9, 9, 3, 3, 2, 2, P, P, B.F32, 4, 1e-3, 1e-2)
    assert lib.codenet_encode(ctypes.byref(d), fake, None, ctypes.byref(h)) == B.E_CODE
    # the MDS test is relative to the scale of the generator (Hadamard's bound on each minor): a tiny
    # but well conditioned P is accepted (the call then goes on to the GPU, which answers differently
    # with and without one -- anything but E_CODE), a huge one with nearly dependent rows is refused
    good = [1.0, 1.0, 1.0, 2.0, 1.0, 3.0]
    tiny = (ctypes.c_double * 6)(*[1e-6 * v for v in good])
    d = B.Desc(9, 9, 3, 3, 2, 2, tiny, tiny, B.F32, 4, 1e-3, 2e-3)
    if not _has_gpu():
        assert lib.codenet_encode(ctypes.byref(d), fake, None, ctypes.byref(h)) != B.E_CODE
    huge = (ctypes.c_double * 6)(1e6, 2e6, 1e6, 2e6 * (1 + 1e-12), 1e6, 3e6)
    d = B.Desc(9, 9, 3, 3, 2, 2, huge, huge, B.F32, 4, 1e-3, 2e-3)
    assert lib.codenet_encode(ctypes.byref(d), fake, None, ctypes.byref(h)) == B.E_CODE
    # a code too long to enumerate (C(32, k) C(8, k) minors per order) is checked by sampling: a
    # generator with two equal rows is still refused (every order k >= 2 has minors on those rows)
    rng = __import__("numpy").random.default_rng(1)
    big = rng.standard_normal((32, 8))
    big[7] = big[19]
    arr = (ctypes.c_double * 256)(*big.reshape(-1))
    d = B.Desc(64, 64, 32, 32, 8, 8, arr, arr, B.F32, 4, 1e-3, 2e-3)
    assert lib.codenet_encode(ctypes.byref(d), fake, None, ctypes.byref(h)) == B.E_CODE
    assert lib.codenet_forward(None, None, 1, None, None) == B.E_NULL
    assert lib.codenet_update(None, 0.1, None) == B.E_NULL
    assert lib.codenet_destroy(None) == B.E_NULL
    assert lib.codenet_strerror(B.E_CODE).decode().startswith("generator")
    assert lib.codenet_strerror(0).decode() == "ok"
