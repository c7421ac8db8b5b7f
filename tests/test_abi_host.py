"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and validates arguments before touching a device."""
import ctypes as ct
import os
import re

import pytest

from paper_2011_10170_amd import binding as B
from paper_2011_10170_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2011_10170_amd import build
        build.build()
    return B.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "pc.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(pc_[a-z_0-9]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    for s in range(0, 7):
        assert lib.pc_status_str(s)
    assert lib.pc_status_str(0) == b"ok"


def test_check_library():
    assert B.pc_check_library(list(I.make_library(8))) == B.PC_OK
    assert B.pc_check_library(list(I.make_library(126))) == B.PC_OK
    assert B.pc_check_library([0b111]) == B.PC_ERR_BAD_LIBRARY              # 3 taps
    assert B.pc_check_library([0b11111]) == B.PC_ERR_BAD_LIBRARY            # 5 taps
    assert B.pc_check_library([0b1000000111]) == B.PC_ERR_BAD_LIBRARY       # bit 9 set
    assert B.pc_check_library([0b1111, 0b1111]) == B.PC_ERR_BAD_LIBRARY     # duplicate
    assert B.pc_check_library([]) == B.PC_ERR_INVALID_ARG or B.pc_check_library([]) == B.PC_ERR_BAD_LIBRARY
    assert B.load().pc_check_library(None, 4) == B.PC_ERR_INVALID_ARG
    assert B.pc_check_library([0b1111] * 127) == B.PC_ERR_BAD_LIBRARY


def test_check_conv_desc():
    ok = B.make_desc(8, 32, 32, 16, 16, 1, B.PC_F32)
    assert B.pc_check_conv_desc(ok) == B.PC_OK
    assert B.pc_check_conv_desc(B.make_desc(8, 32, 32, 16, 16, 2, B.PC_BF16)) == B.PC_OK
    assert B.pc_check_conv_desc(B.make_desc(8, 32, 32, 16, 16, 3, B.PC_F32)) == B.PC_ERR_BAD_SHAPE
    assert B.pc_check_conv_desc(B.make_desc(0, 32, 32, 16, 16, 1, B.PC_F32)) == B.PC_ERR_BAD_SHAPE
    assert B.pc_check_conv_desc(B.make_desc(8, 32, 32, 70000, 16, 1, B.PC_F32)) == B.PC_ERR_BAD_SHAPE
    assert B.pc_check_conv_desc(B.make_desc(8, 32, 32, 16, 16, 1, 7)) == B.PC_ERR_INVALID_ARG
    assert B.load().pc_check_conv_desc(None) == B.PC_ERR_INVALID_ARG


def test_null_context_is_rejected(lib):
    d = B.make_desc(1, 4, 4, 4, 4, 1, B.PC_F32)
    assert lib.pc_conv_fwd(None, ct.byref(d), None, None, None) == B.PC_ERR_INVALID_ARG
    assert lib.pc_pattern_select(None, None, None, 1, 1, None, 1, 0, 0, 0, None, None) == B.PC_ERR_INVALID_ARG
    assert lib.pc_pack(None, None, None, None, 1, 1, None, 1, 0, None) == B.PC_ERR_INVALID_ARG
    lib.pc_destroy(None)
    lib.pc_packed_free(None)


def test_create_without_a_gpu_fails_cleanly(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    ctx = ct.c_void_p()
    assert lib.pc_create(ct.byref(ctx), 0, None) == B.PC_ERR_DEVICE
    assert not ctx.value
