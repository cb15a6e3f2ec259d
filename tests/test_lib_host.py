"""Host-side checks of libdion.so that need no GPU: the library loads, exports every symbol that
include/dion.h declares, and its host-only entry points validate their arguments."""
import ctypes as C
import os
import re

import pytest

from paper_2504_05295_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2504_05295_amd import build
        build.build(verbose=False)
    return B.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dion.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dion_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree(lib):
    names = declared_functions()
    assert "dion_step" in names and "dion_step_batched" in names and "dion_init_state" in names
    assert sorted(B.EXPORTS) == names
    for n in names:
        assert getattr(lib, n) is not None        # raises AttributeError if the symbol is missing


def test_strerror(lib):
    assert B.strerror(0) == "ok"
    assert "argument" in B.strerror(B.DION_EINVAL)
    assert "Cholesky" in B.strerror(B.DION_NUM_BREAKDOWN)
    assert B.strerror(12345) == "unknown code"


def test_workspace_bytes_validation(lib):
    ok = B.dion_workspace_bytes([(256, 256, 64)], B.DION_G_F32, B.DION_MATH_F32)
    assert ok > 0 and ok % 256 == 0
    big = B.dion_workspace_bytes([(256, 256, 64), (512, 256, 64)], B.DION_G_F32, B.DION_MATH_F32)
    assert big > ok
    assert B.dion_workspace_bytes([], B.DION_G_F32, B.DION_MATH_F32) >= 0
    for bad in [(0, 4, 1), (4, 0, 1), (4, 4, 0), (4, 4, 5), (8, 3, 4), (-1, 4, 1)]:
        with pytest.raises(B.DionError) as e:
            B.dion_workspace_bytes([bad], B.DION_G_F32, B.DION_MATH_F32)
        assert e.value.code == B.DION_EINVAL
    with pytest.raises(B.DionError):
        B.dion_workspace_bytes([(8, 8, 2)], 7, B.DION_MATH_F32)
    with pytest.raises(B.DionError):
        B.dion_workspace_bytes([(8, 8, 2)], B.DION_G_F32, 9)
    out = C.c_size_t(0)
    assert lib.dion_workspace_bytes(1, None, None, None, 0, 0, C.byref(out)) == B.DION_EINVAL
    assert lib.dion_workspace_bytes(0, None, None, None, 0, 0, None) == B.DION_EINVAL


def test_null_state_is_rejected(lib):
    assert lib.dion_step(None, None, None, None, None, 4, 4, 2, 0.9, 0.1, None) == B.DION_EINVAL
    assert lib.dion_step_batched(None, 0, None, None, None, None, None, None, None, 0.9, 0.1, None) == B.DION_EINVAL
    assert lib.dion_last_status(None, None, None) == B.DION_EINVAL
    assert lib.dion_set_stage_timing(None, 1) == B.DION_EINVAL
    assert lib.dion_stage_times(None, None) == B.DION_EINVAL
    assert lib.dion_destroy_state(None) == B.DION_OK
    h = C.c_void_p(None)
    assert lib.dion_init_state(None, 0, None, None, None, 0, 0, None, 0, None, None, 1, 0, None) == B.DION_EINVAL
    assert lib.dion_init_state(C.byref(h), 1, None, None, None, 0, 0, None, 0, None, None, 1, 0, None) == B.DION_EINVAL
