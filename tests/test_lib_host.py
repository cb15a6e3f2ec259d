"""Host-side checks of libdion.so that need no GPU: the library loads, exports every symbol that
include/dion.h declares, and its host-only entry points validate their arguments."""
import ctypes as C
import os
import re
import subprocess

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


def test_wait_timeout_has_its_own_code(lib):
    assert B.DION_WAIT_TIMEOUT not in (B.DION_OK, B.DION_NUM_BREAKDOWN)
    assert "wait" in B.strerror(B.DION_WAIT_TIMEOUT)


def test_cholesky_grid_fits_the_compute_units(lib):
    """The single-launch factorisation needs all its workgroups resident at once: whatever the planner picks must
    fit the compute units it was told about, for any batch and rank, and it must fall back to a launch per panel
    (0) when nothing fits."""
    for cus in (1, 2, 7, 64, 104, 228, 256, 304, 1024):
        for batch in (1, 2, 3, 4, 5, 16, 28, 56, 112, 128, 129, 196, 256, 257, 1000):
            for r in (1, 63, 64, 255, 256, 257, 512, 768, 1024, 2048, 4096, 8192, 8193, 32768):
                w = B.dion_cholesky_grid(cus, batch, r)
                nb = (r + 63) // 64
                assert 0 <= w <= 256 and w * batch <= cus
                if nb < 4 or nb > 128 or cus // batch < 2:
                    assert w == 0
                elif cus // batch >= 2:
                    assert w >= 2
    assert B.dion_cholesky_grid(256, 1, 2048) == 256       # 15 x 17 helpers and the workgroup that carries the chain
    assert B.dion_cholesky_grid(256, 1, 768) == 64
    assert B.dion_cholesky_grid(256, 112, 768) == 2
    assert B.dion_cholesky_grid(256, 196, 768) == 0
    for bad in [(0, 1, 64), (256, 0, 64), (256, 1, 0), (256, 1, 40000)]:
        with pytest.raises(B.DionError):
            B.dion_cholesky_grid(*bad)
    assert lib.dion_cholesky_grid(256, 1, 64, None) == B.DION_EINVAL


def test_workspace_bytes_sweep(lib):
    """Planning arithmetic over a grid of shapes and batch sizes, beyond 256 matrices per group (all divisions by
    the batch size are exercised): sizes are 256-byte multiples between what Z, P and R alone take and a generous
    bound.  (The total need not grow with the batch: buffers of split-k partial results shrink as a batch fills the
    GPU without splitting.)"""
    import itertools
    for g_dtype, math in ((B.DION_G_F32, B.DION_MATH_F32), (B.DION_G_BF16, B.DION_MATH_BF16)):
        for (m, n, r) in [(64, 64, 1), (200, 136, 24), (256, 256, 64), (512, 256, 128), (1024, 768, 512), (3072, 8192, 768),
                          (8192, 3072, 768), (8192, 8192, 2048), (16384, 53248, 4096), (70000, 96, 96), (96, 70000, 96)]:
            for count in (1, 2, 3, 7, 112, 196, 255, 256, 257, 300, 1024):
                b = B.dion_workspace_bytes([(m, n, r)] * count, g_dtype, math)
                assert b > 0 and b % 256 == 0
                assert b >= count * 4 * (2 * m * r + n * r)          # at least Z, P and R
                assert b <= 512 + count * (256 * 40 + 4 * (8 * max(m, n) * r + 80 * ((r + 63) // 64 * 64) ** 2 + m * n + 2 * (m + n) * r)) + 8 * 600 * count
    # mixed groups: the total does not depend on the order of the matrices
    shapes = [(256, 256, 64)] * 5 + [(512, 256, 128)] * 3 + [(200, 136, 24)]
    ref = B.dion_workspace_bytes(shapes, B.DION_G_BF16, B.DION_MATH_BF16)
    for perm in itertools.islice(itertools.permutations(range(len(shapes))), 0, 5000, 577):
        assert B.dion_workspace_bytes([shapes[i] for i in perm], B.DION_G_BF16, B.DION_MATH_BF16) == ref


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


def test_host_entry_points_under_the_sanitizers(lib):
    """tests/native/host_san: the host-only entry points (workspace planning over a grid of shapes and batch sizes up to
    the documented limits, the factorisation's grid planner, the argument checks in front of every other call) in a
    build whose host code runs under AddressSanitizer and UndefinedBehaviorSanitizer."""
    exe = os.path.join(ROOT, "tests", "native", "host_san")
    if not os.path.exists(exe):
        from paper_2504_05295_amd import build
        build.build(verbose=False)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, env=env)
    print(p.stdout)
    assert p.returncode == 0, p.stdout[-2000:]
    assert "0 failed expectations" in p.stdout
    assert "runtime error" not in p.stdout and "AddressSanitizer" not in p.stdout
