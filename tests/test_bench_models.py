"""The work models bench.py divides by (algorithmic FLOPs and bytes per stage) against figures worked out by hand
from the step's definition: four products of 2 m n r FLOPs each, CholeskyQR2 at 6 m r^2 + 2/3 r^3, and 30 m n bytes
of matrix traffic per step with a bf16 gradient (M and G read three times, X once; M and X written once)."""
import importlib.util
import os

import pytest

from paper_2504_05295_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


# workload, 8 m n r, orth FLOPs, 30 m n bytes (hand-computed from the shapes)
CASES = [("C3a", 8 * 8192 * 8192 * 2048, 6 * 8192 * 2048 ** 2 + 2 / 3 * 2048 ** 3, 30 * 8192 * 8192),
         ("C4a", 8 * 16384 * 53248 * 1024, 6 * 16384 * 1024 ** 2 + 2 / 3 * 1024 ** 3, 30 * 16384 * 53248),
         ("C4b", 8 * 16384 * 53248 * 4096, 6 * 16384 * 4096 ** 2 + 2 / 3 * 4096 ** 3, 30 * 16384 * 53248)]


@pytest.mark.parametrize("tag,gemm_flops,orth_flops,mn_bytes", CASES)
def test_single_matrix_models(bench, tag, gemm_flops, orth_flops, mn_bytes):
    (m, n, r), = inputs.CONFIGS[tag]["shapes"]
    mdl = bench.kernel_models([(m, n, r)], 2, "bf16")
    assert mdl["k1_BQ"]["flops"] + mdl["k2_BtP"]["flops"] + mdl["k5_update"]["flops"] == pytest.approx(gemm_flops, rel=1e-12)
    assert mdl["orth"]["flops"] == pytest.approx(orth_flops, rel=1e-12)
    small = 4 * m * r + 4 * n * r
    assert mdl["k1_BQ"]["bytes"] == pytest.approx(6 * m * n + small, rel=1e-12)
    assert mdl["k2_BtP"]["bytes"] == pytest.approx(6 * m * n + small, rel=1e-12)
    assert mdl["k5_update"]["bytes"] == pytest.approx(18 * m * n + 4 * m * r + 8 * n * r, rel=1e-12)
    big = sum(mdl[k]["bytes"] for k in ("k1_BQ", "k2_BtP", "k5_update")) - 2 * small - (4 * m * r + 8 * n * r)
    assert big == pytest.approx(mn_bytes, rel=1e-12)
    # which roofline bounds which kernel: the products cross from HBM to MFMA near r = 940, the fused update near 1400
    assert mdl["k1_BQ"]["bound"] == ("mfma" if r >= 1024 else "hbm")
    assert mdl["k5_update"]["bound"] == ("mfma" if r >= 2048 else "hbm")
    assert mdl["k5_update"]["peak"] == (2.5e15 if r >= 2048 else 8.0e12)
    assert mdl["orth"]["peak"] == pytest.approx(2.5e15 / 3)


def test_batched_model_sums_over_the_matrices(bench):
    shapes = inputs.CONFIGS["C5"]["shapes"]
    assert len(shapes) == 196
    mdl = bench.kernel_models(shapes, 2, "bf16")
    total = sum(8.0 * m * n * r for (m, n, r) in shapes)
    assert mdl["k1_BQ"]["flops"] + mdl["k2_BtP"]["flops"] + mdl["k5_update"]["flops"] == pytest.approx(total, rel=1e-12)
    assert total == pytest.approx(1.95e13, rel=5e-3)                 # 3.17e9 parameters x 8 x 768
    assert mdl["k5_update"]["bound"] == "hbm"


def test_fp32_gradient_and_fp32_math(bench):
    mdl = bench.kernel_models([(256, 256, 64)], 4, "f32")
    assert mdl["k5_update"]["bytes"] == 20 * 256 * 256 + 4 * 256 * 64 + 8 * 256 * 64
    assert mdl["k1_BQ"]["peak"] in (157.3e12, 8.0e12) and mdl["orth"]["peak"] == 157.3e12
