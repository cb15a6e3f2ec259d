"""Parity on seeded random shapes: m, n, r drawn without regard to any tile size, every combination of gradient storage
and operand type, the plain step and the Lazy-Dion and transposed variants, each against the oracle's step from the same
state.  The fixed-shape tests cover the paths one by one; this one looks for what falls between them."""
import numpy as np
import pytest

from paper_2504_05295_amd import inputs
from gpu_harness import GpuProblem, one_step_report
import test_gpu_lazy as lazy_tests
import test_gpu_transposed as transposed_tests

pytestmark = pytest.mark.gpu
MU, ETA = inputs.MU, inputs.ETA


def random_shapes(seed, count, hi, rmax):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        m, n = int(rng.integers(8, hi)), int(rng.integers(8, hi))
        out.append((m, n, int(rng.integers(1, min(m, n, rmax) + 1))))
    return out


@pytest.mark.parametrize("g_bf16,math", [(False, "f32"), (True, "bf16"), (False, "bf16"), (True, "f32")])
def test_plain_step_on_random_shapes(g_bf16, math):
    tol = 1e-4 if math == "f32" else 2e-2
    for idx, shape in enumerate(random_shapes(2024, 16, 700, 320)):
        gp = GpuProblem([shape], g_bf16, math, seed=idx)
        for t in range(2):
            g = gp.grads_np(t)[0]
            x_in, m_in, q_in = gp.host()
            gp.upload_grads([g])
            assert gp.step(MU, ETA) == (0, -1), (shape, t)
            rep, _ = one_step_report(gp, 0, x_in, m_in, q_in, gp.grad_as_f32(g, g_bf16), MU, ETA,
                                     "lapack" if max(shape) > 400 else "householder")
            assert rep["X"] <= tol and rep["M"] <= tol and rep["dX"] <= 2 * tol and rep["dM"] <= 2 * tol, (shape, t, rep)
            assert rep["orth"] <= (1e-5 if math == "f32" else 1e-3), (shape, t, rep)


def test_variants_on_random_shapes():
    for shape in random_shapes(77, 6, 500, 200):
        lazy_tests.run_lazy([shape], False, "f32", 3, 2, 1e-4, 1e-5)
        lazy_tests.run_lazy([shape], True, "bf16", 3, 2, 2e-2, 2e-4)
        transposed_tests.run([shape], [transposed_tests.T], False, "f32", 2, 1e-4)
        transposed_tests.run([shape], [transposed_tests.T], True, "bf16", 2, 2e-2)


@pytest.mark.parametrize("shape,math", [((1100, 1000, 900), "f32"), ((1500, 1408, 1344), "f32"), ((2500, 2432, 2368), "f32"),
                                        ((2816, 2560, 2368), "bf16"), ((3328, 3072, 3008), "bf16")])
def test_panel_counts_between_the_benchmark_ranks(shape, math):
    # r / 64 rounded up = 15, 21, 37, 37, 47 panels: the single-launch factorisation with every helper grid, with block
    # counts that are neither powers of two nor multiples of the helper grid's sides, the inverse formed along with it
    tol = 1e-4 if math == "f32" else 2e-2
    gp = GpuProblem([shape], math == "bf16", math, seed=5)
    for t in range(2):
        g = gp.grads_np(t)[0]
        x_in, m_in, q_in = gp.host()
        gp.upload_grads([g])
        assert gp.step(MU, ETA) == (0, -1), (shape, t)
        rep, _ = one_step_report(gp, 0, x_in, m_in, q_in, gp.grad_as_f32(g, math == "bf16"), MU, ETA, "lapack")
        assert rep["X"] <= tol and rep["M"] <= tol and rep["dX"] <= 2 * tol and rep["dM"] <= 2 * tol, (shape, t, rep)
        assert rep["orth"] <= (1e-5 if math == "f32" else 1e-3), (shape, t, rep)
