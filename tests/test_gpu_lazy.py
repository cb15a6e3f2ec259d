"""GPU parity of the Lazy-Dion step (Section 5.1) through the C-ABI against the CPU oracle: every step is
checked from the very state the GPU step started from, with and without a refresh, in fp32 and bf16 operand
modes, on shapes that take the large-tile kernels and shapes that do not, tall and wide, single and batched."""
import numpy as np
import pytest

from oracle import dion_oracle as orc
from paper_2504_05295_amd import inputs
from gpu_harness import GpuProblem, relf

pytestmark = pytest.mark.gpu
MU, ETA = inputs.MU, inputs.ETA


def lazy_report(gp, i, x_in, m_in, v_in, g32, refresh, method="householder"):
    ref = orc.lazy_dion_step(x_in, g32, m_in, v_in, MU, ETA, refresh, method)
    X, M, V = gp.host(i)
    V64 = V.astype(np.float64)
    r = V.shape[1]
    return dict(status=ref["status"],
                X=relf(X, ref["X"]), M=relf(M, ref["M"]),
                dX=relf(X.astype(np.float64) - x_in, ref["X"] - x_in),
                dM=relf(M.astype(np.float64) - (m_in.astype(np.float64) + g32), ref["M"] - ref["B"]),
                V=relf(V, ref["V"]),
                orth=float(np.abs(V64.T @ V64 - np.eye(r)).max())), ref


def run_lazy(shapes, g_bf16, math, steps, k, tol, otol, method="householder"):
    # tol: state and the refreshed V (both products of a refresh round their operands to bf16 in bf16 mode);
    # otol: orthonormality of V, which comes from the fp32 / split-bf16 orthonormalisation in either mode
    gp = GpuProblem(shapes, g_bf16, math)
    for t in range(steps):
        grads = gp.grads_np(t)
        before = [gp.host(i) for i in range(len(shapes))]
        gp.upload_grads(grads)
        refresh = t % k == 0
        assert gp.lazy_step(MU, ETA, refresh) == (0, -1)
        for i in range(len(shapes)):
            g32 = gp.grad_as_f32(grads[i], g_bf16)
            rep, _ = lazy_report(gp, i, *before[i], g32, refresh, method)
            print("lazy step", t, shapes[i], "refresh" if refresh else "no refresh", {k_: "%.2e" % v for k_, v in rep.items()}, flush=True)
            assert rep["X"] <= tol and rep["M"] <= tol, (t, i, shapes[i], rep)
            assert rep["dX"] <= 3 * tol and rep["dM"] <= 3 * tol, (t, i, shapes[i], rep)
            assert rep["V"] <= tol and rep["orth"] <= otol, (t, i, shapes[i], rep)
            if not refresh:
                assert np.array_equal(gp.host(i)[2], before[i][2])          # V untouched between refreshes
    return gp


def test_lazy_fp32_single_and_ragged():
    run_lazy([(256, 256, 64)], False, "f32", 7, 3, 1e-4, 1e-5)
    run_lazy([(200, 136, 24)], False, "f32", 4, 2, 1e-4, 1e-5)
    run_lazy([(136, 200, 24)], False, "f32", 4, 2, 1e-4, 1e-5)


def test_lazy_fp32_batched_mixed_shapes():
    run_lazy([(256, 192, 32)] * 3 + [(128, 384, 32)] * 2 + [(64, 96, 48)], False, "f32", 5, 2, 1e-4, 1e-5)


def test_lazy_bf16_large_tile_path_tall_wide_and_batched():
    run_lazy([(512, 256, 128)], True, "bf16", 5, 2, 2e-2, 2e-4)
    run_lazy([(256, 768, 128)] * 2 + [(768, 256, 128)], True, "bf16", 4, 3, 2e-2, 2e-4)
    run_lazy([(1024, 1024, 512)], True, "bf16", 3, 2, 2e-2, 2e-4)                # single-launch Cholesky on n x r


def test_lazy_bf16_full_size_direct_load_path():
    # 8192 x 8192, r = 1024: the shape class whose K1 / K2 read the stored bf16 copies of M + G (the refresh writes
    # both orientations, a step without refresh only the plain one); one step of each kind against the full oracle step
    run_lazy([(8192, 8192, 1024)], True, "bf16", 2, 2, 2e-2, 2e-4, method="lapack")


def test_lazy_step_without_refresh_is_defined_for_any_v():
    # the column-normalised Gaussian V of dion_init_state is not orthonormal; the formulas still hold
    gp = GpuProblem([(256, 192, 32)], False, "f32")
    grads = gp.grads_np(0)
    before = gp.host(0)
    gp.upload_grads(grads)
    assert gp.lazy_step(MU, ETA, False) == (0, -1)
    ref = orc.lazy_dion_step(*before[:1], grads[0], before[1], before[2], MU, ETA, False)
    X, M, V = gp.host(0)
    assert relf(X, ref["X"]) < 1e-5 and relf(M, ref["M"]) < 1e-5 and np.array_equal(V, before[2])
    W = gp.debug(0, gp.B.DEBUG_Z)[:, :32]
    assert relf(W, ref["W"]) < 1e-5


def test_lazy_refresh_breakdown_is_reported_and_state_untouched():
    m, n, r = 256, 192, 32
    v_raw = inputs.right_factor_raw(n, r)
    v_raw[:, 7] = v_raw[:, 3]                       # two identical columns: B^T B V is rank deficient
    gp = GpuProblem([(m, n, r)], False, "f32", q_raw=[v_raw])
    gp.upload_grads(gp.grads_np(0))
    before = gp.host(0)
    status, bad = gp.lazy_step(MU, ETA, True)
    assert (status, bad) == (gp.B.DION_NUM_BREAKDOWN, 0)
    for u, v in zip(before, gp.host(0)):
        assert np.array_equal(u, v)
    g = gp.grads_np(0)[0]
    assert orc.lazy_dion_step(before[0], g, before[1], before[2], MU, ETA, True)["status"] == orc.STATUS_BREAKDOWN


def test_lazy_and_plain_steps_share_a_state():
    # a Dion step after Lazy-Dion steps on the same state object: the workspace is shared, nothing is left behind
    from gpu_harness import one_step_report
    gp = GpuProblem([(512, 256, 128)], True, "bf16")
    for t in range(2):
        gp.upload_grads(gp.grads_np(t))
        assert gp.lazy_step(MU, ETA, t == 0) == (0, -1)
    grads = gp.grads_np(2)
    before = gp.host(0)
    gp.upload_grads(grads)
    assert gp.step(MU, ETA) == (0, -1)
    rep, _ = one_step_report(gp, 0, *before, gp.grad_as_f32(grads[0], True), MU, ETA)
    assert rep["X"] < 2e-2 and rep["M"] < 2e-2 and rep["orth"] < 1e-3, rep
