"""GPU parity of the transposed form of the Dion step (Section 4.3, other variants) through the C-ABI against
the CPU oracle, step by step from the GPU's own state: fp32 and bf16 operand modes, tall and wide shapes,
shapes on and off the large-tile path, standard and transposed matrices mixed in one batch."""
import numpy as np
import pytest

from oracle import dion_oracle as orc
from paper_2504_05295_amd import inputs, binding as B
from gpu_harness import GpuProblem, one_step_report, relf

pytestmark = pytest.mark.gpu
MU, ETA = inputs.MU, inputs.ETA
T, S = B.DION_FORM_TRANSPOSED, B.DION_FORM_STANDARD


def transposed_report(gp, i, x_in, m_in, v_in, g32, method="householder"):
    ref = orc.dion_step_transposed(x_in, g32, m_in, v_in, MU, ETA, method)
    X, M, V = gp.host(i)
    V64 = V.astype(np.float64)
    return dict(status=ref["status"], X=relf(X, ref["X"]), M=relf(M, ref["M"]),
                dX=relf(X.astype(np.float64) - x_in, ref["X"] - x_in),
                dM=relf(M.astype(np.float64) - (m_in.astype(np.float64) + g32), ref["M"] - ref["B"]),
                vdot=float(np.min(np.abs(np.sum(V64 * ref["Vt"], axis=0)))),
                vnorm=float(np.abs(np.linalg.norm(V64, axis=0) - 1).max()))


def run(shapes, forms, g_bf16, math, steps, tol, method="householder"):
    gp = GpuProblem(shapes, g_bf16, math, forms=forms)
    for t in range(steps):
        grads = gp.grads_np(t)
        before = [gp.host(i) for i in range(len(shapes))]
        gp.upload_grads(grads)
        assert gp.step(MU, ETA) == (0, -1)
        for i in range(len(shapes)):
            g32 = gp.grad_as_f32(grads[i], g_bf16)
            if forms[i] == T:
                rep = transposed_report(gp, i, *before[i], g32, method)
                assert rep["vdot"] > 1 - 10 * tol and rep["vnorm"] < 1e-5, (t, i, shapes[i], rep)
            else:
                rep, _ = one_step_report(gp, i, *before[i], g32, MU, ETA, method)
            print("step", t, shapes[i], "transposed" if forms[i] == T else "standard", {k_: "%.2e" % v for k_, v in rep.items()}, flush=True)
            assert rep["X"] <= tol and rep["M"] <= tol, (t, i, shapes[i], rep)
            assert rep["dX"] <= 3 * tol and rep["dM"] <= 3 * tol, (t, i, shapes[i], rep)
    return gp


def test_transposed_fp32_tall_wide_ragged():
    run([(256, 192, 32)], [T], False, "f32", 4, 1e-4)
    run([(192, 320, 48)], [T], False, "f32", 3, 1e-4)
    run([(200, 136, 24)], [T], False, "f32", 3, 1e-4)


def test_transposed_bf16_large_tile_path():
    run([(768, 256, 128)], [T], True, "bf16", 3, 2e-2)          # tall: the orthonormalisation runs on 256 x 128
    run([(256, 768, 128)], [T], True, "bf16", 3, 2e-2)
    run([(1024, 1024, 512)], [T], True, "bf16", 2, 2e-2)        # single-launch Cholesky


def test_transposed_bf16_full_size_direct_load_path():
    # shapes whose two products read the stored bf16 copies of M + G: square, and tall so that the
    # orthonormalisation runs on the shorter side (8192 x 3072 is the W_down shape of the 3B decoder, batched by four)
    run([(8192, 8192, 1024)], [T], True, "bf16", 2, 2e-2, method="lapack")
    run([(8192, 3072, 768)] * 4, [T, T, T, T], True, "bf16", 1, 2e-2, method="lapack")


def test_mixed_forms_in_one_batch():
    shapes = [(512, 256, 128), (512, 256, 128), (256, 768, 128), (192, 320, 48), (192, 320, 48)]
    run(shapes, [S, T, T, S, T], True, "bf16", 2, 2e-2)
    run([(256, 192, 32), (256, 192, 32), (128, 384, 32)], [T, S, T], False, "f32", 2, 1e-4)


def test_transposed_breakdown_and_retry():
    m, n, r = 256, 192, 32
    v_raw = inputs.right_factor_raw(m, r)
    v_raw[:, 7] = v_raw[:, 3]                       # two identical columns: B^T Vt is rank deficient
    gp = GpuProblem([(m, n, r)], False, "f32", q_raw=[v_raw], forms=[T])
    gp.upload_grads(gp.grads_np(0))
    before = gp.host(0)
    status, bad = gp.step(MU, ETA)
    assert (status, bad) == (B.DION_NUM_BREAKDOWN, 0)
    for u, v in zip(before, gp.host(0)):
        assert np.array_equal(u, v)
    # exact rank deficiency stays a reported breakdown in the robust mode too, and the state stays untouched
    assert B.dion_retry_breakdowns(gp.state, gp.X, gp.G, gp.M, gp.Q, MU, ETA) == 1
    assert B.dion_last_status(gp.state)[0] == B.DION_NUM_BREAKDOWN
    for u, v in zip(before, gp.host(0)):
        assert np.array_equal(u, v)


def test_lazy_calls_reject_transposed_matrices():
    gp = GpuProblem([(256, 192, 32)], False, "f32", forms=[T])
    gp.upload_grads(gp.grads_np(0))
    L = B.lib()
    import ctypes as C
    rc = L.dion_lazy_step(gp.state.handle, gp.X[0].data_ptr(), gp.G[0].data_ptr(), gp.M[0].data_ptr(), gp.Q[0].data_ptr(),
                          256, 192, 32, C.c_float(MU), C.c_float(ETA), 1, None)
    assert rc == B.DION_EINVAL


def test_library_draws_the_m_by_r_factor():
    m, n, r = 320, 128, 16
    gp = GpuProblem([(m, n, r)], False, "f32", q_is_filled=False, init_seed=9, forms=[T])
    V = gp.host(0)[2]
    assert V.shape == (m, r)
    ref, _ = orc.col_norm(orc.gaussian_fill(m * r, 9, 0).reshape(m, r))
    assert relf(V, ref) < 1e-5
