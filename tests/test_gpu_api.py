"""GPU tests of the C-ABI's behaviour beyond plain parity: batched steps over mixed shapes, breakdown
reporting with untouched state, the library's own Gaussian initialisation, argument validation,
determinism and the stage timers."""
import ctypes as C

import numpy as np
import pytest

from oracle import dion_oracle as orc
from paper_2504_05295_amd import inputs
from gpu_harness import GpuProblem, one_step_report, relf

pytestmark = pytest.mark.gpu
MU, ETA = inputs.MU, inputs.ETA


def check_batch(shapes, g_bf16, math, steps=2, orth_mode=None):
    tol = 1e-4 if math == "f32" else 2e-2
    gp = GpuProblem(shapes, g_bf16, math)
    if orth_mode is not None:
        gp.B.dion_set_orth_mode(gp.state, orth_mode)
    for t in range(steps):
        grads = gp.grads_np(t)
        before = [gp.host(i) for i in range(len(shapes))]
        gp.upload_grads(grads)
        status, bad = gp.step(MU, ETA, batched=True)
        assert (status, bad) == (0, -1)
        for i in range(len(shapes)):
            g32 = gp.grad_as_f32(grads[i], g_bf16)
            rep, _ = one_step_report(gp, i, before[i][0], before[i][1], before[i][2], g32, MU, ETA)
            assert rep["X"] <= tol and rep["M"] <= tol, (i, shapes[i], rep)
            assert rep["dX"] <= 2 * tol and rep["dM"] <= 2 * tol, (i, shapes[i], rep)
            assert rep["orth"] <= (1e-5 if math == "f32" else 1e-3)
    return gp


def test_batched_mixed_shapes_fp32():
    check_batch([(256, 256, 64)] * 3 + [(128, 384, 32)] * 2 + [(200, 136, 24), (64, 96, 48)], False, "f32")


def test_batched_mixed_shapes_bf16():
    # includes shapes that take the large-tile kernels (multiples of 256 / 128) and shapes that do not
    check_batch([(512, 256, 128)] * 3 + [(256, 768, 128)] * 2 + [(192, 320, 48)], True, "bf16")


def test_batched_equals_single_and_is_deterministic():
    shapes = [(256, 128, 32)] * 4
    a = GpuProblem(shapes, True, "bf16")
    b = GpuProblem(shapes, True, "bf16")
    singles = [GpuProblem([shapes[i]], True, "bf16", x0=[a.x0[i]], q_raw=[a.q_raw[i]]) for i in range(4)]
    for t in range(2):
        grads = a.grads_np(t)
        a.upload_grads(grads)
        b.upload_grads(grads)
        assert a.step(MU, ETA, batched=True) == (0, -1)
        assert b.step(MU, ETA, batched=True) == (0, -1)
        for i, sp in enumerate(singles):
            sp.upload_grads([grads[i]])
            assert sp.step(MU, ETA, batched=False) == (0, -1)
    for i in range(4):
        for u, v, w in zip(a.host(i), b.host(i), singles[i].host(0)):
            assert np.array_equal(u, v)            # same call twice: bit-identical (no atomics on results)
            assert np.array_equal(u, w)            # same tile configuration => batched == single, bit for bit


def test_breakdown_is_reported_and_state_untouched():
    m, n, r = 256, 192, 32
    q_raw = inputs.right_factor_raw(n, r)
    q_raw[:, 7] = q_raw[:, 3]                       # two identical columns: Z = B Q is rank deficient
    good = inputs.right_factor_raw(n, r, seed=5)
    gp = GpuProblem([(m, n, r), (m, n, r)], False, "f32", q_raw=[good, q_raw])
    grads = gp.grads_np(0)
    gp.upload_grads(grads)
    before = [gp.host(i) for i in range(2)]
    status, bad = gp.step(MU, ETA, batched=True)
    assert status == gp.B.DION_NUM_BREAKDOWN and bad == 1
    for u, v in zip(before[1], gp.host(1)):
        assert np.array_equal(u, v)                 # X, M, Q of the failing matrix untouched
    rep, ref = one_step_report(gp, 0, before[0][0], before[0][1], before[0][2], grads[0], MU, ETA)
    assert rep["X"] < 1e-4 and rep["M"] < 1e-4      # its neighbour in the batch was stepped normally
    assert orc.dion_step(before[1][0], grads[1], before[1][1], before[1][2], MU, ETA)["status"] == orc.STATUS_BREAKDOWN
    # zero buffer (M = 0 and G = 0) is the other degenerate case
    gp2 = GpuProblem([(128, 128, 16)], False, "f32")
    gp2.upload_grads([np.zeros((128, 128), dtype=np.float32)])
    x0 = gp2.host()
    assert gp2.step(MU, ETA)[0] == gp2.B.DION_NUM_BREAKDOWN
    for u, v in zip(x0, gp2.host()):
        assert np.array_equal(u, v)
    # and the state object keeps working afterwards
    gp2.upload_grads(gp2.grads_np(0))
    assert gp2.step(MU, ETA) == (0, -1)


def test_ill_conditioned_input_is_right_or_reported():
    # cond(B Q) about 1e4: beyond what Cholesky-QR in fp32 can promise.  Either the step is accurate or the
    # library says so and leaves the state alone; silent garbage is the one thing not allowed.
    m, n, r = 512, 384, 64
    gp = GpuProblem([(m, n, r)], False, "f32")
    g = inputs.structured_gradient(m, n, 0, k=r // 2, noise=1e-3)
    gp.upload_grads([g])
    x_in, m_in, q_in = gp.host()
    status, _ = gp.step(MU, ETA)
    if status == 0:
        rep, _ = one_step_report(gp, 0, x_in, m_in, q_in, g, MU, ETA)
        assert rep["X"] < 1e-4 and rep["M"] < 1e-4 and rep["orth"] < 1e-4, rep
    else:
        for u, v in zip((x_in, m_in, q_in), gp.host()):
            assert np.array_equal(u, v)


def test_mu_one_eta_zero_is_plain_accumulation():
    gp = GpuProblem([(256, 256, 64)], True, "bf16")
    g = gp.grads_np(0)
    gp.upload_grads(g)
    assert gp.step(MU, ETA) == (0, -1)
    x1, m1, _ = gp.host()
    g2 = gp.grads_np(1)
    gp.upload_grads(g2)
    assert gp.step(1.0, 0.0) == (0, -1)
    x2, m2, _ = gp.host()
    assert np.array_equal(x2, x1)
    assert np.array_equal(m2, m1 + inputs.bf16_bits_to_f32(g2[0]))      # fp32 add of the stored values, no error feedback


def test_library_draws_and_normalises_q():
    shapes = [(128, 96, 16), (64, 200, 8)]
    gp = GpuProblem(shapes, False, "f32", q_is_filled=False, init_seed=1234)
    for i, (m, n, r) in enumerate(shapes):
        _, M, Q = gp.host(i)
        assert np.all(M == 0)
        raw = orc.gaussian_fill(n * r, seed=1234, stream=i).reshape(n, r)
        ref, _ = orc.col_norm(raw)
        assert np.abs(Q - ref).max() < 2e-6
        assert np.abs(np.linalg.norm(Q.astype(np.float64), axis=0) - 1).max() < 1e-6


def test_argument_validation_on_device():
    import torch
    from paper_2504_05295_amd import binding as B
    m, n, r = 128, 128, 16
    gp = GpuProblem([(m, n, r)], False, "f32")
    gp.upload_grads(gp.grads_np(0))
    lib = B.lib()
    st = gp.state.handle
    X, G, M, Q = gp.X[0], gp.G[0], gp.M[0], gp.Q[0]
    before = gp.host()

    def call(x=X.data_ptr(), g=G.data_ptr(), mm=m, nn=n, rr=r, mu=0.9, eta=0.1):
        return lib.dion_step(st, C.c_void_p(x), C.c_void_p(g), C.c_void_p(M.data_ptr()), C.c_void_p(Q.data_ptr()), mm, nn, rr,
                             C.c_float(mu), C.c_float(eta), None)
    assert call(x=X.data_ptr() + 4) == B.DION_EINVAL          # misaligned
    assert call(g=0) == B.DION_EINVAL                         # null
    assert call(mm=64) == B.DION_EINVAL                       # undeclared shape
    assert call(mu=1.5) == B.DION_EINVAL and call(mu=-0.1) == B.DION_EINVAL
    assert call(mu=float("nan")) == B.DION_EINVAL and call(eta=float("inf")) == B.DION_EINVAL
    torch.cuda.synchronize()
    for u, v in zip(before, gp.host()):
        assert np.array_equal(u, v)                           # rejected calls launch nothing
    # workspace too small / misaligned
    need = B.dion_workspace_bytes([(m, n, r)], B.DION_G_F32, B.DION_MATH_F32)
    ws = torch.empty(need + 512, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) // 256 * 256
    h = C.c_void_p(None)
    args = ((C.c_int64 * 1)(m), (C.c_int64 * 1)(n), (C.c_int64 * 1)(r))
    Mp, Qp = (C.c_void_p * 1)(M.data_ptr()), (C.c_void_p * 1)(Q.data_ptr())
    assert lib.dion_init_state(C.byref(h), 1, *args, 0, 0, C.c_void_p(base), need - 1, Mp, Qp, 1, 0, None) == B.DION_EWORKSPACE
    assert lib.dion_init_state(C.byref(h), 1, *args, 0, 0, C.c_void_p(base + 8), need, Mp, Qp, 1, 0, None) == B.DION_EINVAL
    assert h.value is None
    assert call() == B.DION_OK


def test_stage_timers():
    gp = GpuProblem([(512, 512, 128)], True, "bf16")
    gp.B.dion_set_stage_timing(gp.state, True)
    gp.upload_grads(gp.grads_np(0))
    assert gp.step(MU, ETA) == (0, -1)
    times = gp.B.dion_stage_times(gp.state)
    assert set(times) == set(gp.B.STAGES) and all(v > 0 for v in times.values())
    gp.B.dion_set_stage_timing(gp.state, False)
    assert gp.step(MU, ETA) == (0, -1)


def test_ten_steps_equal_five_plus_resume():
    # the whole optimizer state is (X, M, Q) in caller memory: a fresh state object continues bit-identically
    shape = (256, 192, 48)
    a = GpuProblem([shape], True, "bf16")
    for t in range(6):
        a.upload_grads(a.grads_np(t))
        assert a.step(MU, ETA) == (0, -1)
    b = GpuProblem([shape], True, "bf16")
    for t in range(3):
        b.upload_grads(b.grads_np(t))
        assert b.step(MU, ETA) == (0, -1)
    xs, ms, qs = b.host()
    c = GpuProblem([shape], True, "bf16")
    import torch
    c.X[0].copy_(torch.from_numpy(xs)); c.M[0].copy_(torch.from_numpy(ms)); c.Q[0].copy_(torch.from_numpy(qs))
    for t in range(3, 6):
        c.upload_grads(c.grads_np(t))
        assert c.step(MU, ETA) == (0, -1)
    for u, v in zip(a.host(), c.host()):
        assert np.array_equal(u, v)


def test_large_batch_uses_split_cholesky_launches():
    # 40 x 29 Cholesky tiles per panel: the library switches to separate diagonal / tile launches here
    shape = (768, 512, 384)
    x0 = inputs.weight(*shape[:2])
    q0 = inputs.right_factor_raw(shape[1], shape[2])
    n_mat = 40
    for g_bf16, math, tol in [(False, "f32", 1e-4), (True, "bf16", 2e-2)]:
        gp = GpuProblem([shape] * n_mat, g_bf16, math, x0=[x0] * n_mat, q_raw=[q0] * n_mat)
        g = inputs.gradient(shape[0], shape[1], 0, bf16=g_bf16)
        before = gp.host(0)
        gp.upload_grads([g] * n_mat)
        assert gp.step(MU, ETA, batched=True) == (0, -1)
        rep, _ = one_step_report(gp, 0, before[0], before[1], before[2], gp.grad_as_f32(g, g_bf16), MU, ETA, "lapack")
        assert rep["X"] <= tol and rep["M"] <= tol and rep["dX"] <= 2 * tol and rep["dM"] <= 2 * tol, rep
        ref = gp.host(0)
        for i in (1, 17, 39):
            for u, v in zip(ref, gp.host(i)):
                assert np.array_equal(u, v)


def test_second_pass_takes_full_factorisation_when_needed():
    # cond(B Q) about 1100: after the first Cholesky-QR pass P1^T P1 is far from the identity, so the second pass
    # cannot use its first-order shortcut and must run the full factorisation; the result must still be right.
    m, n, r = 512, 384, 64
    gp = GpuProblem([(m, n, r)], False, "f32")
    g = inputs.structured_gradient(m, n, 0, k=64, noise=5e-3)
    gp.upload_grads([g])
    x_in, m_in, q_in = gp.host()
    assert gp.step(MU, ETA) == (0, -1)
    P1 = gp.debug(0, gp.B.DEBUG_P1).astype(np.float64)
    assert np.linalg.norm(P1.T @ P1 - np.eye(r)) > 1e-3          # the shortcut's precondition does not hold
    rep, _ = one_step_report(gp, 0, x_in, m_in, q_in, g, MU, ETA)
    assert rep["X"] < 1e-4 and rep["M"] < 1e-4 and rep["orth"] < 1e-5, rep
    assert rep["dX"] < 1e-3 and rep["dM"] < 1e-3, rep


@pytest.mark.parametrize("shape", [(1024, 768, 512), (8192, 2048, 1024)])
def test_bf16_second_pass_takes_full_factorisation_when_needed(shape):
    # The same on the split-bf16 path, where a second pass that finds its input orthonormal enough does nothing at
    # all: a power-law gradient (cond(B Q) about 2000) must send it through the full factorisation, the triangular
    # inverse, the late split of the low parts and the three-term product written in place (on the register-staged
    # kernel for the first shape, on the direct-load kernel for the second).  Which way a step went shows in W, the
    # inverse factor of the last factorisation that ran: that of a nearly orthonormal input is close to the identity.
    m, n, r = shape
    eye = np.eye(r)
    control = GpuProblem([shape], True, "bf16")
    control.upload_grads(control.grads_np(0))
    assert control.step(MU, ETA) == (0, -1)
    assert np.abs(control.debug(0, control.B.DEBUG_W)[:r, :r] - eye).max() > 0.5      # Gaussian input: first-pass factor
    del control
    gp = GpuProblem([shape], True, "bf16")
    g = inputs.structured_gradient(m, n, 0, k=r, noise=1e-2, decay=0.5, bf16=True)
    gp.upload_grads([g])
    x_in, m_in, q_in = gp.host()
    assert gp.step(MU, ETA) == (0, -1)
    assert np.abs(gp.debug(0, gp.B.DEBUG_W)[:r, :r] - eye).max() < 0.2                # second-pass factor
    rep, _ = one_step_report(gp, 0, x_in, m_in, q_in, inputs.bf16_bits_to_f32(g), MU, ETA, "lapack")
    assert rep["X"] < 2e-2 and rep["M"] < 2e-2 and rep["orth"] < 1e-4, rep


def qr_properties(gp, i, m_in, q_in, g32):
    """What defines P = thin-QR factor of Z = (M+G) Q with positive diagonal, measured without a reference P."""
    B = gp.B
    m, n, r = gp.shapes[i]
    Z = orc.accumulate(m_in, g32) @ q_in.astype(np.float64)
    P = gp.debug(i, B.DEBUG_P)[:, :r].astype(np.float64)
    T = P.T @ Z
    return dict(cond=float(np.linalg.cond(Z)),
                orth=float(np.abs(P.T @ P - np.eye(r)).max()),
                resid=relf(P @ np.triu(T), Z),                      # Z = P T with T upper triangular
                diag_min=float(np.min(np.diag(T)) / np.linalg.norm(Z, 2)))


def rest_of_step_from_P(gp, i, x_in, m_in, q_in, g32, mu, eta):
    """Errors of R, M, Q, X against the paper's formulas evaluated in fp64, each from the library's own
    inputs to that stage (the weak columns of R are tiny next to the strong ones when B Q is ill conditioned,
    so their fp32 rounding, harmless in R, would dominate a comparison of the column-normalised Q)."""
    B = gp.B
    m, n, r = gp.shapes[i]
    P = gp.debug(i, B.DEBUG_P)[:, :r].astype(np.float64)
    Bm = orc.accumulate(m_in, g32)
    R = Bm.T @ P
    R_lib = gp.debug(i, B.DEBUG_R)[:, :r].astype(np.float64)
    Qn, _ = orc.col_norm(R_lib)
    X, M, Q = gp.host(i)
    return dict(R=relf(R_lib, R), M=relf(M, Bm - (1 - mu) * P @ R.T), Q=relf(Q, Qn),
                dX=relf(X.astype(np.float64) - x_in, -eta * np.sqrt(m / n) * P @ Q.astype(np.float64).T))


def test_shifted_cholqr3_handles_what_cholqr2_reports():
    # cond(B Q) of 1e4 and more: the default mode may report a breakdown (and then leaves the state alone);
    # the shifted three-pass mode must produce the thin-QR factor, and the caller may simply repeat the step.
    cases = [((512, 384, 64), inputs.structured_gradient(512, 384, 0, k=32, noise=1e-3)),
             ((512, 384, 64), inputs.structured_gradient(512, 384, 0, k=32, noise=2e-4)),
             ((64, 64, 64), inputs.gradient(64, 64, 0, 0, 0, bf16=False))]
    for shape, g in cases:
        gp = GpuProblem([shape], False, "f32")
        gp.upload_grads([g])
        x_in, m_in, q_in = gp.host()
        status, _ = gp.step(MU, ETA)
        if status != 0:
            for u, v in zip((x_in, m_in, q_in), gp.host()):
                assert np.array_equal(u, v)
            gp.B.dion_set_orth_mode(gp.state, gp.B.DION_ORTH_SHIFTED_CHOLQR3)
            assert gp.step(MU, ETA) == (0, -1), shape
        else:
            # default mode coped: the robust mode must agree with it
            gp = GpuProblem([shape], False, "f32")
            gp.B.dion_set_orth_mode(gp.state, gp.B.DION_ORTH_SHIFTED_CHOLQR3)
            gp.upload_grads([g])
            assert gp.step(MU, ETA) == (0, -1), shape
        pr = qr_properties(gp, 0, m_in, q_in, g)
        assert pr["cond"] < 3e5, pr                     # the range the mode is documented for
        assert pr["orth"] < 1e-5 and pr["resid"] < 1e-5 and pr["diag_min"] > 0, (shape, pr)
        rest = rest_of_step_from_P(gp, 0, x_in, m_in, q_in, g, MU, ETA)
        assert max(rest.values()) < 1e-5, (shape, rest)
        # the thin-QR factor is unique, so the oracle's is still the target; its forward error grows with cond(Z)
        rep, _ = one_step_report(gp, 0, x_in, m_in, q_in, g, MU, ETA)
        assert rep["PQt"] < 1e-6 * pr["cond"] and rep["PRt"] < 1e-6 * pr["cond"], (shape, pr, rep)
        print("shifted-cholqr3", shape, pr, rest, rep)


def test_shifted_cholqr3_matches_oracle_on_regular_inputs():
    check_batch([(256, 256, 64), (200, 136, 24)], False, "f32", orth_mode=1)
    check_batch([(512, 256, 128)] * 2 + [(192, 320, 48)], True, "bf16", orth_mode=1)
    # ranks of four and six panels: the three passes run on the single-launch factorisation and inverse, the split-bf16
    # ones in place
    check_batch([(1024, 768, 256)] * 2 + [(768, 512, 384)], True, "bf16", orth_mode=1)
    check_batch([(512, 512, 256)], False, "f32", orth_mode=1)


def test_fallback_mode_equals_default_on_regular_inputs():
    # nothing breaks down: the fallback passes return at once and the step is the default step, bit for bit
    for shapes, g_bf16, math in [([(256, 256, 64), (200, 136, 24)], False, "f32"), ([(1024, 768, 256)] * 2, True, "bf16"),
                                 ([(512, 512, 256)], False, "f32")]:
        a = check_batch(shapes, g_bf16, math)
        b = check_batch(shapes, g_bf16, math, orth_mode=2)
        for i in range(len(shapes)):
            for u, v in zip(a.host(i), b.host(i)):
                assert np.array_equal(u, v), (shapes[i], math)


def test_fallback_mode_completes_the_step_on_the_device():
    # a batch of three whose middle matrix is too ill conditioned for CholeskyQR2: with the fallback mode the one call
    # completes all three, no host round trip, and the other two come out exactly as without it
    shape = (512, 384, 64)
    results = {}
    for mode in (0, 2):
        gp = GpuProblem([shape] * 3, False, "f32")
        gp.B.dion_set_orth_mode(gp.state, mode)
        grads = gp.grads_np(0)
        grads[1] = inputs.structured_gradient(512, 384, 0, k=32, noise=2e-4)
        gp.upload_grads(grads)
        before = [gp.host(i) for i in range(3)]
        results[mode] = (gp, gp.step(MU, ETA, batched=True), before, grads)
    assert results[0][1] == (results[0][0].B.DION_NUM_BREAKDOWN, 1)
    gp, outcome, before, grads = results[2]
    assert outcome == (0, -1)
    for i in (0, 2):
        for u, v in zip(results[0][0].host(i), gp.host(i)):
            assert np.array_equal(u, v)
    pr = qr_properties(gp, 1, before[1][1], before[1][2], grads[1])
    assert 1e4 < pr["cond"] < 3e5, pr
    assert pr["orth"] < 1e-5 and pr["resid"] < 1e-5 and pr["diag_min"] > 0, pr
    rest = rest_of_step_from_P(gp, 1, *before[1], grads[1], MU, ETA)
    assert max(rest.values()) < 1e-5, rest
    rep, _ = one_step_report(gp, 1, *before[1], grads[1], MU, ETA)
    assert rep["PQt"] < 1e-6 * pr["cond"] and rep["PRt"] < 1e-6 * pr["cond"], (pr, rep)
    # an exactly rank-deficient product is still reported, and the state left alone
    q_raw = inputs.right_factor_raw(192, 32)
    q_raw[:, 7] = q_raw[:, 3]                       # two identical columns
    for kind in ("duplicate column", "zero buffer"):
        gp = GpuProblem([(256, 192, 32)], False, "f32", q_raw=[q_raw] if kind == "duplicate column" else None)
        gp.B.dion_set_orth_mode(gp.state, 2)
        gp.upload_grads(gp.grads_np(0) if kind == "duplicate column" else [np.zeros((256, 192), dtype=np.float32)])
        x_in, m_in, q_in = gp.host()
        assert gp.step(MU, ETA) == (gp.B.DION_NUM_BREAKDOWN, 0), kind
        for u, v in zip((x_in, m_in, q_in), gp.host()):
            assert np.array_equal(u, v)


def test_orth_mode_validation():
    gp = GpuProblem([(128, 128, 16)], False, "f32")
    L = gp.B.lib()
    assert L.dion_set_orth_mode(gp.state.handle, 3) == gp.B.DION_EINVAL
    assert L.dion_set_orth_mode(gp.state.handle, 2) == 0
    assert L.dion_set_orth_mode(None, 0) == gp.B.DION_EINVAL
    assert L.dion_set_orth_mode(gp.state.handle, 1) == 0


def test_retry_completes_only_the_matrices_that_broke_down():
    # a batch of three: the middle one is too ill conditioned for CholeskyQR2 in fp32
    shape = (512, 384, 64)
    gp = GpuProblem([shape] * 3, False, "f32")
    grads = gp.grads_np(0)
    grads[1] = inputs.structured_gradient(512, 384, 0, k=32, noise=2e-4)
    gp.upload_grads(grads)
    before = [gp.host(i) for i in range(3)]
    status, bad = gp.step(MU, ETA, batched=True)
    assert (status, bad) == (gp.B.DION_NUM_BREAKDOWN, 1)
    after_first = [gp.host(i) for i in range(3)]
    for u, v in zip(before[1], after_first[1]):
        assert np.array_equal(u, v)
    assert gp.B.dion_retry_breakdowns(gp.state, gp.X, gp.G, gp.M, gp.Q, MU, ETA) == 1
    assert gp.B.dion_last_status(gp.state) == (0, -1)
    for i in (0, 2):                                    # stepped once, not twice
        for u, v in zip(after_first[i], gp.host(i)):
            assert np.array_equal(u, v)
    pr = qr_properties(gp, 1, before[1][1], before[1][2], grads[1])
    assert pr["orth"] < 1e-5 and pr["resid"] < 1e-5 and pr["diag_min"] > 0, pr
    rest = rest_of_step_from_P(gp, 1, *before[1], grads[1], MU, ETA)
    assert max(rest.values()) < 1e-5, rest
    rep, _ = one_step_report(gp, 1, *before[1], grads[1], MU, ETA)
    assert rep["X"] < 1e-4 and rep["M"] < 1e-4, rep
    # nothing to do when nothing broke down
    assert gp.B.dion_retry_breakdowns(gp.state, gp.X, gp.G, gp.M, gp.Q, MU, ETA) == 0
    for i in range(3):
        ref = orc.dion_step(before[i][0], grads[i], before[i][1], before[i][2], MU, ETA)
        assert relf(gp.host(i)[0], ref["X"]) < 1e-4 and relf(gp.host(i)[1], ref["M"]) < 1e-4


def test_bounded_waits_of_the_single_launch_cholesky():
    # r = 512 takes the single-launch Cholesky kernel, whose workgroups wait for one another.  With the wait
    # limit at zero every wait that is not satisfied at once gives up: the kernel must still end, the step must
    # be reported as failed with the state untouched, and the next step (normal limit) must be right again.
    shape = (1024, 768, 512)
    gp = GpuProblem([shape], True, "bf16")
    grads = gp.grads_np(0)
    gp.upload_grads(grads)
    before = gp.host(0)
    gp.B.dion_set_wait_limit(gp.state, 0)
    status, bad = gp.step(MU, ETA)
    assert (status, bad) == (gp.B.DION_WAIT_TIMEOUT, 0)      # a scheduling outcome, not a property of the matrix
    for u, v in zip(before, gp.host(0)):
        assert np.array_equal(u, v)
    # the fallback repeats the step without the kernels that wait (the limit is still 0: they would time out again)
    assert gp.B.dion_retry_breakdowns(gp.state, gp.X, gp.G, gp.M, gp.Q, MU, ETA) == 1
    assert gp.B.dion_last_status(gp.state) == (0, -1)
    rep, _ = one_step_report(gp, 0, *before, gp.grad_as_f32(grads[0], True), MU, ETA)
    assert rep["X"] < 2e-2 and rep["M"] < 2e-2 and rep["orth"] < 1e-3, rep
    # a later step with the default limit is not affected
    before = gp.host(0)
    gp.B.dion_set_wait_limit(gp.state, 1 << 20)
    assert gp.step(MU, ETA) == (0, -1)
    rep, _ = one_step_report(gp, 0, *before, gp.grad_as_f32(grads[0], True), MU, ETA)
    assert rep["X"] < 2e-2 and rep["M"] < 2e-2 and rep["orth"] < 1e-3, rep


def test_captured_step_replays_like_eager_steps():
    # A step only launches kernels (no allocation, no host synchronisation, no memset), so a caller may capture
    # it into a HIP graph.  Each replay must give what the eager step gives, bit for bit, also for the
    # single-launch Cholesky kernel whose flags are tagged with a launch counter (kept on the device).
    import torch
    shape = (1024, 768, 512)
    eager = GpuProblem([shape], True, "bf16")
    graphed = GpuProblem([shape], True, "bf16")
    B = graphed.B
    g0 = eager.grads_np(0)
    eager.upload_grads(g0)
    graphed.upload_grads(g0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            B.dion_step(graphed.state, graphed.X[0], graphed.G[0], graphed.M[0], graphed.Q[0], MU, ETA)
    torch.cuda.synchronize()
    for t in range(4):
        eager.upload_grads(eager.grads_np(t))
        graphed.G[0].copy_(eager.G[0])
        assert eager.step(MU, ETA) == (0, -1)
        graph.replay()
        torch.cuda.synchronize()
        assert B.dion_last_status(graphed.state) == (0, -1)
        for u, v in zip(eager.host(0), graphed.host(0)):
            assert np.array_equal(u, v), t


def test_measured_ceilings_are_plausible():
    import torch
    from paper_2504_05295_amd import binding as B
    scratch = torch.empty(1 << 29, dtype=torch.uint8, device="cuda")
    c = B.dion_measure_ceilings(scratch)
    print(c, flush=True)
    # published peaks: 2500 TFLOP/s dense bf16, 8000 GB/s; a working MI355X delivers a good part of both
    assert 500.0 < c["mfma_tflops"] < 2600.0
    assert 1500.0 < c["stream_gbps"] < 8100.0
    with pytest.raises(B.DionError):
        B.dion_measure_ceilings(scratch[: 1 << 20])


def test_empty_batch_is_a_no_op():
    import torch
    from paper_2504_05295_amd import binding as B
    lib = B.lib()
    need = C.c_size_t(0)
    assert lib.dion_workspace_bytes(0, None, None, None, B.DION_G_F32, B.DION_MATH_F32, C.byref(need)) == B.DION_OK
    ws = torch.empty(need.value + 256, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) // 256 * 256
    h = C.c_void_p(None)
    assert lib.dion_init_state(C.byref(h), 0, None, None, None, B.DION_G_F32, B.DION_MATH_F32, C.c_void_p(base), need.value,
                               None, None, 1, 0, None) == B.DION_OK
    assert lib.dion_step_batched(h, 0, None, None, None, None, None, None, None, C.c_float(0.95), C.c_float(0.01), None) == B.DION_OK
    status, bad = C.c_int(7), C.c_int(7)
    assert lib.dion_last_status(h, C.byref(status), C.byref(bad)) == B.DION_OK
    assert (status.value, bad.value) == (0, -1)
    assert lib.dion_destroy_state(h) == B.DION_OK


def test_fallback_mode_in_a_bf16_batch_on_the_large_tile_path():
    # three matrices on the 128-wide-tile bf16 path, the middle one with cond(B Q) of a few 1e4: the fallback passes run
    # in fp32 for that one only, gated per matrix; its neighbours come out exactly as in the default mode
    shape = (1024, 768, 256)
    m, n, r = shape
    out = {}
    for mode in (0, 2):
        gp = GpuProblem([shape] * 3, True, "bf16")
        gp.B.dion_set_orth_mode(gp.state, mode)
        grads = gp.grads_np(0)
        grads[1] = inputs.structured_gradient(m, n, 0, k=r, noise=1e-4, decay=1.0, bf16=True)
        gp.upload_grads(grads)
        before = [gp.host(i) for i in range(3)]
        out[mode] = (gp, gp.step(MU, ETA, batched=True), before, grads)
    assert out[0][1] == (out[0][0].B.DION_NUM_BREAKDOWN, 1)
    gp, outcome, before, grads = out[2]
    assert outcome == (0, -1)
    for i in (0, 2):
        for u, v in zip(out[0][0].host(i), gp.host(i)):
            assert np.array_equal(u, v)
    B = gp.B
    x_in, m_in, q_in = before[1]
    g32 = inputs.bf16_bits_to_f32(grads[1]).astype(np.float64)
    Bm = m_in.astype(np.float64) + g32
    Z = out[0][0].debug(1, B.DEBUG_Z)[:, :r].astype(np.float64)     # the default-mode run formed the same Z and kept it
    P = gp.debug(1, B.DEBUG_P)[:, :r].astype(np.float64)
    R = gp.debug(1, B.DEBUG_R)[:, :r].astype(np.float64)
    X, M, Q = gp.host(1)
    w = np.linalg.eigvalsh(Z.T @ Z)
    assert 3e3 < np.sqrt(w[-1] / w[0]) < 1e5
    T = P.T @ Z
    assert np.abs(P.T @ P - np.eye(r)).max() < 1e-5 and relf(P @ np.triu(T), Z) < 1e-5 and np.min(np.diag(T)) > 0
    assert relf(R, Bm.T @ P) < 2e-2 and relf(M, Bm - (1 - MU) * P @ R.T) < 2e-2
    Qn, _ = orc.col_norm(R)
    assert relf(Q, Qn) < 1e-5
    assert relf(X.astype(np.float64) - x_in, -ETA * np.sqrt(m / n) * P @ Q.astype(np.float64).T) < 2e-2
