"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

A full fp64 oracle step of the Llama-3-405B MLP shape (16384 x 53248, r up to 4096) takes many minutes
on the host, so that configuration is checked stage by stage instead: every stage's output is compared
with the oracle's per-entry definition on sampled entries, evaluated from that stage's actual inputs,
and the orthonormalisation is pinned by the uniqueness of the QR factor (P^T P = I, P^T Z upper
triangular with positive diagonal, P (P^T Z) = Z).  The 3B-decoder shapes are small enough for full
oracle steps, one per shape class, plus a run of the whole 196-matrix batch."""
import numpy as np
import pytest

from oracle import dion_oracle as orc
from paper_2504_05295_amd import inputs
from gpu_harness import GpuProblem, one_step_report, relf

pytestmark = pytest.mark.gpu
MU, ETA = inputs.MU, inputs.ETA


@pytest.mark.parametrize("r", [1024, 4096])
def test_c4_llama_mlp_stagewise(r):
    m, n = 16384, 53248
    gp = GpuProblem([(m, n, r)], True, "bf16")
    B = gp.B
    rng = np.random.default_rng(7)
    for t in range(2):                       # second step starts from a non-zero momentum buffer
        g = gp.grads_np(t)[0]
        gp.upload_grads([g])
        x_in, m_in, q_in = gp.host()
        status, _ = gp.step(MU, ETA)
        assert status == 0
        print("step", t, "done", flush=True)
    g32 = gp.grad_as_f32(g, True)
    X, M, Q = gp.host()
    Z = gp.debug(0, B.DEBUG_Z)
    P = gp.debug(0, B.DEBUG_P)
    R = gp.debug(0, B.DEBUG_R)
    ns = 48
    # stage 1: Z = (M+G) Q on sampled entries (bf16 operands: compare against the scale of Z)
    ri, ci = rng.integers(0, m, ns), rng.integers(0, r, ns)
    zref = orc.entry_Z(m_in, g32, q_in, ri, ci)
    zscale = np.sqrt(np.mean(Z[ri, :].astype(np.float64) ** 2))
    assert np.abs(Z[ri, ci] - zref).max() <= 2e-2 * zscale
    # stage 2: P is THE QR factor of Z (unique): orthonormal, P^T Z upper triangular with positive diagonal, P T = Z
    P64 = P.astype(np.float64)
    gram = P64.T @ P64
    assert np.abs(gram - np.eye(r)).max() <= 1e-4
    T = P64.T @ Z.astype(np.float64)
    tscale = np.abs(np.diag(T)).min()
    assert np.all(np.diag(T) > 0)
    assert np.abs(np.tril(T, -1)).max() <= 1e-3 * np.abs(np.diag(T)).max()
    rows = rng.integers(0, m, 32)
    assert relf(P64[rows, :] @ T, Z[rows, :]) <= 1e-3
    print("orth checked, min/max diag(T) %.3e %.3e" % (tscale, np.abs(np.diag(T)).max()), flush=True)
    # stage 3: R = (M+G)^T P on sampled entries
    rj, ca = rng.integers(0, n, ns), rng.integers(0, r, ns)
    rref = orc.entry_R(m_in, g32, P, rj, ca)
    rscale = np.sqrt(np.mean(R[rj, :].astype(np.float64) ** 2))
    assert np.abs(R[rj, ca] - rref).max() <= 2e-2 * rscale
    # stage 4: column norms and the new Q
    s = gp.debug(0, B.DEBUG_S)[:, 0] if gp.debug(0, B.DEBUG_S).ndim == 2 else gp.debug(0, B.DEBUG_S)
    sref = np.sqrt(np.sum(R.astype(np.float64) ** 2, axis=0))
    assert np.abs(s.reshape(-1)[:r] - sref).max() <= 1e-5 * sref.max()
    assert relf(Q, R / (sref + orc.COLNORM_EPS)) <= 1e-6
    # stage 5: the fused update on sampled entries, from the factors it actually used
    ui, uj = rng.integers(0, m, ns), rng.integers(0, n, ns)
    xs, ms = orc.entry_update(x_in, g32, m_in, P, R, MU, ETA, ui, uj)
    dx_ref = xs - x_in[ui, uj]
    dm_ref = ms - (m_in[ui, uj].astype(np.float64) + g32[ui, uj])
    dx = X[ui, uj].astype(np.float64) - x_in[ui, uj]
    dm = M[ui, uj].astype(np.float64) - (m_in[ui, uj].astype(np.float64) + g32[ui, uj])
    assert np.abs(X[ui, uj] - xs).max() <= 2e-2 * np.abs(xs).max()
    assert np.linalg.norm(dx - dx_ref) <= 2e-2 * np.linalg.norm(dx_ref) + 1e-7 * np.linalg.norm(xs)
    assert np.linalg.norm(dm - dm_ref) <= 2e-2 * np.linalg.norm(dm_ref) + 1e-7 * np.linalg.norm(ms)
    # whole-matrix invariant of the step: ||X_new - X|| = eta sqrt(m/n) sqrt(r)  (P orthonormal, Q unit columns)
    dxn = np.linalg.norm(X.astype(np.float64) - x_in)
    assert abs(dxn / (ETA * np.sqrt(m / n) * np.sqrt(r)) - 1) <= 1e-2


@pytest.mark.parametrize("shape", [(3072, 3072, 768), (3072, 8192, 768), (8192, 3072, 768)])
def test_c5_shape_classes_full_oracle(shape):
    gp = GpuProblem([shape], True, "bf16")
    for t in range(2):
        g = gp.grads_np(t)[0]
        gp.upload_grads([g])
        x_in, m_in, q_in = gp.host()
        assert gp.step(MU, ETA) == (0, -1)
    rep, _ = one_step_report(gp, 0, x_in, m_in, q_in, gp.grad_as_f32(g, True), MU, ETA, "lapack")
    print(shape, {k: "%.2e" % v for k, v in rep.items()}, flush=True)
    assert rep["X"] <= 2e-2 and rep["M"] <= 2e-2 and rep["dX"] <= 2e-2 and rep["dM"] <= 2e-2
    assert rep["orth"] <= 1e-3 and rep["PQt"] <= 2e-2 and rep["PRt"] <= 2e-2


def test_c5_whole_batch_of_196():
    import torch
    cfg = inputs.CONFIGS["C5"]
    shapes = cfg["shapes"]
    classes = sorted(set(shapes))
    host = {c: (inputs.weight(c[0], c[1], 1, 0), inputs.right_factor_raw(c[1], c[2], 2, 0),
                inputs.gradient(c[0], c[1], 0, 0, 0, bf16=True)) for c in classes}
    gp = GpuProblem(shapes, True, "bf16", x0=[host[s][0] for s in shapes], q_raw=[host[s][1] for s in shapes])
    firsts = {c: shapes.index(c) for c in classes}
    before = {c: gp.host(firsts[c]) for c in classes}
    gp.upload_grads([host[s][2] for s in shapes])
    assert gp.step(MU, ETA, batched=True) == (0, -1)
    print("batched step done", flush=True)
    for c in classes:
        i0 = firsts[c]
        rep, _ = one_step_report(gp, i0, before[c][0], before[c][1], before[c][2], inputs.bf16_bits_to_f32(host[c][2]), MU, ETA, "lapack")
        print(c, {k: "%.2e" % v for k, v in rep.items()}, flush=True)
        assert rep["X"] <= 2e-2 and rep["M"] <= 2e-2 and rep["dX"] <= 2e-2 and rep["dM"] <= 2e-2 and rep["orth"] <= 1e-3
        # every matrix of the class got identical inputs, so it must hold identical results
        ref = [t.clone() for t in (gp.X[i0], gp.M[i0], gp.Q[i0])]
        for i, s in enumerate(shapes):
            if s == c and i != i0:
                assert torch.equal(gp.X[i], ref[0]) and torch.equal(gp.M[i], ref[1]) and torch.equal(gp.Q[i], ref[2])
