"""Pins of the Lazy-Dion part of the CPU oracle (Section 5.1: Lazy-Dion update rule, SymPowerIter1) against
things other than itself: a hand-worked rank-1 step, closed forms that hold for an orthonormal V, the SVD
fixed point from a brute-force Jacobi SVD, the convergence rate of orthogonal iteration on B^T B, and the
no-refresh step written out with explicit loops.  CPU only."""
import os

import numpy as np

from oracle import dion_oracle as orc
from jacobi_svd import jacobi_svd

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, rows, cols, *v = line.split()
            out[k] = np.array([float(x) for x in v]).reshape(int(rows), int(cols))
    return out


def test_rank1_lazy_step_hand_computed():
    gold = read_golden("lazy_step_rank1.txt")
    B = np.array([[2.0, 0.0], [0.0, 1.0], [0.0, 0.0]])
    M = np.array([[0.5, 0.0], [0.0, 0.25], [0.0, 0.0]])
    res = orc.lazy_dion_step(np.zeros((3, 2)), B - M, M, np.array([[0.6], [0.8]]), 0.9, 0.5, True)
    assert np.abs(res["V"] - gold["V_new"]).max() < 1e-15
    assert np.abs(res["W"] - gold["W"]).max() < 1e-15
    assert np.abs(res["M"] - gold["M_new"]).max() < 1e-15
    assert np.abs(res["X"] - gold["X_new"]).max() < 1e-8          # the 1e-8 ColNorm guard


def test_closed_forms_for_orthonormal_v():
    m, n, r = 40, 28, 6
    rng = np.random.default_rng(3)
    X = rng.standard_normal((m, n))
    M = rng.standard_normal((m, n))
    G = rng.standard_normal((m, n))
    V, _ = np.linalg.qr(rng.standard_normal((n, r)))
    mu, eta = 0.95, 0.01
    for refresh in (False, True):
        res = orc.lazy_dion_step(X, G, M, V, mu, eta, refresh)
        Vn, B = res["V"], M + G
        assert np.abs(Vn.T @ Vn - np.eye(r)).max() < 1e-12
        if not refresh:
            assert np.array_equal(Vn, V)
        # M_new = B (I - beta V V^T): damped by mu on span(V), untouched on its complement
        assert np.abs(res["M"] @ Vn - mu * (B @ Vn)).max() < 1e-12
        comp = np.eye(n) - Vn @ Vn.T
        assert np.abs(res["M"] @ comp - B @ comp).max() < 1e-12
        # U has unit columns and V is orthonormal: ||U V^T||_F^2 = trace(U^T U) = r
        dx = res["X"] - X
        assert abs(np.linalg.norm(dx) - eta * np.sqrt(m / n) * np.sqrt(r)) < 1e-8
        # dX V = -eta sqrt(m/n) U, and U_j is parallel to (B V)_j with the same orientation
        U = -(dx @ Vn) / (eta * np.sqrt(m / n))
        W = B @ Vn
        cos = np.sum(U * W, axis=0) / np.linalg.norm(W, axis=0)
        assert np.abs(cos - 1).max() < 1e-7
        assert np.abs(res["s"] - np.linalg.norm(W, axis=0)).max() < 1e-12


def test_no_refresh_step_with_explicit_loops():
    # V need not be orthonormal for the formulas to be defined: write them out entry by entry
    m, n, r = 5, 4, 2
    rng = np.random.default_rng(11)
    X, G, M = rng.standard_normal((3, m, n))
    V = rng.standard_normal((n, r))
    mu, eta = 0.7, 0.3
    res = orc.lazy_dion_step(X, G, M, V, mu, eta, False)
    W = [[sum((M[i][k] + G[i][k]) * V[k][j] for k in range(n)) for j in range(r)] for i in range(m)]
    s = [np.sqrt(sum(W[i][j] ** 2 for i in range(m))) for j in range(r)]
    for i in range(m):
        for c in range(n):
            mexp = M[i][c] + G[i][c] - (1 - mu) * sum(W[i][j] * V[c][j] for j in range(r))
            xexp = X[i][c] - eta * np.sqrt(m / n) * sum(W[i][j] / (s[j] + 1e-8) * V[c][j] for j in range(r))
            assert abs(res["M"][i][c] - mexp) < 1e-13 and abs(res["X"][i][c] - xexp) < 1e-13


def test_sym_power_iter_is_the_qr_factor_of_btbv():
    m, n, r = 30, 22, 5
    rng = np.random.default_rng(5)
    B = rng.standard_normal((m, n))
    V = rng.standard_normal((n, r))
    Vn, Y, T, status = orc.sym_power_iter1(B, V)
    assert status == orc.STATUS_OK
    Yexp = np.zeros((n, r))
    for i in range(m):                                   # B^T (B V) as a sum of outer products of rows of B
        Yexp += np.outer(B[i], B[i] @ V)
    assert np.abs(Y - Yexp).max() < 1e-11
    Qn, Rn = np.linalg.qr(Yexp)
    sg = np.sign(np.diag(Rn))
    assert np.abs(Vn - Qn * sg).max() < 1e-11             # unique thin-QR factor with positive diagonal
    assert np.all(np.diag(T) > 0) and np.abs(np.tril(T, -1)).max() == 0


def test_svd_fixed_point_of_the_refresh():
    m, n, r = 18, 14, 4
    rng = np.random.default_rng(8)
    B = rng.standard_normal((m, n))
    U, sig, V = jacobi_svd(B)
    Ur, Vr = U[:, :r], V[:, :r]
    X = rng.standard_normal((m, n))
    mu, eta = 0.95, 0.02
    res = orc.lazy_dion_step(X, B, np.zeros((m, n)), Vr, mu, eta, True)
    assert np.abs(res["V"] - Vr).max() < 1e-10            # B^T B V_r = V_r Sigma^2: positive diagonal, no sign flips
    assert np.abs(res["s"] - sig[:r]).max() < 1e-10       # ||W_j|| = sigma_j
    assert np.abs(res["X"] - (X - eta * np.sqrt(m / n) * Ur @ Vr.T)).max() < 1e-8
    assert np.abs(res["M"] - (B - (1 - mu) * (Ur * sig[:r]) @ Vr.T)).max() < 1e-10


def test_refreshes_converge_at_the_squared_rate_of_power_iteration():
    # G = 0, mu = 1 keeps M = A; a refresh every step is orthogonal iteration on A^T A, whose subspace error
    # contracts by (sigma_{r+1} / sigma_r)^2 per step
    m, n, r = 24, 20, 3
    rng = np.random.default_rng(4)
    U0, _ = np.linalg.qr(rng.standard_normal((m, n)))
    V0, _ = np.linalg.qr(rng.standard_normal((n, n)))
    sig = np.concatenate([[10.0, 8.0, 6.0], 3.0 * 0.9 ** np.arange(n - 3)])   # gap 3/6
    A = (U0 * sig) @ V0.T
    _, sj, Vj = jacobi_svd(A)
    assert np.abs(sj - sig).max() < 1e-10
    V, _ = orc.col_norm(rng.standard_normal((n, r)))
    errs = []
    for _ in range(14):
        res = orc.lazy_dion_step(np.zeros((m, n)), np.zeros((m, n)), A, V, 1.0, 0.0, True)
        assert np.array_equal(res["M"], A)
        V = res["V"]
        errs.append(np.linalg.norm(V @ V.T - Vj[:, :r] @ Vj[:, :r].T, 2))
    rho2 = (3.0 / 6.0) ** 2
    for a, b in zip(errs[3:10], errs[4:11]):
        assert b <= 1.3 * rho2 * a + 1e-13
    assert errs[-1] < 1e-6


def test_run_lazy_steps_refresh_schedule_and_breakdown():
    m, n, r = 12, 10, 3
    rng = np.random.default_rng(2)
    X = 0.02 * rng.standard_normal((m, n))
    grads = [1e-2 * rng.standard_normal((m, n)) for _ in range(5)]
    V0, _ = orc.col_norm(rng.standard_normal((n, r)))
    out = orc.run_lazy_steps(X, grads, np.zeros((m, n)), V0, 0.95, 0.01, k=2)
    assert not np.array_equal(out[0]["V"], V0.astype(np.float32))          # t = 0 refreshes
    assert np.array_equal(out[1]["V"], out[0]["V"])                        # t = 1 does not
    assert not np.array_equal(out[2]["V"], out[1]["V"])                    # t = 2 does
    # manual replay of step 1 from the rounded state of step 0
    res = orc.lazy_dion_step(out[0]["X"], grads[1], out[0]["M"], out[0]["V"], 0.95, 0.01, False)
    assert np.array_equal(res["X"].astype(np.float32), out[1]["X"])
    # a rank-deficient refresh (two equal columns of V) is reported and leaves the state alone
    Vbad = V0.copy()
    Vbad[:, 2] = Vbad[:, 0]
    res = orc.lazy_dion_step(X, grads[0], np.zeros((m, n)), Vbad, 0.95, 0.01, True)
    assert res["status"] == orc.STATUS_BREAKDOWN
    assert np.array_equal(res["X"], X) and np.array_equal(res["V"], Vbad)
