"""Pins of the transposed form of the Dion step in the CPU oracle (Section 4.3, "Other variants") against things
other than the function itself: the already pinned standard step applied to the transposed problem, closed
forms, the SVD fixed point (where both forms give the same update), an explicit-loop evaluation.  CPU only."""
import numpy as np

from oracle import dion_oracle as orc
from jacobi_svd import jacobi_svd


def problem(m, n, r, seed):
    rng = np.random.default_rng(seed)
    X = 0.02 * rng.standard_normal((m, n))
    G = 1e-2 * rng.standard_normal((m, n))
    M = 3e-2 * rng.standard_normal((m, n))
    Vt, _ = orc.col_norm(rng.standard_normal((m, r)))
    return X, G, M, Vt


def test_equals_the_standard_step_on_the_transposed_problem():
    for (m, n, r) in [(14, 9, 3), (9, 14, 4), (12, 12, 12)]:
        X, G, M, Vt = problem(m, n, r, m * n)
        mu, eta = 0.9, 0.05
        res = orc.dion_step_transposed(X, G, M, Vt, mu, eta)
        std = orc.dion_step(X.T, G.T, M.T, Vt, mu, eta)      # n x m problem, factor on its "column" side (m)
        assert np.abs(res["M"] - std["M"].T).max() < 1e-13
        assert np.abs(res["Vt"] - std["Q"]).max() < 1e-12
        assert np.abs(res["Pt"] - std["P"]).max() < 1e-12
        # the standard step scales by sqrt(rows/cols) of what it is given, i.e. sqrt(n/m); the parameter's own
        # factor sqrt(m/n) is kept in the transposed form
        upd_std = (std["X"] - X.T).T / np.sqrt(n / m)
        assert np.abs((res["X"] - X) / np.sqrt(m / n) - upd_std).max() < 1e-12


def test_closed_forms():
    m, n, r = 30, 22, 5
    X, G, M, Vt = problem(m, n, r, 7)
    mu, eta = 0.95, 0.01
    res = orc.dion_step_transposed(X, G, M, Vt, mu, eta)
    B, P = M + G, res["Pt"]
    assert np.abs(P.T @ P - np.eye(r)).max() < 1e-12
    assert np.abs(res["M"] + (1 - mu) * res["Rt"] @ P.T - B).max() < 1e-13
    assert np.abs(res["M"] @ P - mu * (B @ P)).max() < 1e-12            # damped on span(P'), P' on the column side
    comp = np.eye(n) - P @ P.T
    assert np.abs(res["M"] @ comp - B @ comp).max() < 1e-12
    assert abs(np.linalg.norm(res["X"] - X) - eta * np.sqrt(m / n) * np.sqrt(r)) < 1e-8
    assert np.abs(np.linalg.norm(res["Vt"], axis=0) - 1).max() < 1e-7
    T = Vt.T @ res["Rt"]            # = (P'^T B^T Vt)^T = T'^T: lower triangular, positive diagonal
    assert np.abs(np.triu(T, 1)).max() < 1e-12 and np.all(np.diag(T) > 0)


def test_explicit_loops_rank_one():
    m, n = 4, 3
    rng = np.random.default_rng(1)
    X, G, M = rng.standard_normal((3, m, n))
    v = rng.standard_normal((m, 1))
    mu, eta = 0.6, 0.2
    res = orc.dion_step_transposed(X, G, M, v, mu, eta)
    B = M + G
    z = [sum(B[i][j] * v[i][0] for i in range(m)) for j in range(n)]
    nz = np.sqrt(sum(t * t for t in z))
    p = [t / nz for t in z]
    rr = [sum(B[i][j] * p[j] for j in range(n)) for i in range(m)]
    nr = np.sqrt(sum(t * t for t in rr))
    for i in range(m):
        for j in range(n):
            assert abs(res["M"][i][j] - (B[i][j] - (1 - mu) * rr[i] * p[j])) < 1e-13
            assert abs(res["X"][i][j] - (X[i][j] - eta * np.sqrt(m / n) * rr[i] / (nr + 1e-8) * p[j])) < 1e-13


def test_svd_fixed_point_gives_the_same_update_as_the_standard_form():
    m, n, r = 18, 14, 4
    rng = np.random.default_rng(8)
    B = rng.standard_normal((m, n))
    U, sig, V = jacobi_svd(B)
    Ur, Vr = U[:, :r], V[:, :r]
    X = rng.standard_normal((m, n))
    mu, eta = 0.95, 0.02
    res = orc.dion_step_transposed(X, B, np.zeros((m, n)), Ur, mu, eta)
    sg = np.sign(np.sum(res["Pt"] * Vr, axis=0))
    assert np.abs(res["Pt"] * sg - Vr).max() < 1e-10
    assert np.abs(res["s"] - sig[:r]).max() < 1e-10
    assert np.abs(res["Vt"] * sg - Ur).max() < 1e-7
    assert np.abs(res["X"] - (X - eta * np.sqrt(m / n) * Ur @ Vr.T)).max() < 1e-8
    std = orc.dion_step(X, B, np.zeros((m, n)), Vr, mu, eta)
    assert np.abs(res["X"] - std["X"]).max() < 1e-8 and np.abs(res["M"] - std["M"]).max() < 1e-9


def test_breakdown_leaves_state_untouched():
    m, n, r = 12, 10, 3
    X, G, M, Vt = problem(m, n, r, 2)
    Vt[:, 2] = Vt[:, 0]
    res = orc.dion_step_transposed(X, G, M, Vt, 0.95, 0.01)
    assert res["status"] == orc.STATUS_BREAKDOWN
    assert np.array_equal(res["X"], X) and np.array_equal(res["M"], M) and np.array_equal(res["Vt"], Vt)
