"""Pins of the CPU oracle against things other than itself: closed forms, a brute-force
Jacobi SVD, LAPACK's QR, a hand-computed rank-1 step, Gram-Schmidt in long double, published
known-answer vectors.  Each test is chosen so that a plausible slip in the oracle (dropped
term, wrong sign, transposed operand, old-vs-new Q) fails it.  CPU only."""
import os

import numpy as np
import pytest

from oracle import dion_oracle as orc
from jacobi_svd import jacobi_svd

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rand_problem(m, n, r, seed=0, mzero=False):
    rng = np.random.default_rng(seed)
    X = 0.02 * rng.standard_normal((m, n))
    G = 1e-2 * rng.standard_normal((m, n))
    M = np.zeros((m, n)) if mzero else 3e-2 * rng.standard_normal((m, n))
    Q, _ = orc.col_norm(rng.standard_normal((n, r)))
    return X, G, M, Q


def mgs2(Z):
    """Modified Gram-Schmidt applied twice, long double: an orth route independent of Householder."""
    A = np.array(Z, dtype=np.longdouble)
    for _ in range(2):
        for j in range(A.shape[1]):
            for k in range(j):
                A[:, j] -= np.dot(A[:, k], A[:, j]) * A[:, k]
            A[:, j] /= np.sqrt(np.dot(A[:, j], A[:, j]))
    return np.array(A, dtype=np.float64)


# ---------------------------------------------------------------- orth
@pytest.mark.parametrize("m,r", [(7, 3), (64, 64), (200, 37)])
def test_householder_is_the_qr_factor(m, r):
    Z = np.random.default_rng(m * r).standard_normal((m, r))
    P, T = orc.householder_qr(Z)
    assert np.abs(P.T @ P - np.eye(r)).max() < 1e-13            # orthonormal columns
    assert np.abs(np.tril(T, -1)).max() == 0.0                   # upper triangular
    assert np.all(np.diag(T) > 0)                                # sign convention
    assert np.abs(P @ T - Z).max() < 1e-13                       # it factors Z
    # library routine, sign-fixed: the QR factor of a full-rank matrix is unique
    Pl, Tl = np.linalg.qr(Z)
    s = np.sign(np.diag(Tl))
    assert np.abs(P - Pl * s).max() < 1e-12
    # classical route: Gram-Schmidt (long double) gives the same factor, signs included
    assert np.abs(P - mgs2(Z)).max() < 1e-12
    P2, T2 = orc.lapack_qr(Z)
    assert np.abs(P - P2).max() < 1e-12 and np.abs(T - T2).max() < 1e-12


def test_householder_cholesky_relation():
    # Cholesky-QR (Appendix A): T is the transposed Cholesky factor of Z^T Z
    Z = np.random.default_rng(5).standard_normal((90, 11))
    _, T = orc.householder_qr(Z)
    L = np.linalg.cholesky(Z.T @ Z)
    assert np.abs(T - L.T).max() < 1e-12


def test_orthonormalize_reports_rank_deficiency():
    Z = np.random.default_rng(1).standard_normal((30, 4))
    Z[:, 3] = Z[:, 1]
    assert orc.orthonormalize(Z)[2] == orc.STATUS_BREAKDOWN
    assert orc.orthonormalize(np.zeros((9, 2)))[2] == orc.STATUS_BREAKDOWN
    assert orc.orthonormalize(np.random.default_rng(2).standard_normal((30, 4)))[2] == orc.STATUS_OK


# ---------------------------------------------------------------- one step: invariants
@pytest.mark.parametrize("m,n,r", [(24, 16, 5), (16, 24, 8), (40, 40, 40)])
def test_step_invariants(m, n, r):
    X, G, M, Q = rand_problem(m, n, r, seed=m + n + r)
    mu, eta = 0.95, 0.01
    res = orc.dion_step(X, G, M, Q, mu, eta)
    P, R, B = res["P"], res["R"], M + G
    assert res["status"] == orc.STATUS_OK
    # P orthonormal
    assert np.abs(P.T @ P - np.eye(r)).max() < 1e-12
    # R = B^T P by an independent loop order
    R2 = np.zeros((n, r))
    for i in range(m):
        R2 += np.outer(B[i, :], P[i, :])
    assert np.abs(R - R2).max() < 1e-13
    # error feedback: M_new + (1-mu) P R^T reconstructs B; both forms of the equation agree
    assert np.abs(res["M"] + (1 - mu) * P @ R.T - B).max() < 1e-14
    beta = 1 - mu
    delta = B - P @ R.T
    assert np.abs(res["M"] - ((1 - beta) * B + beta * delta)).max() < 1e-14
    # basis independence: M_new = (I - (1-mu) Pi) B with Pi the projector on range(B Q) from
    # (a) Gram-Schmidt and (b) left singular vectors by brute-force Jacobi SVD
    Pa = mgs2(B @ Q)
    Ub, sb, _ = jacobi_svd(B @ Q)
    for basis in (Pa, Ub[:, :r]):
        Pi = basis @ basis.T
        assert np.abs(res["M"] - (B - (1 - mu) * Pi @ B)).max() < 1e-11
    # Q_new has unit columns and is ColNorm(R) (not of the old Q)
    # (the 1e-8 guard in the denominator shows up as 1e-8/||R_j||)
    sR = np.linalg.norm(R, axis=0)
    assert np.abs(np.linalg.norm(res["Q"], axis=0) - sR / (sR + orc.COLNORM_EPS)).max() < 1e-14
    assert np.abs(np.linalg.norm(res["Q"], axis=0) - 1).max() < 1e-5
    assert np.abs(res["Q"] * (sR + orc.COLNORM_EPS) - R).max() < 1e-14
    # closed form for the size of the weight update: ||P Q_new^T||_F^2 = trace(Q^T Q) = r
    dX = res["X"] - X
    assert abs(np.linalg.norm(dX) / (eta * np.sqrt(m / n) * np.sqrt(r)) - 1) < 1e-5
    # X moves against P Q_new^T (sign) with the NEW Q and sqrt(m/n), not sqrt(n/m)
    assert np.abs(dX + eta * np.sqrt(m / n) * P @ res["Q"].T).max() < 1e-15
    # Q_old^T R = T^T : lower triangular with positive diagonal => orth is the QR factor, not a rotation
    Tt = Q.T @ R
    assert np.abs(np.triu(Tt, 1)).max() < 1e-12
    assert np.all(np.diag(Tt) > 0)
    assert np.abs(Tt - res["T"].T).max() < 1e-12


def test_full_rank_is_plain_momentum():
    # r = n <= m, B of full column rank: P P^T B = B, hence M_new = mu * B exactly
    m, n = 20, 12
    X, G, M, Q = rand_problem(m, n, n, seed=3)
    for mu in (0.95, 0.3):
        res = orc.dion_step(X, G, M, Q, mu, 0.01)
        assert np.abs(res["M"] - mu * (M + G)).max() < 1e-13


def test_exact_low_rank_buffer_is_captured():
    m, n, r = 30, 22, 4
    rng = np.random.default_rng(11)
    B = rng.standard_normal((m, r)) @ rng.standard_normal((r, n))
    Q, _ = orc.col_norm(rng.standard_normal((n, r)))
    res = orc.dion_step(np.zeros((m, n)), B, np.zeros((m, n)), Q, 0.9, 0.01)
    assert np.abs(res["M"] - 0.9 * B).max() < 1e-12


def test_rank1_step_hand_computed():
    vals = {}
    with open(os.path.join(GOLD, "power_step_rank1.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            vals[k] = np.array([float(x) for x in v])
    B = np.array([[3.0, 0.0], [0.0, 4.0], [0.0, 0.0]])
    M = np.array([[1.0, 0.0], [0.0, 1.5], [0.0, 0.0]])
    G = B - M
    q = np.array([[0.6], [0.8]])
    mu, eta = 0.5, 0.1
    res = orc.dion_step(np.zeros((3, 2)), G, M, q, mu, eta)
    zz = vals["zz"][0]
    assert np.abs(res["Z"][:, 0] - vals["z"]).max() < 1e-15
    p = vals["z"] / np.sqrt(zz)
    assert np.abs(res["P"][:, 0] - p).max() < 1e-15
    assert np.abs(res["R"][:, 0] - vals["r_num"] / np.sqrt(zz)).max() < 1e-14
    qn = vals["r_num"] / np.sqrt(vals["rr_num"][0])
    assert np.abs(res["Q"][:, 0] - qn).max() < 1e-8          # the 1e-8 ColNorm guard
    prt = vals["prt_num"].reshape(3, 2) / zz
    assert np.abs(res["M"] - (B - 0.5 * prt)).max() < 1e-14
    assert np.abs(res["X"] + 0.1 * np.sqrt(1.5) * np.outer(p, qn)).max() < 1e-8
    assert abs(res["s"][0] - np.sqrt(vals["rr_num"][0] / zz)) < 1e-14


def test_tiny_brute_force_long_double():
    # every quantity recomputed with scalar loops in long double and classical Gram-Schmidt
    m, n, r = 6, 5, 3
    X, G, M, Q = rand_problem(m, n, r, seed=21)
    mu, eta = 0.8, 0.05
    ld = np.longdouble
    B = [[ld(M[i, j]) + ld(G[i, j]) for j in range(n)] for i in range(m)]
    Z = [[sum(B[i][j] * ld(Q[j, a]) for j in range(n)) for a in range(r)] for i in range(m)]
    P = [[ld(0)] * r for _ in range(m)]
    for a in range(r):
        v = [Z[i][a] for i in range(m)]
        for _ in range(2):
            for k in range(a):
                d = sum(P[i][k] * v[i] for i in range(m))
                v = [v[i] - d * P[i][k] for i in range(m)]
        nv = np.sqrt(sum(x * x for x in v))
        for i in range(m):
            P[i][a] = v[i] / nv
    R = [[sum(B[i][j] * P[i][a] for i in range(m)) for a in range(r)] for j in range(n)]
    s = [np.sqrt(sum(R[j][a] ** 2 for j in range(n))) for a in range(r)]
    res = orc.dion_step(X, G, M, Q, mu, eta)
    for i in range(m):
        for j in range(n):
            pr = sum(P[i][a] * R[j][a] for a in range(r))
            pq = sum(P[i][a] * R[j][a] / (s[a] + ld(orc.COLNORM_EPS)) for a in range(r))
            assert abs(float(B[i][j] - ld(1 - mu) * pr) - res["M"][i, j]) < 1e-14
            assert abs(float(ld(X[i, j]) - ld(eta) * np.sqrt(ld(m) / ld(n)) * pq) - res["X"][i, j]) < 1e-14


# ---------------------------------------------------------------- SVD fixed point and convergence
def test_svd_fixed_point():
    m, n, r = 18, 14, 4
    rng = np.random.default_rng(8)
    B = rng.standard_normal((m, n))
    U, sig, V = jacobi_svd(B)
    Vr, Ur = V[:, :r], U[:, :r]
    X = rng.standard_normal((m, n))
    mu, eta = 0.95, 0.02
    res = orc.dion_step(X, B, np.zeros((m, n)), Vr, mu, eta)
    sg = np.sign(np.sum(res["P"] * Ur, axis=0))
    assert np.abs(res["P"] * sg - Ur).max() < 1e-10
    assert np.abs(res["s"] - sig[:r]).max() < 1e-10                       # ||R_j|| = sigma_j
    assert np.abs(res["Q"] * sg - Vr).max() < 1e-7
    assert np.abs(res["X"] - (X - eta * np.sqrt(m / n) * Ur @ Vr.T)).max() < 1e-8
    assert np.abs(res["M"] - (B - (1 - mu) * (Ur * sig[:r]) @ Vr.T)).max() < 1e-10


def test_repeated_steps_converge_to_top_singular_subspace():
    # G = 0, mu = 1: M stays A, the steps are orthogonal iteration on A^T A.
    m, n, r = 24, 20, 3
    rng = np.random.default_rng(4)
    U0, _ = np.linalg.qr(rng.standard_normal((m, n)))
    V0, _ = np.linalg.qr(rng.standard_normal((n, n)))
    sig = np.concatenate([[10.0, 8.0, 6.0], 2.0 * 0.9 ** np.arange(n - 3)])   # gap 2/6
    A = (U0 * sig) @ V0.T
    Uj, sj, Vj = jacobi_svd(A)
    assert np.abs(sj - sig).max() < 1e-10
    M = A.copy()
    Q, _ = orc.col_norm(rng.standard_normal((n, r)))
    X = np.zeros((m, n))
    errs = []
    for _ in range(12):
        res = orc.dion_step(X, np.zeros((m, n)), M, Q, 1.0, 0.0)
        assert np.array_equal(res["M"], M)              # mu = 1: no error feedback
        Q = res["Q"]
        errs.append(np.linalg.norm(res["P"] @ res["P"].T - Uj[:, :r] @ Uj[:, :r].T, 2))
    rho2 = (2.0 / 6.0) ** 2
    for a, b in zip(errs[2:8], errs[3:9]):
        assert b <= 1.5 * rho2 * a + 1e-13              # contraction by about (sigma_{r+1}/sigma_r)^2
    assert errs[-1] < 1e-9
    # distinct sigma: columns converge individually, so P Q^T -> U_r V_r^T and ||R_j|| -> sigma_j
    for _ in range(120):
        res = orc.dion_step(X, np.zeros((m, n)), M, Q, 1.0, 0.0)
        Q = res["Q"]
    assert np.abs(res["P"] @ res["Q"].T - Uj[:, :r] @ Vj[:, :r].T).max() < 1e-8
    assert np.abs(res["s"] - sig[:r]).max() < 1e-8


# ---------------------------------------------------------------- symmetries
def test_sign_flip_invariance_and_permutation_dependence():
    m, n, r = 15, 13, 4
    X, G, M, Q = rand_problem(m, n, r, seed=6)
    a = orc.dion_step(X, G, M, Q, 0.95, 0.01)
    b = orc.dion_step(X, G, M, Q * np.array([1, -1, -1, 1.0]), 0.95, 0.01)
    assert np.abs(a["X"] - b["X"]).max() < 1e-15 and np.abs(a["M"] - b["M"]).max() < 1e-15
    c = orc.dion_step(X, G, M, Q[:, [2, 0, 3, 1]], 0.95, 0.01)
    assert np.abs(a["M"] - c["M"]).max() < 1e-13        # only range(Z) matters for M
    assert np.abs(a["X"] - c["X"]).max() > 1e-6         # but not for X: ColNorm is not rotation invariant


def test_linearity_of_the_two_products():
    # compressed data-parallel sync (Section 3.3): partial Z and R of replicas add up
    m, n, r = 10, 9, 3
    rng = np.random.default_rng(2)
    M1, M2 = rng.standard_normal((2, m, n))
    Q, _ = orc.col_norm(rng.standard_normal((n, r)))
    P, R, Z, _, _ = orc.power_iter1(M1 + M2, Q)
    assert np.abs(Z - (M1 @ Q + M2 @ Q)).max() < 1e-13
    assert np.abs(R - (M1.T @ P + M2.T @ P)).max() < 1e-13


def test_breakdown_leaves_state_untouched():
    m, n, r = 12, 10, 3
    X, G, M, Q = rand_problem(m, n, r, seed=9)
    Q[:, 2] = Q[:, 0]
    res = orc.dion_step(X, G, M, Q, 0.95, 0.01)
    assert res["status"] == orc.STATUS_BREAKDOWN
    assert np.array_equal(res["X"], X) and np.array_equal(res["M"], M) and np.array_equal(res["Q"], Q)
    res = orc.dion_step(X, np.zeros((m, n)), np.zeros((m, n)), rand_problem(m, n, r)[3], 0.95, 0.01)
    assert res["status"] == orc.STATUS_BREAKDOWN


def test_zero_column_colnorm_is_finite():
    R = np.random.default_rng(0).standard_normal((6, 3))
    R[:, 1] = 0
    Qn, s = orc.col_norm(R)
    assert np.all(np.isfinite(Qn)) and np.all(Qn[:, 1] == 0) and s[1] == 0


# ---------------------------------------------------------------- multi-step driver and entry forms
def test_run_steps_matches_manual_loop_and_checkpoint():
    m, n, r = 16, 12, 4
    X, _, _, Qraw = rand_problem(m, n, r, seed=13)
    rng = np.random.default_rng(14)
    grads = [np.float32(1e-2) * rng.standard_normal((m, n)).astype(np.float32) for _ in range(6)]
    M0, Q0 = orc.init_state(m, n, Qraw)
    assert np.all(M0 == 0) and np.abs(np.linalg.norm(Q0, axis=0) - 1).max() < 1e-7
    full = orc.run_steps(X, grads, M0, Q0, 0.95, 0.01)
    half = orc.run_steps(X, grads[:3], M0, Q0, 0.95, 0.01)
    rest = orc.run_steps(half[-1]["X"], grads[3:], half[-1]["M"], half[-1]["Q"], 0.95, 0.01)
    for k in ("X", "M", "Q"):
        assert full[-1][k].dtype == np.float32
        assert np.array_equal(full[-1][k], rest[-1][k])     # state = (X, M, Q) only


def test_entry_forms_match_full_step():
    m, n, r = 14, 11, 3
    X, G, M, Q = rand_problem(m, n, r, seed=17)
    res = orc.dion_step(X, G, M, Q, 0.9, 0.03)
    rows = [0, 5, 13, 7]
    assert np.abs(orc.entry_Z(M, G, Q, rows, [0, 2, 1, 1]) - res["Z"][rows, [0, 2, 1, 1]]).max() < 1e-14
    jr = [0, 10, 4, 4]
    assert np.abs(orc.entry_R(M, G, res["P"], jr, [0, 2, 1, 0]) - res["R"][jr, [0, 2, 1, 0]]).max() < 1e-14
    xs, ms = orc.entry_update(X, G, M, res["P"], res["R"], 0.9, 0.03, rows, jr)
    assert np.abs(xs - res["X"][rows, jr]).max() < 1e-14
    assert np.abs(ms - res["M"][rows, jr]).max() < 1e-14


def test_block_forms_match_full_step_and_explicit_loops():
    m, n, r = 19, 13, 4
    X, G, M, Q = rand_problem(m, n, r, seed=23)
    mu, eta = 0.9, 0.03
    res = orc.dion_step(X, G, M, Q, mu, eta)
    rows, cols_r, rows_n, cols_n = [0, 18, 7], [3, 0], [12, 0, 5], [1, 12]
    assert np.abs(orc.rows_Z(M, G, Q, rows) - res["Z"][rows, :]).max() < 1e-13
    assert np.abs(orc.cols_Z(M, G, Q, cols_r, chunk=5) - res["Z"][:, cols_r]).max() < 1e-13
    assert np.abs(orc.rows_R(M, G, res["P"], rows_n) - res["R"][rows_n, :]).max() < 1e-13
    assert np.abs(orc.cols_R(M, G, res["P"], cols_r, chunk=5) - res["R"][:, cols_r]).max() < 1e-13
    xr, mr = orc.rows_update(X, G, M, res["P"], res["R"], mu, eta, rows)
    assert np.abs(xr - res["X"][rows, :]).max() < 1e-13 and np.abs(mr - res["M"][rows, :]).max() < 1e-13
    xc, mc = orc.cols_update(X, G, M, res["P"], res["R"], mu, eta, cols_n)
    assert np.abs(xc - res["X"][:, cols_n]).max() < 1e-13 and np.abs(mc - res["M"][:, cols_n]).max() < 1e-13
    # one entry of each by explicit loops over the defining sums (catches a transposed operand in a block form)
    i, a, j = 7, 3, 12
    B = [[float(M[p, q]) + float(G[p, q]) for q in range(n)] for p in range(m)]
    z = sum(B[i][q] * float(Q[q, a]) for q in range(n))
    assert abs(orc.rows_Z(M, G, Q, [i])[0, a] - z) < 1e-13 and abs(orc.cols_Z(M, G, Q, [a])[i, 0] - z) < 1e-13
    rr = sum(B[p][j] * res["P"][p, a] for p in range(m))
    assert abs(orc.rows_R(M, G, res["P"], [j])[0, a] - rr) < 1e-13 and abs(orc.cols_R(M, G, res["P"], [a])[j, 0] - rr) < 1e-13
    s = [np.sqrt(sum(res["R"][q, c] ** 2 for q in range(n))) for c in range(r)]
    mn = B[i][j] - (1 - mu) * sum(res["P"][i, c] * res["R"][j, c] for c in range(r))
    xn = float(X[i, j]) - eta * np.sqrt(m / n) * sum(res["P"][i, c] * res["R"][j, c] / (s[c] + orc.COLNORM_EPS) for c in range(r))
    xr, mr = orc.rows_update(X, G, M, res["P"], res["R"], mu, eta, [i])
    xc, mc = orc.cols_update(X, G, M, res["P"], res["R"], mu, eta, [j])
    assert abs(xr[0, j] - xn) < 1e-13 and abs(mr[0, j] - mn) < 1e-13
    assert abs(xc[i, 0] - xn) < 1e-13 and abs(mc[i, 0] - mn) < 1e-13


# ---------------------------------------------------------------- counter-based generator
def test_philox_known_answers():
    with open(os.path.join(GOLD, "philox4x32_10_kat.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        w = [int(x, 16) for x in row]
        out = orc.philox4x32_10(np.array([w[0:4]]), (w[4], w[5]))[0]
        assert [int(x) for x in out] == w[6:10]


def test_gaussian_fill_statistics_and_indexing():
    g = orc.gaussian_fill(200001, seed=7, stream=3)
    assert abs(g.mean()) < 0.01 and abs(g.std() - 1) < 0.01
    assert abs(np.mean(g ** 4) - 3) < 0.1                     # Gaussian kurtosis
    assert abs(np.corrcoef(g[0::2][:100000], g[1::2][:100000])[0, 1]) < 0.01
    assert np.array_equal(g[:1001], orc.gaussian_fill(1001, seed=7, stream=3))   # prefix-stable
    assert not np.array_equal(g[:100], orc.gaussian_fill(100, seed=7, stream=4))
    # Box-Muller pair: g0^2 + g1^2 = -2 ln u1 with u1 = (w0+1)/2^32 from the block's first word
    w = orc.philox4x32_10(np.array([[0, 0, 3, 0]]), (7, 0))[0]
    assert abs(g[0] ** 2 + g[1] ** 2 + 2 * np.log((float(w[0]) + 1) / 2 ** 32)) < 1e-12
