"""Pins of the Double Dion step of the CPU oracle (Section 5.2, Double Dion algorithm): it must equal two chained
standard steps (already pinned) with the stage-1 sketch as the second stage's gradient; closed forms; the case
r1 = full rank, where the sketch is the whole buffer; the orthonormalisation of stage 2 on linearly dependent columns
(against the library QR of the independent ones, and a cold start worked out from a brute-force SVD of the sketch).
CPU only."""
import numpy as np

from oracle import dion_oracle as orc


def problem(m, n, r1, r2, seed):
    rng = np.random.default_rng(seed)
    X = 0.02 * rng.standard_normal((m, n))
    G = 1e-2 * rng.standard_normal((m, n))
    M1 = 3e-2 * rng.standard_normal((m, n))
    M2 = 3e-2 * rng.standard_normal((m, n))
    V1, _ = orc.col_norm(rng.standard_normal((n, r1)))
    V2, _ = orc.col_norm(rng.standard_normal((n, r2)))
    return X, G, M1, V1, M2, V2


def test_equals_two_chained_standard_steps():
    m, n, r1, r2 = 20, 14, 2, 5
    X, G, M1, V1, M2, V2 = problem(m, n, r1, r2, 1)
    mu1, mu2, eta = 0.999, 0.95, 0.01
    res = orc.double_dion_step(X, G, M1, V1, M2, V2, mu1, mu2, eta)
    s1 = orc.dion_step(np.zeros((m, n)), G, M1, V1, mu1, 0.0)            # stage 1 moves no weights
    D = s1["P"] @ s1["R"].T
    assert np.abs(res["D"] - D).max() < 1e-14
    assert np.abs(res["M1"] - s1["M"]).max() < 1e-14 and np.abs(res["V1"] - s1["Q"]).max() < 1e-14
    s2 = orc.dion_step(X, D, M2, V2, mu2, eta)                           # the sketch is stage 2's gradient
    for a, b in (("X", "X"), ("M2", "M"), ("V2", "Q")):
        assert np.abs(res[a] - s2[b]).max() < 1e-14


def test_closed_forms():
    m, n, r1, r2 = 24, 18, 3, 6
    X, G, M1, V1, M2, V2 = problem(m, n, r1, r2, 2)
    mu1, mu2, eta = 0.9, 0.95, 0.02
    res = orc.double_dion_step(X, G, M1, V1, M2, V2, mu1, mu2, eta)
    D = res["D"]
    assert np.linalg.matrix_rank(D) == r1
    assert np.abs(res["M1"] + (1 - mu1) * D - (M1 + G)).max() < 1e-13            # error feedback of stage 1
    assert abs(np.linalg.norm(res["X"] - X) - eta * np.sqrt(m / n) * np.sqrt(r2)) < 1e-8


def test_full_rank_stage_one_passes_the_whole_buffer_on():
    m, n, r2 = 16, 6, 3
    X, G, M1, V1, M2, V2 = problem(m, n, n, r2, 4)            # r1 = n: U1 U1^T B1 = B1
    mu1, mu2, eta = 0.9, 0.95, 0.02
    res = orc.double_dion_step(X, G, M1, V1, M2, V2, mu1, mu2, eta)
    assert np.abs(res["D"] - (M1 + G)).max() < 1e-12
    assert np.abs(res["M1"] - mu1 * (M1 + G)).max() < 1e-12
    s2 = orc.dion_step(X, M1 + G, M2, V2, mu2, eta)
    assert np.abs(res["X"] - s2["X"]).max() < 1e-11


def test_stage_one_breakdown_leaves_everything_untouched():
    m, n, r1, r2 = 12, 10, 3, 4
    X, G, M1, V1, M2, V2 = problem(m, n, r1, r2, 5)
    bad1 = V1.copy(); bad1[:, 2] = bad1[:, 0]
    res = orc.double_dion_step(X, G, M1, bad1, M2, V2, 0.99, 0.95, 0.01)
    assert res["status"] == orc.STATUS_BREAKDOWN
    assert np.array_equal(res["X"], X) and np.array_equal(res["M1"], M1) and np.array_equal(res["M2"], M2)
    assert np.array_equal(res["V1"], bad1) and np.array_equal(res["V2"], V2)


# ---- the orthonormalisation of stage 2: columns that depend on the ones before them

def test_dependent_orthonormalisation_equals_the_standard_one_at_full_rank():
    rng = np.random.default_rng(11)
    Z = rng.standard_normal((30, 7))
    P0, _, status = orc.orthonormalize(Z)
    for method in ("householder", "lapack"):
        P, keep, _ = orc.orthonormalize_dependent(Z, method)
        assert status == orc.STATUS_OK and keep.all() and np.abs(P - P0).max() < 1e-13


def test_dependent_columns_are_dropped_and_the_rest_is_the_qr_factor_of_the_rest():
    rng = np.random.default_rng(12)
    Z = rng.standard_normal((40, 9))
    Z[:, 4] = 2.0 * Z[:, 1] - 0.5 * Z[:, 3]          # depends on earlier columns
    Z[:, 6] = 0.0                                     # a zero column
    Z[:, 8] = Z[:, 7] + 1e-3 * Z[:, 8]               # nearly parallel to column 7: squared sine about 1e-6 < RANK_TOL
    want = np.array([1, 1, 1, 1, 0, 1, 0, 1, 0], dtype=bool)
    Pref, _ = orc.lapack_qr(Z[:, want])               # library QR of the independent columns alone
    for method in ("householder", "lapack"):
        P, keep, ratio = orc.orthonormalize_dependent(Z, method)
        assert np.array_equal(keep, want)
        assert ratio[4] < 1e-25 and ratio[6] == 0.0 and 1e-7 < ratio[8] < 1e-5 and abs(ratio[0] - 1.0) < 1e-12
        # forcing a borderline decision the other way: column 8 kept, column 5 dropped
        f = -np.ones(9, dtype=int); f[8] = 1; f[5] = 0
        Pf, keepf, _ = orc.orthonormalize_dependent(Z, method, forced=f)
        wantf = want.copy(); wantf[8] = True; wantf[5] = False
        assert np.array_equal(keepf, wantf) and np.abs(Pf[:, wantf] - orc.lapack_qr(Z[:, wantf])[0]).max() < 1e-9
        assert np.all(P[:, ~want] == 0.0)
        assert np.abs(P[:, want] - Pref).max() < 1e-12
        # what defines the factor: orthonormal, spans the same nested subspaces, positive diagonal
        T = P[:, want].T @ Z[:, want]
        assert np.abs(np.tril(T, -1)).max() < 1e-12 and np.all(np.diag(T) > 0)
    # a column just inside / outside the threshold: squared sine s2 against RANK_TOL
    for s2, expect in ((0.5 * orc.RANK_TOL, False), (2.0 * orc.RANK_TOL, True)):
        a = rng.standard_normal(25); a /= np.linalg.norm(a)
        b = rng.standard_normal(25); b -= a * (a @ b); b /= np.linalg.norm(b)
        Z2 = np.stack([a, np.sqrt(1 - s2) * a + np.sqrt(s2) * b], axis=1)
        for method in ("householder", "lapack"):
            assert orc.orthonormalize_dependent(Z2, method)[1][1] == expect


def test_cold_start_moves_the_weights_with_the_rank_that_is_there():
    # From M2 = 0 the buffer of stage 2 is the rank-r1 sketch.  What a QR-based step yields then, written without the
    # oracle's routine: with D = U S V^T (brute-force Jacobi SVD, rank r1), the first r1 columns of Z = D V2 span
    # range(D) and the rest depend on them; P1 = U Qf with Qf Tf the QR factor of the r1 x r1 matrix S V^T V2[:, :r1];
    # M2_new = D - beta2 P1 P1^T D = mu2 D;  X moves by eta sqrt(m/n) P1 ColNorm(D^T P1)^T.
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from jacobi_svd import jacobi_svd
    m, n, r1, r2 = 22, 15, 3, 7
    X, G, M1, V1, _, V2 = problem(m, n, r1, r2, 21)
    mu1, mu2, eta = 0.999, 0.95, 0.01
    res = orc.double_dion_step(X, G, M1, V1, np.zeros((m, n)), V2, mu1, mu2, eta)
    assert res["status"] == orc.STATUS_OK
    assert np.array_equal(res["keep"], np.arange(r2) < r1)
    D = res["D"]
    U, S, Vr = jacobi_svd(D)                          # D = U diag(S) Vr^T, singular values in descending order
    assert S[r1 - 1] > 1e-3 and S[r1] < 1e-12 * S[0]  # rank r1 exactly
    U, S, Vr = U[:, :r1], S[:r1], Vr[:, :r1]
    Qf, Tf = np.linalg.qr((S[:, None] * Vr.T) @ V2[:, :r1])
    Qf = Qf * np.where(np.diag(Tf) < 0, -1.0, 1.0)[None, :]
    P1 = U @ Qf
    W1 = D.T @ P1
    Q1 = W1 / (np.linalg.norm(W1, axis=0) + orc.COLNORM_EPS)
    Xref = X - eta * np.sqrt(m / n) * P1 @ Q1.T
    assert np.abs(res["X"] - Xref).max() < 1e-12
    assert np.linalg.norm(res["X"] - X) > 0.5 * eta * np.sqrt(m / n) * np.sqrt(r1)      # the weights do move
    assert abs(np.linalg.norm(res["X"] - X) - eta * np.sqrt(m / n) * np.sqrt(r1)) < 1e-8
    assert np.abs(res["M2"] - mu2 * D).max() < 1e-13
    assert np.abs(res["V2"][:, :r1] - Q1).max() < 1e-12
    assert np.array_equal(res["V2"][:, r1:], V2[:, r1:])                                # dependent columns keep their factor
    # the same through the pinned standard step of rank r1 on the sketch
    s2 = orc.dion_step(X, D, np.zeros((m, n)), V2[:, :r1], mu2, eta)
    assert np.abs(res["X"] - s2["X"]).max() < 1e-12 and np.abs(res["M2"] - s2["M"]).max() < 1e-12


def test_rank_of_stage_two_grows_by_r1_per_step_until_full():
    m, n, r1, r2 = 20, 16, 2, 6
    rng = np.random.default_rng(6)
    X = rng.standard_normal((m, n))
    M1, M2 = np.zeros((m, n)), np.zeros((m, n))
    V1, _ = orc.col_norm(rng.standard_normal((n, r1)))
    V2, _ = orc.col_norm(rng.standard_normal((n, r2)))
    ranks = []
    for t in range(5):
        Xo = X
        res = orc.double_dion_step(X, rng.standard_normal((m, n)), M1, V1, M2, V2, 0.9, 0.95, 0.01)
        assert res["status"] == orc.STATUS_OK
        X, M1, V1, M2, V2 = res["X"], res["M1"], res["V1"], res["M2"], res["V2"]
        k = int(res["keep"].sum())
        ranks.append(k)
        assert abs(np.linalg.norm(X - Xo) - 0.01 * np.sqrt(m / n) * np.sqrt(k)) < 1e-8
        assert np.abs(np.linalg.norm(V2, axis=0) - 1).max() < 1e-7                       # every column of V2 stays a unit vector
    assert ranks == [2, 4, 6, 6, 6]


def test_lapack_and_householder_variants_agree_on_a_deficient_stage_two():
    m, n, r1, r2 = 26, 17, 2, 6
    X, G, M1, V1, _, V2 = problem(m, n, r1, r2, 31)
    a = orc.double_dion_step(X, G, M1, V1, np.zeros((m, n)), V2, 0.99, 0.95, 0.01, "householder")
    b = orc.double_dion_step(X, G, M1, V1, np.zeros((m, n)), V2, 0.99, 0.95, 0.01, "lapack")
    assert np.array_equal(a["keep"], b["keep"])
    for k in ("X", "M1", "V1", "M2", "V2"):
        assert np.abs(a[k] - b[k]).max() < 1e-12
