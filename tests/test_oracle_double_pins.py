"""Pins of the Double Dion step of the CPU oracle (Section 5.2, Double Dion algorithm): it must equal two chained
standard steps (already pinned) with the stage-1 sketch as the second stage's gradient; closed forms; the case
r1 = full rank, where the sketch is the whole buffer; breakdown handling.  CPU only."""
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


def test_breakdown_handling():
    m, n, r1, r2 = 12, 10, 3, 4
    X, G, M1, V1, M2, V2 = problem(m, n, r1, r2, 5)
    bad1 = V1.copy(); bad1[:, 2] = bad1[:, 0]
    bad2 = V2.copy(); bad2[:, 3] = bad2[:, 1]
    # stage 1 fails: nothing moves
    res = orc.double_dion_step(X, G, M1, bad1, M2, V2, 0.99, 0.95, 0.01)
    assert res["status"] == orc.STATUS_BREAKDOWN
    assert np.array_equal(res["X"], X) and np.array_equal(res["M1"], M1) and np.array_equal(res["M2"], M2)
    assert np.array_equal(res["V1"], bad1) and np.array_equal(res["V2"], V2)
    # stage 2 fails: stage 1 has taken its (ordinary) step, M2 only accumulates the sketch, X and V2 are untouched
    res = orc.double_dion_step(X, G, M1, V1, M2, bad2, 0.99, 0.95, 0.01)
    assert res["status"] == orc.STATUS_BREAKDOWN
    s1 = orc.dion_step(np.zeros((m, n)), G, M1, V1, 0.99, 0.0)
    assert np.array_equal(res["M1"], s1["M"]) and np.array_equal(res["V1"], s1["Q"])
    assert np.array_equal(res["X"], X) and np.array_equal(res["V2"], bad2)
    assert np.array_equal(res["M2"], M2 + s1["P"] @ s1["R"].T)


def test_cold_start_grows_m2_into_full_rank():
    # from M2 = 0 the second stage sees a buffer of rank r1, 2 r1, ... and can only start once that reaches r2
    m, n, r1, r2 = 20, 16, 2, 6
    rng = np.random.default_rng(6)
    X = rng.standard_normal((m, n))
    M1, M2 = np.zeros((m, n)), np.zeros((m, n))
    V1, _ = orc.col_norm(rng.standard_normal((n, r1)))
    V2, _ = orc.col_norm(rng.standard_normal((n, r2)))
    statuses = []
    for t in range(5):
        res = orc.double_dion_step(X, rng.standard_normal((m, n)), M1, V1, M2, V2, 0.9, 0.95, 0.01)
        statuses.append(res["status"])
        X, M1, V1, M2, V2 = res["X"], res["M1"], res["V1"], res["M2"], res["V2"]
        assert np.linalg.matrix_rank(M2) == min((t + 1) * r1, n) or res["status"] == orc.STATUS_OK
    assert statuses[:2] == [orc.STATUS_BREAKDOWN] * 2 and statuses[2:] == [orc.STATUS_OK] * 3
