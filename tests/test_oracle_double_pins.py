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


def test_breakdown_in_either_stage_leaves_everything_untouched():
    m, n, r1, r2 = 12, 10, 3, 4
    X, G, M1, V1, M2, V2 = problem(m, n, r1, r2, 5)
    bad1 = V1.copy(); bad1[:, 2] = bad1[:, 0]
    bad2 = V2.copy(); bad2[:, 3] = bad2[:, 1]
    for a, b in ((bad1, V2), (V1, bad2)):
        res = orc.double_dion_step(X, G, M1, a, M2, b, 0.99, 0.95, 0.01)
        assert res["status"] == orc.STATUS_BREAKDOWN
        assert np.array_equal(res["X"], X) and np.array_equal(res["M1"], M1) and np.array_equal(res["M2"], M2)
        assert np.array_equal(res["V1"], a) and np.array_equal(res["V2"], b)
