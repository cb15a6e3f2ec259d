"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

A full fp64 oracle step of the Llama-3-405B MLP shape (16384 x 53248, r up to 4096) takes many minutes
on the host, so that configuration is checked stage by stage instead: every stage's output is compared
with the oracle's definition on whole rows and whole columns that cover every tile of the producing kernel,
evaluated from that stage's actual inputs,
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


def seg_relf(got, ref, seg, axis):
    """Relative Frobenius error of every length-`seg` segment along `axis` (one number per tile-sized piece of each
    sampled row or column), so that an error confined to one tile shows at full size."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if axis == 0:
        got, ref = got.T, ref.T
    k, length = ref.shape
    assert length % seg == 0
    d = (got - ref).reshape(k, length // seg, seg)
    return np.sqrt((d ** 2).sum(-1)) / np.maximum(np.sqrt((ref.reshape(k, length // seg, seg) ** 2).sum(-1)), 1e-300)


def one_per_tile(rng, total, tile):
    """One random index inside every block of `tile` consecutive indices."""
    return np.arange(0, total, tile) + rng.integers(0, tile, total // tile)


@pytest.mark.parametrize("r", [1024, 4096])
def test_c4_llama_mlp_stagewise(r):
    """Every stage against its defining formula in fp64, evaluated from that stage's own inputs, on whole rows and
    whole columns that touch every tile row and every tile column of the kernel that produced it (256 x 256 tiles for
    the two products, 256 x 128 for the fused update), compared tile-sized segment by segment."""
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
    TOL = 2e-2
    # stage 1: Z = (M+G) Q: one whole row per 256-row tile, one whole column per 256-column tile
    zr, zc = one_per_tile(rng, m, 256), one_per_tile(rng, r, 256)
    e = seg_relf(Z[zr, :], orc.rows_Z(m_in, g32, q_in, zr), 256, 1)
    print("Z rows: %d segments, worst %.2e" % (e.size, e.max()), flush=True)
    assert e.max() <= TOL
    e = seg_relf(Z[:, zc], orc.cols_Z(m_in, g32, q_in, zc), 256, 0)
    print("Z cols: %d segments, worst %.2e" % (e.size, e.max()), flush=True)
    assert e.max() <= TOL
    # stage 2: P is THE QR factor of Z (unique): orthonormal, P^T Z upper triangular with positive diagonal, P T = Z
    P64 = P.astype(np.float64)
    gram = P64.T @ P64
    assert np.abs(gram - np.eye(r)).max() <= 1e-4
    T = P64.T @ Z.astype(np.float64)
    tscale = np.abs(np.diag(T)).min()
    assert np.all(np.diag(T) > 0)
    assert np.abs(np.tril(T, -1)).max() <= 1e-3 * np.abs(np.diag(T)).max()
    pr = one_per_tile(rng, m, 256)
    e = seg_relf(P64[pr, :] @ T, Z[pr, :], 256, 1)
    print("orth checked, min/max diag(T) %.3e %.3e, P T = Z worst segment %.2e" % (tscale, np.abs(np.diag(T)).max(), e.max()), flush=True)
    assert e.max() <= 1e-3
    # stage 3: R = (M+G)^T P: one whole row per 256-row tile of the n side, one whole column per 256-column tile
    rr_, rc = one_per_tile(rng, n, 256), one_per_tile(rng, r, 256)
    e = seg_relf(R[rr_, :], orc.rows_R(m_in, g32, P, rr_), 256, 1)
    print("R rows: %d segments, worst %.2e" % (e.size, e.max()), flush=True)
    assert e.max() <= TOL
    e = seg_relf(R[:, rc], orc.cols_R(m_in, g32, P, rc), 256, 0)
    print("R cols: %d segments, worst %.2e" % (e.size, e.max()), flush=True)
    assert e.max() <= TOL
    # stage 4: column norms and the new Q
    s = gp.debug(0, B.DEBUG_S)[:, 0] if gp.debug(0, B.DEBUG_S).ndim == 2 else gp.debug(0, B.DEBUG_S)
    sref = np.sqrt(np.sum(R.astype(np.float64) ** 2, axis=0))
    assert np.abs(s.reshape(-1)[:r] - sref).max() <= 1e-5 * sref.max()
    assert relf(Q, R / (sref + orc.COLNORM_EPS)) <= 1e-6
    # stage 5: the fused update from the factors it actually used: one whole row per 256-row tile and one whole
    # column per 128-column tile of M_new and X_new, and of the updates themselves (X moves by about 1e-4 of its size
    # per step, so the error of the update is the sharper test; fp32 rounding of X adds 1e-7 |X| to it)
    ur, uc = one_per_tile(rng, m, 256), one_per_tile(rng, n, 128)
    for name, idx, axis, seg in (("rows", ur, 1, 128), ("cols", uc, 0, 256)):
        if axis == 1:
            xs, ms = orc.rows_update(x_in, g32, m_in, P, R, MU, ETA, idx)
            xg, mg, x0, b0 = X[idx, :], M[idx, :], x_in[idx, :], m_in[idx, :].astype(np.float64) + g32[idx, :]
        else:
            xs, ms = orc.cols_update(x_in, g32, m_in, P, R, MU, ETA, idx)
            xg, mg, x0, b0 = X[:, idx], M[:, idx], x_in[:, idx], m_in[:, idx].astype(np.float64) + g32[:, idx]
        ex, em = seg_relf(xg, xs, seg, axis), seg_relf(mg, ms, seg, axis)
        edx = seg_relf(xg.astype(np.float64) - x0, xs - x0, seg, axis)
        edm = seg_relf(mg.astype(np.float64) - b0, ms - b0, seg, axis)
        print("update %s: %d segments, worst X %.2e M %.2e dX %.2e dM %.2e" % (name, ex.size, ex.max(), em.max(), edx.max(), edm.max()), flush=True)
        assert ex.max() <= TOL and em.max() <= TOL
        assert edx.max() <= TOL + 1e-3 and edm.max() <= TOL     # (dX: plus the fp32 rounding of X, see above)
    # whole-matrix digests: M_new y and X_new y for Gaussian probe vectors y against the update rule evaluated in fp64
    # from the factors (E ||E y||^2 = ||E||_F^2 for Gaussian y, so an error anywhere in the matrices shows up here)
    def matvec(A, y, extra=None):                     # fp64 product of an fp32 (or bf16-as-fp32) matrix, by row blocks
        out = np.empty(A.shape[0])
        for i in range(0, A.shape[0], 1024):
            blk = A[i:i + 1024].astype(np.float64)
            if extra is not None:
                blk += extra[i:i + 1024]
            out[i:i + 1024] = blk @ y
        return out
    P64r, R64, Q64 = P.astype(np.float64), R.astype(np.float64), Q.astype(np.float64)
    for probe in range(2):
        y = np.random.default_rng(100 + probe).standard_normal(n)
        by = matvec(m_in, y, g32)                                   # (M + G) y
        pr_y = P64r @ (R64.T @ y)
        pq_y = P64r @ (Q64.T @ y)
        em = np.linalg.norm(matvec(M, y) - (by - (1 - MU) * pr_y)) / np.linalg.norm((1 - MU) * pr_y)
        ex = np.linalg.norm((matvec(X, y) - matvec(x_in, y)) + ETA * np.sqrt(m / n) * pq_y) / np.linalg.norm(ETA * np.sqrt(m / n) * pq_y)
        print("probe %d: error of the M update %.2e, of the X update %.2e (relative to the update's image of y)" % (probe, em, ex), flush=True)
        assert em <= TOL and ex <= TOL + 1e-2          # (X: plus the fp32 rounding of X itself, as above)
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


def test_fallback_orthonormalisation_at_8192_bf16():
    """cond(B Q) of a few 1e4 at 8192 x 8192, r = 2048, bf16 operands: the default mode reports a breakdown; with the
    fallback mode the same call completes on the device.  The thin-QR factor is pinned by what defines it, measured on
    the library's own Z (the products of this mode round their operands to bf16, and at this condition number the
    factor of the rounded product is far from the factor of the exact one); the stages after it against their formulas
    from their own inputs."""
    m = n = 8192
    r = 2048
    g = inputs.structured_gradient(m, n, 0, k=r, noise=1e-4, decay=1.0, bf16=True)
    g32 = inputs.bf16_bits_to_f32(g).astype(np.float64)
    gp = GpuProblem([(m, n, r)], True, "bf16")
    B = gp.B
    gp.upload_grads([g])
    x_in, m_in, q_in = gp.host()
    assert gp.step(MU, ETA) == (B.DION_NUM_BREAKDOWN, 0)
    for u, v in zip((x_in, m_in, q_in), gp.host()):
        assert np.array_equal(u, v)
    print("default mode reported the breakdown", flush=True)
    # Z = bf16(B) bf16(Q) as the library formed it: the same in both steps (same inputs, same kernel); taken now because
    # the fallback passes use its buffer
    Z = gp.debug(0, B.DEBUG_Z)[:, :r].astype(np.float64)
    B.dion_set_orth_mode(gp.state, B.DION_ORTH_CHOLQR2_FALLBACK)
    assert gp.step(MU, ETA) == (0, -1)
    P = gp.debug(0, B.DEBUG_P)[:, :r].astype(np.float64)
    R = gp.debug(0, B.DEBUG_R)[:, :r].astype(np.float64)
    X, M, Q = gp.host()
    Bm = m_in.astype(np.float64) + g32
    w = np.linalg.eigvalsh(Z.T @ Z)
    cond = float(np.sqrt(w[-1] / w[0]))
    assert 1e4 < cond < 1e5, cond
    assert relf(Z, Bm @ q_in.astype(np.float64)) < 1e-2                # Z itself: bf16 operands
    T = P.T @ Z
    orth = float(np.abs(P.T @ P - np.eye(r)).max())
    resid = relf(P @ np.triu(T), Z)
    print("cond %.3g orth %.2e resid %.2e" % (cond, orth, resid), flush=True)
    assert orth < 1e-5 and resid < 1e-5 and np.min(np.diag(T)) > 0
    # the rest of the step from this P, bf16-operand tolerances
    TOL = 2e-2
    assert relf(R, Bm.T @ P) < TOL
    Qn, _ = orc.col_norm(R)
    assert relf(Q, Qn) < 1e-5
    assert relf(M, Bm - (1 - MU) * P @ R.T) < TOL
    assert relf(X.astype(np.float64) - x_in, -ETA * np.sqrt(m / n) * P @ Q.astype(np.float64).T) < TOL


def test_captured_step_at_c4_replays_like_eager_steps():
    """At 16384 x 53248, r = 1024 the first product runs in parts next to the parts of the bf16 copy of M + G, which are
    launched on a second stream of the library's own.  A caller capturing its stream into a HIP graph captures both;
    every replay must give what the eager step gives, bit for bit, with the program's own work between the replays."""
    import torch
    shape = (16384, 53248, 1024)
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
    for t in range(3):
        eager.upload_grads(eager.grads_np(t))
        graphed.G[0].copy_(eager.G[0])
        assert eager.step(MU, ETA) == (0, -1)
        graph.replay()
        torch.cuda.synchronize()
        assert B.dion_last_status(graphed.state) == (0, -1)
        for name in ("X", "M", "Q"):
            assert torch.equal(getattr(eager, name)[0], getattr(graphed, name)[0]), (t, name)
        print("replay", t, "equal", flush=True)


def test_lazy_step_at_c4_product_in_parts():
    """Lazy-Dion between refreshes at 16384 x 53248, r = 1024: W = (M + G) V is the product that runs in four parts
    beside the parts of the bf16 copy.  W against its formula in fp64 on one whole row per 256-row tile and one whole
    column per 256-column tile, segment by segment, on a second step (non-zero momentum)."""
    m, n, r = 16384, 53248, 1024
    gp = GpuProblem([(m, n, r)], True, "bf16")
    B = gp.B
    rng = np.random.default_rng(11)
    for t in range(2):
        g = gp.grads_np(t)[0]
        gp.upload_grads([g])
        x_in, m_in, v_in = gp.host()
        assert gp.lazy_step(MU, ETA, False) == (0, -1)
    g32 = gp.grad_as_f32(g, True)
    W = gp.debug(0, B.DEBUG_Z)
    zr, zc = one_per_tile(rng, m, 256), one_per_tile(rng, r, 256)
    e = seg_relf(W[zr, :], orc.rows_Z(m_in, g32, v_in, zr), 256, 1)
    assert e.max() <= 2e-2, e.max()
    e = seg_relf(W[:, zc], orc.cols_Z(m_in, g32, v_in, zc), 256, 0)
    assert e.max() <= 2e-2, e.max()
    X, M, V = gp.host()
    assert np.array_equal(V, v_in)                       # no refresh: V is untouched
    assert np.isfinite(X).all() and np.isfinite(M).all()
