"""GPU parity of the Double Dion step (Section 5.2) through the C-ABI against the CPU oracle, step by step from
the GPU's own state; fp32 and bf16 operand modes, single and batched, and the two breakdown cases."""
import numpy as np
import pytest
import torch

from oracle import dion_oracle as orc
from paper_2504_05295_amd import inputs, binding as B
from gpu_harness import relf

pytestmark = pytest.mark.gpu
MU1, MU2, ETA = 0.999, 0.95, inputs.ETA          # the paper's beta1 = 0.001, beta2 = 0.05


class DoubleProblem:
    def __init__(self, shapes, r1, r2, g_bf16, math, v1_raw=None, v2_raw=None, warm=True):
        self.shapes, self.r1, self.r2, self.g_bf16 = shapes, r1, r2, g_bf16
        dev = "cuda"
        cnt = len(shapes)
        self.X = [torch.from_numpy(inputs.weight(m, n, 1, i)).to(dev) for i, (m, n) in enumerate(shapes)]
        self.M1 = [torch.empty((m, n), dtype=torch.float32, device=dev) for (m, n) in shapes]
        self.M2 = [torch.empty((m, n), dtype=torch.float32, device=dev) for (m, n) in shapes]
        self.D = [torch.empty((m, n), dtype=torch.float32, device=dev) for (m, n) in shapes]
        v1 = v1_raw or [inputs.right_factor_raw(n, r1, 2, i) for i, (m, n) in enumerate(shapes)]
        v2 = v2_raw or [inputs.right_factor_raw(n, r2, 3, i) for i, (m, n) in enumerate(shapes)]
        self.V1 = [torch.from_numpy(v.copy()).to(dev) for v in v1]
        self.V2 = [torch.from_numpy(v.copy()).to(dev) for v in v2]
        mth = B.DION_MATH_BF16 if math == "bf16" else B.DION_MATH_F32
        self.s1 = B.dion_init_state([(m, n, r1) for (m, n) in shapes], B.DION_G_BF16 if g_bf16 else B.DION_G_F32, mth,
                                    self.M1, self.V1)
        self.s2 = B.dion_init_state([(m, n, r2) for (m, n) in shapes], B.DION_G_F32, mth, self.M2, self.V2)
        if warm:
            # as after many steps: M2 has full rank (from M2 = 0 it is a sum of rank-r1 sketches, see the cold-start test)
            for i, (m, n) in enumerate(shapes):
                self.M2[i].copy_(torch.from_numpy(inputs.gaussian((m, n), 3e-2, 7, 11, 0, i)))
        self.G = [None] * cnt

    def upload(self, grads):
        for i, g in enumerate(grads):
            t = torch.from_numpy(g.view(np.int16)).view(torch.bfloat16) if self.g_bf16 else torch.from_numpy(g)
            self.G[i] = t.to("cuda")

    def step(self):
        B.dion_double_step(self.s1, self.s2, self.X, self.G, self.M1, self.V1, self.M2, self.V2, self.D, MU1, MU2, ETA)
        return B.dion_last_status(self.s1), B.dion_last_status(self.s2)

    def host(self, i):
        return [t[i].cpu().numpy() for t in (self.X, self.M1, self.V1, self.M2, self.V2)]


def run(shapes, r1, r2, g_bf16, math, steps, tol):
    dp = DoubleProblem(shapes, r1, r2, g_bf16, math)
    for t in range(steps):
        grads = [inputs.gradient(m, n, t, 0, i, bf16=g_bf16) for i, (m, n) in enumerate(shapes)]
        before = [dp.host(i) for i in range(len(shapes))]
        dp.upload(grads)
        assert dp.step() == ((0, -1), (0, -1))
        for i in range(len(shapes)):
            g32 = inputs.bf16_bits_to_f32(grads[i]) if g_bf16 else grads[i]
            x, m1, v1, m2, v2 = before[i]
            ref = orc.double_dion_step(x, g32, m1, v1, m2, v2, MU1, MU2, ETA)
            X, M1, V1, M2, V2 = dp.host(i)
            err = dict(X=relf(X, ref["X"]), M1=relf(M1, ref["M1"]), M2=relf(M2, ref["M2"]),
                       dX=relf(X.astype(np.float64) - x, ref["X"] - x), D=relf(dp.D[i].cpu().numpy(), ref["D"]),
                       v1=float(np.min(np.abs(np.sum(V1.astype(np.float64) * ref["V1"], axis=0)))),
                       v2=float(np.min(np.abs(np.sum(V2.astype(np.float64) * ref["V2"], axis=0)))))
            assert max(err["X"], err["M1"], err["M2"], err["D"]) <= tol and err["dX"] <= 3 * tol, (t, i, err)
            assert err["v1"] > 1 - 10 * tol and err["v2"] > 1 - 10 * tol, (t, i, err)


def test_double_dion_fp32():
    run([(256, 192)], 8, 32, False, "f32", 3, 1e-4)
    run([(200, 136), (200, 136), (128, 384)], 8, 24, False, "f32", 2, 1e-4)


def test_double_dion_bf16_large_tile_path():
    run([(512, 256), (256, 768)], 128, 128, True, "bf16", 2, 2e-2)


def test_double_dion_breakdowns():
    m, n, r1, r2 = 256, 192, 8, 32
    good1 = [inputs.right_factor_raw(n, r1, 2, i) for i in range(2)]
    good2 = [inputs.right_factor_raw(n, r2, 3, i) for i in range(2)]
    bad1 = good1[1].copy(); bad1[:, 5] = bad1[:, 2]
    bad2 = good2[1].copy(); bad2[:, 9] = bad2[:, 4]
    grads = [inputs.gradient(m, n, 0, 0, i, bf16=False) for i in range(2)]
    # stage 1 of matrix 1 fails: that matrix is left alone entirely, its neighbour is stepped
    dp = DoubleProblem([(m, n)] * 2, r1, r2, False, "f32", v1_raw=[good1[0], bad1])
    before = [dp.host(i) for i in range(2)]
    dp.upload(grads)
    st1, st2 = dp.step()
    assert st1 == (B.DION_NUM_BREAKDOWN, 1) and st2 == (B.DION_NUM_BREAKDOWN, 1)
    for u, v in zip(before[1], dp.host(1)):
        assert np.array_equal(u, v)
    ref = orc.double_dion_step(*before[0][:1], grads[0], *before[0][1:], MU1, MU2, ETA)
    assert relf(dp.host(0)[0], ref["X"]) < 1e-4
    # stage 2 of matrix 1 fails: stage 1 has taken its step, M2 takes in the sketch, X and V2 are untouched
    dp = DoubleProblem([(m, n)] * 2, r1, r2, False, "f32", v2_raw=[good2[0], bad2])
    before = [dp.host(i) for i in range(2)]
    dp.upload(grads)
    st1, st2 = dp.step()
    assert st1 == (0, -1) and st2 == (B.DION_NUM_BREAKDOWN, 1)
    X, M1, V1, M2, V2 = dp.host(1)
    assert np.array_equal(X, before[1][0]) and np.array_equal(V2, before[1][4])
    ref = orc.double_dion_step(before[1][0], grads[1], before[1][1], before[1][2], before[1][3], before[1][4], MU1, MU2, ETA)
    assert ref["status"] == orc.STATUS_BREAKDOWN and relf(M1, ref["M1"]) < 1e-4
    assert relf(M2, ref["M2"]) < 1e-5                                     # M2 <- M2 + sketch


def test_double_dion_cold_start():
    # from M2 = 0 the second stage cannot orthonormalise until M2 has collected r2 / r1 sketches
    m, n, r1, r2 = 256, 192, 16, 32
    dp = DoubleProblem([(m, n)], r1, r2, False, "f32", warm=False)
    statuses = []
    for t in range(4):
        g = inputs.gradient(m, n, t, 0, 0, bf16=False)
        x, m1, v1, m2, v2 = dp.host(0)
        dp.upload([g])
        st1, st2 = dp.step()
        assert st1 == (0, -1)
        ref = orc.double_dion_step(x, g, m1, v1, m2, v2, MU1, MU2, ETA)
        X, M1, V1, M2, V2 = dp.host(0)
        statuses.append((st2[0], ref["status"]))
        assert relf(M2, ref["M2"]) < 1e-4 and relf(M1, ref["M1"]) < 1e-4, t
        if st2[0] != 0:
            assert np.array_equal(X, x) and np.array_equal(V2, v2)
    assert statuses[0] == (B.DION_NUM_BREAKDOWN, orc.STATUS_BREAKDOWN)      # rank 16 < 32
    assert statuses[-1] == (0, orc.STATUS_OK)
