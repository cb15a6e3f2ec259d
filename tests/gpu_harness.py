"""Shared plumbing of the GPU parity tests: builds seeded problems, runs them through the C-ABI
binding, runs the same inputs through the CPU oracle, and measures the agreed error metrics."""
import numpy as np

from oracle import dion_oracle as orc
from paper_2504_05295_amd import inputs


def relf(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


class GpuProblem:
    """One batch of matrices living on the GPU, stepped through the library."""

    def __init__(self, shapes, g_bf16, math, seed=0, q_raw=None, x0=None, q_is_filled=True, init_seed=0, forms=None):
        import torch
        from paper_2504_05295_amd import binding as B
        self.B = B
        self.torch = torch
        self.shapes = list(shapes)
        self.g_bf16 = g_bf16
        self.seed = seed
        dev = "cuda"
        self.x0 = x0 if x0 is not None else [inputs.weight(m, n, seed + 1, i) for i, (m, n, r) in enumerate(shapes)]
        self.forms = forms
        tr = [forms is not None and forms[i] == B.DION_FORM_TRANSPOSED for i in range(len(shapes))]
        self.q_raw = q_raw if q_raw is not None else [inputs.right_factor_raw(m if tr[i] else n, r, seed + 2, i)
                                                        for i, (m, n, r) in enumerate(shapes)]
        self.X = [torch.from_numpy(x.copy()).to(dev) for x in self.x0]
        self.M = [torch.full((m, n), 7.0, dtype=torch.float32, device=dev) for (m, n, r) in shapes]  # init must zero it
        self.Q = [torch.from_numpy(q.copy()).to(dev) for q in self.q_raw]
        self.state = B.dion_init_state(self.shapes, B.DION_G_BF16 if g_bf16 else B.DION_G_F32,
                                       B.DION_MATH_BF16 if math == "bf16" else B.DION_MATH_F32,
                                       self.M, self.Q, q_is_filled=q_is_filled, seed=init_seed, forms=forms)
        self.G = [None] * len(shapes)

    def grads_np(self, step, kind="gaussian"):
        out = []
        for i, (m, n, r) in enumerate(self.shapes):
            if kind == "gaussian":
                g = inputs.gradient(m, n, step, self.seed, i, bf16=self.g_bf16)
            else:
                g = inputs.structured_gradient(m, n, step, k=2 * r, seed=self.seed, index=i, bf16=self.g_bf16, noise=1e-2)
            out.append(g)
        return out

    def upload_grads(self, grads):
        torch = self.torch
        for i, g in enumerate(grads):
            t = torch.from_numpy(g.view(np.int16)).view(torch.bfloat16) if self.g_bf16 else torch.from_numpy(g)
            self.G[i] = t.to("cuda")

    @staticmethod
    def grad_as_f32(g, g_bf16):
        return inputs.bf16_bits_to_f32(g) if g_bf16 else g

    def step(self, mu, eta, batched=None):
        B = self.B
        if batched is None:
            batched = len(self.shapes) > 1
        if batched:
            B.dion_step_batched(self.state, self.X, self.G, self.M, self.Q, mu, eta)
        else:
            B.dion_step(self.state, self.X[0], self.G[0], self.M[0], self.Q[0], mu, eta)
        return B.dion_last_status(self.state)

    def lazy_step(self, mu, eta, refresh, batched=None):
        B = self.B
        if batched is None:
            batched = len(self.shapes) > 1
        if batched:
            B.dion_lazy_step_batched(self.state, self.X, self.G, self.M, self.Q, mu, eta, refresh)
        else:
            B.dion_lazy_step(self.state, self.X[0], self.G[0], self.M[0], self.Q[0], mu, eta, refresh)
        return B.dion_last_status(self.state)

    def host(self, i=0):
        return (self.X[i].cpu().numpy(), self.M[i].cpu().numpy(), self.Q[i].cpu().numpy())

    def debug(self, i, which):
        return self.B.dion_debug_buffer(self.state, i, which).cpu().numpy()


def one_step_report(gp, i, x_in, m_in, q_in, g32, mu, eta, method="householder"):
    """Oracle step from the very state the GPU step started from; returns the error metrics."""
    B = gp.B
    ref = orc.dion_step(x_in, g32, m_in, q_in, mu, eta, method)
    X, M, Q = gp.host(i)
    m, n, r = gp.shapes[i]
    P = gp.debug(i, B.DEBUG_P)[:, :r].astype(np.float64)
    R = gp.debug(i, B.DEBUG_R)[:, :r].astype(np.float64)
    rep = dict(
        status=ref["status"],
        X=relf(X, ref["X"]), M=relf(M, ref["M"]),
        dX=relf(X.astype(np.float64) - x_in, ref["X"] - x_in),
        dM=relf(M.astype(np.float64) - (m_in.astype(np.float64) + g32), ref["M"] - ref["B"]),
        orth=float(np.abs(P.T @ P - np.eye(r)).max()),
        PQt=relf(P @ Q.astype(np.float64).T, ref["P"] @ ref["Q"].T),
        PRt=relf(P @ R.T, ref["P"] @ ref["R"].T),
        qdot=float(np.min(np.abs(np.sum(Q.astype(np.float64) * ref["Q"], axis=0)))),
        qnorm=float(np.abs(np.linalg.norm(Q.astype(np.float64), axis=0) - 1).max()),
    )
    return rep, ref
