"""The entry point that allocates nothing (dion_step_static: the step on the library's static device array)
against dion_step on a caller-provided workspace: same inputs, two calls in a row, the second on a smaller matrix,
which finds the array full of what the first one left there."""
import numpy as np
import pytest

from paper_2504_05295_amd import inputs
from gpu_harness import GpuProblem, relf

pytestmark = pytest.mark.gpu
MU, ETA = inputs.MU, inputs.ETA


def test_static_workspace_step_matches_dion_step():
    import torch
    from paper_2504_05295_amd import binding as B
    # (shape, bf16 gradient, operand mode, tolerance of the parity tests for that mode)
    cases = [((1024, 1024, 256), True, "bf16", 2e-2), ((512, 768, 128), True, "bf16", 2e-2), ((256, 256, 64), False, "f32", 1e-4),
             ((200, 136, 24), False, "f32", 1e-4)]
    status = torch.full((1,), 77, dtype=torch.int32, device="cuda")
    for (shape, g_bf16, math, tol) in cases:
        m, n, r = shape
        assert B.dion_workspace_bytes([shape], B.DION_G_BF16 if g_bf16 else B.DION_G_F32,
                                      B.DION_MATH_BF16 if math == "bf16" else B.DION_MATH_F32) <= B.DION_STATIC_SCRATCH_BYTES
        ref = GpuProblem([shape], g_bf16, math)                    # the existing entry point, workspace from torch
        # the caller of the static entry point owns M and Q: start them as dion_init_state leaves them
        X = ref.X[0].clone()
        M = ref.M[0].clone()
        Q = ref.Q[0].clone()
        for t in range(2):                                         # second step: non-zero momentum, a used workspace
            grads = ref.grads_np(t)
            ref.upload_grads(grads)
            assert ref.step(MU, ETA) == (0, -1)
            B.dion_step_static(X, ref.G[0], M, Q, B.DION_G_BF16 if g_bf16 else B.DION_G_F32,
                               B.DION_MATH_BF16 if math == "bf16" else B.DION_MATH_F32, MU, ETA, status=status)
            torch.cuda.synchronize()
            assert int(status.item()) == 0
            ex, em, eq = relf(X.cpu().numpy(), ref.X[0].cpu().numpy()), relf(M.cpu().numpy(), ref.M[0].cpu().numpy()), \
                relf(Q.cpu().numpy(), ref.Q[0].cpu().numpy())
            same = torch.equal(X, ref.X[0]) and torch.equal(M, ref.M[0]) and torch.equal(Q, ref.Q[0])
            print(shape, "step", t, "rel err X %.1e M %.1e Q %.1e" % (ex, em, eq), "bit-identical" if same else "", flush=True)
            assert ex <= tol and em <= tol and eq <= tol
            assert same          # the same kernels in the same order on the same inputs: nothing to differ by


def test_static_workspace_rejects_what_does_not_fit():
    import torch
    from paper_2504_05295_amd import binding as B
    m, n, r = 2048, 2048, 512
    X = torch.zeros((m, n), device="cuda")
    M = torch.zeros((m, n), device="cuda")
    G = torch.zeros((m, n), device="cuda", dtype=torch.bfloat16)
    Q = torch.zeros((n, r), device="cuda")
    with pytest.raises(B.DionError) as e:
        B.dion_step_static(X, G, M, Q, B.DION_G_BF16, B.DION_MATH_BF16, MU, ETA)
    assert e.value.code == B.DION_EWORKSPACE
    with pytest.raises(B.DionError) as e:
        B.dion_step_static(X[:256, :256].contiguous(), G[:256, :256].contiguous(), M[:256, :256].contiguous(),
                           Q[:256, :64].contiguous(), B.DION_G_BF16, B.DION_MATH_BF16, 1.5, ETA)
    assert e.value.code == B.DION_EINVAL
