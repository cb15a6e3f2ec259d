"""Brute-force one-sided Jacobi SVD (Hestenes), used only to pin the oracle.

Independent of the oracle and of LAPACK: rotates column pairs of A until all columns are
mutually orthogonal; singular values are the column norms.
"""
import numpy as np


def jacobi_svd(A, tol=1e-15, max_sweeps=60):
    U = np.array(A, dtype=np.float64)
    m, n = U.shape
    V = np.eye(n)
    for _ in range(max_sweeps):
        off = 0.0
        for p in range(n - 1):
            for q in range(p + 1, n):
                alpha = np.dot(U[:, p], U[:, p])
                beta = np.dot(U[:, q], U[:, q])
                gamma = np.dot(U[:, p], U[:, q])
                if alpha == 0.0 or beta == 0.0:
                    continue
                off = max(off, abs(gamma) / np.sqrt(alpha * beta))
                if abs(gamma) <= tol * np.sqrt(alpha * beta):
                    continue
                zeta = (beta - alpha) / (2.0 * gamma)
                t = np.sign(zeta) / (abs(zeta) + np.sqrt(1.0 + zeta * zeta)) if zeta != 0.0 else 1.0
                c = 1.0 / np.sqrt(1.0 + t * t)
                s = c * t
                up = U[:, p].copy()
                U[:, p] = c * up - s * U[:, q]
                U[:, q] = s * up + c * U[:, q]
                vp = V[:, p].copy()
                V[:, p] = c * vp - s * V[:, q]
                V[:, q] = s * vp + c * V[:, q]
        if off <= tol:
            break
    sig = np.sqrt(np.sum(U * U, axis=0))
    order = np.argsort(-sig)
    sig = sig[order]
    U = U[:, order]
    V = V[:, order]
    nz = sig > 0
    U[:, nz] /= sig[nz]
    return U, sig, V
