"""CPU oracle of the Dion optimizer step.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy written from the paper's algorithm statement (Algorithm
"Unsharded Dion update rule" with its PowerIter1 sub-routine, the outer step of
Algorithm 1, the error-feedback equation of Section 3.1 and the Orthonormalize
discussion of Section 3.2 / Appendix A).  It shares no code with the HIP library and
must never be imported by the product path: only tests, the smoke check and the
benchmark's cpu_baseline leg may call it.

Names: the paper's current text writes V, P, U, W, beta; this file uses the names of
the paper's future-work paragraph and of the library's interface:
    Q = V (right factor, n x r)     Z = P (power-iteration product, m x r)
    P = U (orthonormal left factor) R = W (right factor before ColNorm)
    mu = 1 - beta                   B = M + G (buffer after accumulation)

lazy_dion_step / sym_power_iter1 follow the Lazy-Dion update rule of Section 5.1 (the
paper's V, W, U keep their names there, since Q/R/P would clash with their roles above).

Every function is pinned by tests that do not use the function itself (closed forms,
a brute-force Jacobi SVD, LAPACK's QR, hand-computed tiny cases); nothing here is
"parity unpinned".  Two conventions are ours because the paper is silent: the ColNorm
guard COLNORM_EPS and the rank-deficiency threshold BREAKDOWN_TOL.
"""
from __future__ import annotations

import numpy as np

COLNORM_EPS = 1e-8      # ColNorm divides by (||R_j|| + eps): a zero column stays zero
BREAKDOWN_TOL = 1e-12   # |T_jj| <= tol * max|T_kk|  => Z is numerically rank deficient

STATUS_OK = 0
STATUS_BREAKDOWN = 1


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def accumulate(M, G):
    """B = M + G (first line of the unsharded update rule)."""
    return _f64(M) + _f64(G)


def householder_qr(Z):
    """Thin QR of Z (m x r, m >= r) by Householder reflections, unblocked, fp64.

    Returns (P, T): P is m x r with orthonormal columns, T is r x r upper triangular with
    a non-negative diagonal and Z = P T.  For full-column-rank Z this factorisation is
    unique, which is what makes "Orthonormalize" (Section 3.2: a QR decomposition or one of
    its faster variants) a well-defined function up to the column signs fixed here.
    """
    A = _f64(Z).copy()
    m, r = A.shape
    if m < r:
        raise ValueError("householder_qr needs m >= r")
    V = []
    for k in range(r):
        x = A[k:, k]
        normx = np.sqrt(np.dot(x, x))
        v = x.copy()
        if normx == 0.0:
            # nothing to annihilate; identity reflector (v = 0)
            V.append(np.zeros_like(v))
            continue
        alpha = -normx if x[0] >= 0.0 else normx
        v[0] -= alpha
        v /= np.sqrt(np.dot(v, v))
        V.append(v)
        # apply H = I - 2 v v^T to the trailing block
        A[k:, k:] -= 2.0 * np.outer(v, v @ A[k:, k:])
    T = np.triu(A[:r, :r])
    # P = H_0 H_1 ... H_{r-1} applied to the first r columns of the identity
    P = np.zeros((m, r))
    P[np.arange(r), np.arange(r)] = 1.0
    for k in range(r - 1, -1, -1):
        v = V[k]
        P[k:, :] -= 2.0 * np.outer(v, v @ P[k:, :])
    # make diag(T) >= 0:  Z = (P S)(S T) for any sign matrix S
    sgn = np.where(np.diag(T) < 0.0, -1.0, 1.0)
    P *= sgn[None, :]
    T *= sgn[:, None]
    return P, T


def lapack_qr(Z):
    """The same thin-QR factor through the library routine (for sizes where the
    unblocked loop above would take minutes).  Same sign convention."""
    P, T = np.linalg.qr(_f64(Z), mode="reduced")
    sgn = np.where(np.diag(T) < 0.0, -1.0, 1.0)
    return P * sgn[None, :], T * sgn[:, None]


def orthonormalize(Z, method="householder"):
    """P = Orthonormalize(Z): the Q-factor of the thin QR of Z (PowerIter1, Section 3.2).

    Returns (P, T, status).  status is STATUS_BREAKDOWN when Z is numerically rank
    deficient (Appendix A: the fast orthonormalisation reports failure instead of
    returning garbage); P is then not meaningful.
    """
    if method == "householder":
        P, T = householder_qr(Z)
    elif method == "lapack":
        P, T = lapack_qr(Z)
    else:
        raise ValueError(method)
    d = np.abs(np.diag(T))
    status = STATUS_OK
    if not np.all(np.isfinite(d)) or d.max() == 0.0 or d.min() <= BREAKDOWN_TOL * d.max():
        status = STATUS_BREAKDOWN
    return P, T, status


RANK_TOL = 1e-3         # a column whose squared distance to the span of the columns before it is at most
                        # RANK_TOL times its own squared norm counts as linearly dependent on them


def orthonormalize_dependent(Z, method="householder", tol=RANK_TOL, forced=None):
    """Orthonormalize for a Z whose columns may be linearly dependent (the second stage of Double Dion, whose
    buffer is a sum of a few low-rank sketches at first).

    A QR factorisation of such a Z has zero diagonal entries in T, and the matching columns of its orthogonal factor
    are an arbitrary completion of the basis: they are orthogonal to range(Z), meet only zero columns of
    W = B^T P whenever range(Z) = range(B), and so never reach the update.  The reading taken here makes that
    exact and unique: the columns are taken in order; column j is *dependent* when the distance from z_j to the
    span of the independent columns before it is at most sqrt(tol) ||z_j|| (i.e. |T_jj|^2 <= tol ||z_j||^2 in the
    Householder factorisation of the independent columns so far followed by z_j).  Dependent columns get a zero
    column of P and do not join the basis; the independent ones get the thin-QR factor (positive diagonal) of the
    sub-matrix they form.  Returns (P, keep, ratio): P is m x r, keep[j] is False for dependent columns, ratio[j] is
    the squared relative distance the decision was taken on.  With all columns independent this is orthonormalize().
    `forced` (length r, entries -1 / 0 / 1): 0 and 1 override the decision for that column (drop / keep); a test uses
    it to take borderline decisions the way the implementation under test took them in its own precision."""
    Z = _f64(Z)
    m, r = Z.shape
    P = np.zeros((m, r))
    keep = np.zeros(r, dtype=bool)
    ratio = np.zeros(r)
    norms2 = np.sum(Z * Z, axis=0)
    if forced is None:
        forced = -np.ones(r, dtype=int)
    if method == "householder":
        V = []                                  # reflectors of the independent columns so far
        cols = []
        for j in range(r):
            y = Z[:, j].copy()
            for k, v in enumerate(V):           # apply H_{k-1} ... H_0
                y[k:] -= 2.0 * v * np.dot(v, y[k:])
            k = len(V)
            if k >= m:
                continue
            x = y[k:]
            dist2 = np.dot(x, x)
            ratio[j] = dist2 / norms2[j] if norms2[j] > 0.0 else 0.0
            if forced[j] == 0 or (forced[j] < 0 and not (dist2 > tol * norms2[j])) or dist2 == 0.0:
                continue                         # dependent (also: a zero column)
            normx = np.sqrt(dist2)
            v = x.copy()
            v[0] -= -normx if x[0] >= 0.0 else normx
            v /= np.sqrt(np.dot(v, v))
            V.append(v)
            cols.append(j)
            keep[j] = True
        if cols:
            Ps, _ = householder_qr(Z[:, cols])
            P[:, cols] = Ps
    elif method == "lapack":
        # The same decisions, column by column, with the distances taken from an orthonormal basis of the independent
        # columns so far that is extended by two Gram-Schmidt sweeps per column (library matrix products); then the
        # library QR factor of the independent columns alone.
        Qb = np.zeros((m, 0))
        for j in range(r):
            z = Z[:, j]
            res = z - Qb @ (Qb.T @ z)
            res = res - Qb @ (Qb.T @ res)
            dist2 = np.dot(res, res)
            ratio[j] = dist2 / norms2[j] if norms2[j] > 0.0 else 0.0
            if forced[j] == 0 or (forced[j] < 0 and not (dist2 > tol * norms2[j])) or dist2 == 0.0 or Qb.shape[1] >= m:
                continue
            keep[j] = True
            Qb = np.concatenate([Qb, (res / np.sqrt(dist2))[:, None]], axis=1)
        if keep.any():
            Ps, _ = lapack_qr(Z[:, keep])
            P[:, keep] = Ps
    else:
        raise ValueError(method)
    return P, keep, ratio


def power_iter1(B, Q, method="householder"):
    """One power-iteration step (PowerIter1, without the data-parallel all-reduces):
    Z = B Q;  P = Orthonormalize(Z);  R = B^T P.  Returns (P, R, Z, T, status)."""
    B = _f64(B)
    Q = _f64(Q)
    Z = B @ Q
    P, T, status = orthonormalize(Z, method)
    R = B.T @ P
    return P, R, Z, T, status


def col_norm(R):
    """ColNorm: divide every column by its Euclidean norm.  Returns (Q_new, s), s_j = ||R_j||."""
    R = _f64(R)
    s = np.sqrt(np.sum(R * R, axis=0))
    return R / (s + COLNORM_EPS)[None, :], s


def dion_step(X, G, M, Q, mu, eta, method="householder"):
    """One Dion step for one m x n matrix (unsharded update rule + X_new = X - eta * O).

    Inputs are the stored values (any float dtype; bf16 gradients are passed already
    upcast, which is exact); all arithmetic is fp64.  Returns a dict with X, M, Q (new
    state, fp64), the intermediates Z, P, R, T, s and `status`.  On STATUS_BREAKDOWN the
    state is returned unchanged.
    """
    X = _f64(X)
    m, n = X.shape
    B = accumulate(M, G)                                   # M <- M + G
    P, R, Z, T, status = power_iter1(B, Q, method)         # U, W <- PowerIter1(M, V)
    if status != STATUS_OK:
        return dict(X=X, M=_f64(M), Q=_f64(Q), Z=Z, P=P, R=R, T=T, s=None, B=B, status=status)
    beta = 1.0 - mu
    M_new = B - beta * (P @ R.T)                           # error feedback
    Q_new, s = col_norm(R)                                 # V_new <- ColNorm(W)
    O = P @ Q_new.T                                        # orthonormal update
    X_new = X - eta * np.sqrt(m / n) * O                   # scaled by sqrt(|I|/|J|)
    return dict(X=X_new, M=M_new, Q=Q_new, Z=Z, P=P, R=R, T=T, s=s, B=B, status=status)


def dion_step_transposed(X, G, M, Vt, mu, eta, method="householder"):
    """One Dion step in the transposed form (Section 4.3, "Other variants": the power iteration runs on the
    transpose of the buffer).  The state factor Vt is m x r and lives on the row side:

        B = M + G;   Z' = B^T Vt (n x r);   P' = Orthonormalize(Z');   R' = B P' (m x r)
        M_new = B - beta R' P'^T;   Vt_new = ColNorm(R');   X_new = X - eta sqrt(m/n) Vt_new P'^T

    This is the unsharded update rule applied to the n x m matrix X^T with the roles of the axes swapped;
    the scale factor stays sqrt(d_out/d_in) = sqrt(m/n) of the parameter itself (the paper says the forms are
    equivalent up to renaming and gives no separate factor).  Orthonormalisation acts on n x r.
    Returns X, M, Vt (new state), the intermediates Zt, Pt, Rt, s and `status`."""
    X = _f64(X)
    m, n = X.shape
    B = accumulate(M, G)
    Vt = _f64(Vt)
    Zt = B.T @ Vt
    Pt, T, status = orthonormalize(Zt, method)
    if status != STATUS_OK:
        return dict(X=X, M=_f64(M), Vt=Vt, Zt=Zt, Pt=Pt, Rt=None, s=None, B=B, status=status)
    Rt = B @ Pt
    beta = 1.0 - mu
    M_new = B - beta * (Rt @ Pt.T)
    Vt_new, s = col_norm(Rt)
    X_new = X - eta * np.sqrt(m / n) * (Vt_new @ Pt.T)
    return dict(X=X_new, M=M_new, Vt=Vt_new, Zt=Zt, Pt=Pt, Rt=Rt, s=s, B=B, status=status)


def double_dion_step(X, G, M1, V1, M2, V2, mu1, mu2, eta, method="householder", forced=None):
    """One Double Dion step (Section 5.2 and the Double Dion algorithm, without the sharding and the
    data-parallel synchronisation of stage 1) for one m x n matrix, beta_i = 1 - mu_i:

        stage 1 (rank r1):  B1 = M1 + G;  U1, W1 = PowerIter1(B1, V1);  M1 <- B1 - beta1 U1 W1^T;  V1 <- ColNorm(W1)
        stage 2 (rank r2):  B2 = M2 + U1 W1^T;  U2, W2 = PowerIter1(B2, V2);  M2 <- B2 - beta2 U2 W2^T;  V2 <- ColNorm(W2)
        X <- X - eta sqrt(m/n) U2 V2_new^T

    The buffer of stage 2 is a sum of rank-r1 sketches, so while it has collected fewer than r2 / r1 of them (from
    M2 = 0: the first steps) B2 V2 is rank deficient.  The algorithm has no failure branch: a QR-based Orthonormalize
    returns a basis anyway, and the step uses the rank that is there.  Stage 2 therefore orthonormalises with
    orthonormalize_dependent(): dependent columns of B2 V2 get zero columns in U2, hence in W2, contribute nothing
    to M2 and X, and their columns of V2 stay as they were (ColNorm of a zero column has nothing to normalise; keeping
    the old column is what lets the rank grow as M2 fills up).  X moves on every step, also from M2 = 0.
    Stage 1 is the standard step; a breakdown there (reported as `status`) leaves the whole state unchanged.
    Returns the new state (X, M1, V1, M2, V2), the sketch D = U1 W1^T, `keep` (which columns of stage 2 were
    independent), `ratio` (the numbers those decisions were taken on) and `status`.  `forced`: see
    orthonormalize_dependent()."""
    X = _f64(X)
    m, n = X.shape
    same = dict(X=X, M1=_f64(M1), V1=_f64(V1), M2=_f64(M2), V2=_f64(V2), D=None, keep=None, ratio=None)
    B1 = accumulate(M1, G)
    U1, W1, _, _, status = power_iter1(B1, V1, method)
    if status != STATUS_OK:
        return dict(same, status=status)
    D = U1 @ W1.T
    M1_new = B1 - (1.0 - mu1) * D
    V1_new, _ = col_norm(W1)
    B2 = accumulate(M2, D)
    V2 = _f64(V2)
    U2, keep, ratio = orthonormalize_dependent(B2 @ V2, method, RANK_TOL, forced)
    W2 = B2.T @ U2
    M2_new = B2 - (1.0 - mu2) * (U2 @ W2.T)
    V2_new, _ = col_norm(W2)
    V2_new[:, ~keep] = V2[:, ~keep]
    X_new = X - eta * np.sqrt(m / n) * (U2[:, keep] @ V2_new[:, keep].T)
    return dict(X=X_new, M1=M1_new, V1=V1_new, M2=M2_new, V2=V2_new, D=D, keep=keep, ratio=ratio, status=STATUS_OK)


def sym_power_iter1(B, V, method="householder"):
    """SymPowerIter1 of the faster-variants algorithm (Section 5.1): V <- Orthonormalize(B^T (B V)).
    One step of orthogonal iteration on B^T B.  Returns (V_new, Y, T, status), Y = B^T B V."""
    B = _f64(B)
    V = _f64(V)
    Y = B.T @ (B @ V)
    V_new, T, status = orthonormalize(Y, method)
    return V_new, Y, T, status


def lazy_dion_step(X, G, M, V, mu, eta, refresh, method="householder"):
    """One Lazy-Dion step (Section 5.1, unsharded Lazy-Dion update rule) for one m x n matrix.

    B = M + G;  if refresh: V <- SymPowerIter1(B, V);  W = B V;  M_new = B - beta W V^T;
    U = ColNorm(W);  X_new = X - eta sqrt(m/n) U V^T.   `refresh` is the caller's
    "t mod k = 0".  Returns X, M, V (new state), the intermediates W, U, s and `status`
    (STATUS_BREAKDOWN from the refresh leaves the state unchanged).
    """
    X = _f64(X)
    m, n = X.shape
    B = accumulate(M, G)
    V = _f64(V)
    status = STATUS_OK
    if refresh:
        V_new, _, _, status = sym_power_iter1(B, V, method)
        if status != STATUS_OK:
            return dict(X=X, M=_f64(M), V=V, W=None, U=None, s=None, B=B, status=status)
        V = V_new
    beta = 1.0 - mu
    W = B @ V
    M_new = B - beta * (W @ V.T)
    U, s = col_norm(W)
    X_new = X - eta * np.sqrt(m / n) * (U @ V.T)
    return dict(X=X_new, M=M_new, V=V, W=W, U=U, s=s, B=B, status=status)


def run_lazy_steps(X, grads, M, V, mu, eta, k, method="householder", store=np.float32, first_t=0):
    """Lazy-Dion over len(grads) steps with a refresh whenever t mod k = 0 (t counts from first_t, so the
    default refreshes at the very first step, which also makes the initial V orthonormal).  State rounded
    to the storage dtype after each step."""
    out = []
    X = np.asarray(X, dtype=store)
    M = np.asarray(M, dtype=store)
    V = np.asarray(V, dtype=store)
    for i, G in enumerate(grads):
        res = lazy_dion_step(X, G, M, V, mu, eta, (first_t + i) % k == 0, method)
        X = res["X"].astype(store)
        M = res["M"].astype(store)
        V = res["V"].astype(store)
        res = dict(res, X=X, M=M, V=V)
        out.append(res)
    return out


def init_state(m, n, Q_raw):
    """Initial optimizer state: M = 0 and Q = ColNorm(Q_raw) with Q_raw i.i.d. N(0,1).
    (The paper gives the state as (M, V) without an initialiser; this is the
    benchmark configurations' choice.)"""
    Q, _ = col_norm(Q_raw)
    return np.zeros((m, n)), Q


def run_steps(X, grads, M, Q, mu, eta, method="householder", store=np.float32):
    """Run len(grads) steps, rounding the state to the storage dtype (fp32) after each step,
    as the library's caller-owned fp32 buffers do.  Returns the list of per-step dicts
    (state entries already rounded)."""
    out = []
    X = np.asarray(X, dtype=store)
    M = np.asarray(M, dtype=store)
    Q = np.asarray(Q, dtype=store)
    for G in grads:
        res = dion_step(X, G, M, Q, mu, eta, method)
        X = res["X"].astype(store)
        M = res["M"].astype(store)
        Q = res["Q"].astype(store)
        res = dict(res, X=X, M=M, Q=Q)
        out.append(res)
    return out


# ---- per-entry forms, for sampled checks at sizes where a full fp64 step is too slow ----

def entry_Z(M, G, Q, rows, cols):
    """Z[i, a] = sum_j (M[i,j] + G[i,j]) Q[j,a] for the listed (i, a) pairs."""
    Qd = _f64(Q)
    out = np.empty(len(rows))
    for t, (i, a) in enumerate(zip(rows, cols)):
        out[t] = np.dot(_f64(M[i, :]) + _f64(G[i, :]), Qd[:, a])
    return out


def entry_R(M, G, P, rows, cols):
    """R[j, a] = sum_i (M[i,j] + G[i,j]) P[i,a] for the listed (j, a) pairs."""
    out = np.empty(len(rows))
    for t, (j, a) in enumerate(zip(rows, cols)):
        out[t] = np.dot(_f64(M[:, j]) + _f64(G[:, j]), _f64(P[:, a]))
    return out


def entry_update(X, G, M, P, R, mu, eta, rows, cols):
    """(X_new[i,j], M_new[i,j]) for listed (i, j) pairs, given the factors P and R:
    M_new = B - (1-mu) P R^T;  X_new = X - eta sqrt(m/n) P ColNorm(R)^T."""
    m, n = X.shape
    R = _f64(R)
    s = np.sqrt(np.sum(R * R, axis=0))
    d = 1.0 / (s + COLNORM_EPS)
    xs = np.empty(len(rows))
    ms = np.empty(len(rows))
    c = eta * np.sqrt(m / n)
    for t, (i, j) in enumerate(zip(rows, cols)):
        p = _f64(P[i, :])
        rj = R[j, :]
        ms[t] = (float(M[i, j]) + float(G[i, j])) - (1.0 - mu) * np.dot(p, rj)
        xs[t] = float(X[i, j]) - c * np.dot(p, rj * d)
    return xs, ms


# ---- block forms: whole rows / columns of one stage's output from that stage's inputs, for checks at sizes
# ---- where a full fp64 step is too slow.  Each is the defining formula restricted to the listed rows or columns.

def rows_Z(M, G, Q, rows):
    """Z[rows, :] = (M + G)[rows, :] Q   (PowerIter1, first product)."""
    rows = np.asarray(rows)
    return (_f64(M[rows, :]) + _f64(G[rows, :])) @ _f64(Q)


def cols_Z(M, G, Q, cols, chunk=2048):
    """Z[:, cols] = (M + G) Q[:, cols], accumulated over blocks of `chunk` rows of M + G (memory only)."""
    cols = np.asarray(cols)
    Qc = _f64(Q[:, cols])
    m = M.shape[0]
    out = np.empty((m, len(cols)))
    for i0 in range(0, m, chunk):
        out[i0:i0 + chunk, :] = (_f64(M[i0:i0 + chunk, :]) + _f64(G[i0:i0 + chunk, :])) @ Qc
    return out


def rows_R(M, G, P, rows):
    """R[rows, :] = ((M + G)[:, rows])^T P   (PowerIter1, second product; `rows` index the n side)."""
    rows = np.asarray(rows)
    return (_f64(M[:, rows]) + _f64(G[:, rows])).T @ _f64(P)


def cols_R(M, G, P, cols, chunk=2048):
    """R[:, cols] = (M + G)^T P[:, cols], accumulated over blocks of `chunk` rows of M + G."""
    cols = np.asarray(cols)
    m, n = M.shape
    out = np.zeros((n, len(cols)))
    for i0 in range(0, m, chunk):
        out += (_f64(M[i0:i0 + chunk, :]) + _f64(G[i0:i0 + chunk, :])).T @ _f64(P[i0:i0 + chunk, :][:, cols])
    return out


def rows_update(X, G, M, P, R, mu, eta, rows):
    """(X_new[rows, :], M_new[rows, :]) given the factors P and R:
    M_new = B - (1-mu) P R^T;  X_new = X - eta sqrt(m/n) P ColNorm(R)^T."""
    rows = np.asarray(rows)
    m, n = X.shape
    Qn, _ = col_norm(R)
    Pr = _f64(P[rows, :])
    Mn = (_f64(M[rows, :]) + _f64(G[rows, :])) - (1.0 - mu) * (Pr @ _f64(R).T)
    Xn = _f64(X[rows, :]) - eta * np.sqrt(m / n) * (Pr @ Qn.T)
    return Xn, Mn


def cols_update(X, G, M, P, R, mu, eta, cols):
    """(X_new[:, cols], M_new[:, cols]) given the factors P and R (ColNorm needs all of R's rows)."""
    cols = np.asarray(cols)
    m, n = X.shape
    Qn, _ = col_norm(R)
    Pd = _f64(P)
    Mn = (_f64(M[:, cols]) + _f64(G[:, cols])) - (1.0 - mu) * (Pd @ _f64(R[cols, :]).T)
    Xn = _f64(X[:, cols]) - eta * np.sqrt(m / n) * (Pd @ Qn[cols, :].T)
    return Xn, Mn


# ---- counter-based Gaussian fill used by the library's init call when it draws Q itself ----

_PHILOX_M0 = 0xD2511F53
_PHILOX_M1 = 0xCD9E8D57
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85


def philox4x32_10(counter, key):
    """Philox-4x32 with 10 rounds (Salmon et al., "Parallel random numbers: as easy as
    1, 2, 3", SC'11).  counter: (..., 4) uint32, key: (2,) uint32.  Returns (..., 4) uint32."""
    c = np.array(counter, dtype=np.uint64)
    k0 = np.uint64(key[0])
    k1 = np.uint64(key[1])
    mask = np.uint64(0xFFFFFFFF)
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    for _ in range(10):
        p0 = np.uint64(_PHILOX_M0) * c0
        p1 = np.uint64(_PHILOX_M1) * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & mask
        hi1, lo1 = p1 >> np.uint64(32), p1 & mask
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & mask, lo1, (hi0 ^ c3 ^ k1) & mask, lo0
        k0 = (k0 + np.uint64(_PHILOX_W0)) & mask
        k1 = (k1 + np.uint64(_PHILOX_W1)) & mask
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def gaussian_fill(count, seed, stream):
    """count N(0,1) values, element e drawn from Philox block e//4 (counter = (e//4, 0,
    stream, 0), key = (seed low, seed high)): words (0,1) and (2,3) of a block feed two
    Box-Muller transforms, u1 = (w+1)/2^32 in (0,1], u2 = w'/2^32; elements 4b..4b+3 are
    (r1 cos, r1 sin, r2 cos, r2 sin)."""
    nblk = (count + 3) // 4
    ctr = np.zeros((nblk, 4), dtype=np.uint64)
    ctr[:, 0] = np.arange(nblk, dtype=np.uint64) & np.uint64(0xFFFFFFFF)
    ctr[:, 1] = np.arange(nblk, dtype=np.uint64) >> np.uint64(32)
    ctr[:, 2] = np.uint64(stream)
    key = (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    w = philox4x32_10(ctr, key).astype(np.float64)
    out = np.empty((nblk, 4))
    for h in range(2):
        u1 = (w[:, 2 * h] + 1.0) / 4294967296.0
        u2 = w[:, 2 * h + 1] / 4294967296.0
        rad = np.sqrt(-2.0 * np.log(u1))
        out[:, 2 * h] = rad * np.cos(2.0 * np.pi * u2)
        out[:, 2 * h + 1] = rad * np.sin(2.0 * np.pi * u2)
    return out.reshape(-1)[:count]
