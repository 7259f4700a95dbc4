"""FAVOR# oracle: a plain, slow, fp64 CPU implementation written from the paper.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke
check and the benchmark's `cpu_baseline` leg may import it.  It shares no code
with the HIP path (no kernels, headers, helpers, tables or pre/post-processing)
and never calls into it.  Everything is numpy float64; numpy's `eigh`, `svd`
and `matmul` are used as library primitives, nothing is blocked, fused or
reordered beyond what the cited passage states.

Notation follows the paper: `x^(i)`, `y^(j)` are the (already scaled) query /
key vectors, `omega^(m)` the random projections (rows of `Omega`), `M` their
number, `P`, `S` the query-/key-side feature matrices, `K_hat = P S^T`.

Pins (tests/test_oracle_*.py, all CPU): PosRF and GERF as special cases of the
DERF formula; Monte-Carlo mean of f1*f2 against exp(x.y) with a z-test from
the closed-form variance; empirical variance against the closed-form one;
hand values of the scalar minimiser; closed-form objective values against a
brute-force evaluation; optimality against feasible perturbations and against
a derivative-free optimiser in d=2; attention against brute-force softmax as
M grows.  No function here is "parity unpinned".
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

__all__ = [
    "Theta", "a_star", "statistics", "fit_posrf", "fit_gerf", "fit_saderf",
    "fit_aderf", "fit_sderf", "fit", "validity_residuals", "second_moment_log",
    "variance", "lbar_bruteforce", "log_features", "features", "kernel_matvec",
    "attention", "attention_khat_definition", "exact_kernel", "exact_kernel_matvec",
    "exact_attention",
]


# --------------------------------------------------------------------------
# parameters
# --------------------------------------------------------------------------
@dataclass
class Theta:
    """DERF parameters theta = {A, B1, B2, C1, C2, D} (Section 4, DERF definition).

    `A` holds the diagonal of the matrix A (Section 4 shows a diagonal A loses
    nothing).  `lbar` is the closed-form value of the shifted log-variance
    objective at this theta when the fit provides one, else None.
    """
    A: np.ndarray          # (d,)   diagonal of A
    B1: np.ndarray         # (d, d)
    B2: np.ndarray         # (d, d)
    C1: np.ndarray         # (d, d)
    C2: np.ndarray         # (d, d)
    logD: float            # log D
    lbar: float | None = None
    name: str = "derf"

    @property
    def d(self) -> int:
        return int(self.A.shape[0])

    @property
    def D(self) -> float:
        return float(np.exp(self.logD))


def a_star(phi):
    """Minimiser of log(1-4A) - 0.5 log(1-8A) + phi/(1-8A) on A < 1/8
    (appendix lemma on the scalar minimiser, its closed form)."""
    phi = np.asarray(phi, dtype=np.float64)
    return (1.0 - 2.0 * phi - np.sqrt((2.0 * phi + 1.0) ** 2 + 8.0 * phi)) / 16.0


def statistics(X: np.ndarray, Y: np.ndarray):
    """Data statistics used by the closed-form fits (Theorems on ADERF, SDERF):
    M1 = mean x x^T, M2 = mean y y^T, mu4 = mean x, mu5 = mean y."""
    X = np.asarray(X, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    M1 = X.T @ X / X.shape[0]
    M2 = Y.T @ Y / Y.shape[0]
    mu4 = X.mean(axis=0)
    mu5 = Y.mean(axis=0)
    return M1, M2, mu4, mu5


def _gerf_theta(A: float, d: int, name: str) -> Theta:
    # GERF conditions (Section 2.3): B = sqrt(1-4A), C = -1/2, D = (1-4A)^(d/4),
    # written as the DERF with A*I, B*I, C*I (Section 4).
    B = np.sqrt(1.0 - 4.0 * A)
    eye = np.eye(d)
    return Theta(A=np.full(d, A), B1=B * eye, B2=B * eye, C1=-0.5 * eye, C2=-0.5 * eye,
                 logD=0.25 * d * np.log(1.0 - 4.0 * A), name=name)


def fit_posrf(d: int) -> Theta:
    """PosRF, exp(omega.x - |x|^2/2) (Section 2.3): the GERF with A = 0."""
    return _gerf_theta(0.0, d, "posrf")


def _gerf_lbar(A: float, d: int, mean_sq_sum: float, mean_sq_x: float, mean_sq_y: float) -> float:
    # GERF instance of the shifted log-variance objective (Section 3.1).
    return (d * np.log((1.0 - 4.0 * A) / np.sqrt(1.0 - 8.0 * A))
            + (2.0 - 8.0 * A) / (1.0 - 8.0 * A) * mean_sq_sum - mean_sq_x - mean_sq_y)


def fit_gerf(X: np.ndarray, Y: np.ndarray) -> Theta:
    """GERF with the homogeneity heuristic (Sections 2.3, 3.1): A minimises the
    GERF objective, i.e. the scalar lemma with phi = mean|x+y|^2 / d."""
    M1, M2, mu4, mu5 = statistics(X, Y)
    d = M1.shape[0]
    mean_sq_x, mean_sq_y = np.trace(M1), np.trace(M2)
    mean_sq_sum = mean_sq_x + mean_sq_y + 2.0 * mu4 @ mu5     # L^-2 sum_ij |x_i + y_j|^2
    A = float(a_star(mean_sq_sum / d))
    th = _gerf_theta(A, d, "gerf")
    th.lbar = float(_gerf_lbar(A, d, mean_sq_sum, mean_sq_x, mean_sq_y))
    return th


def fit_saderf(X: np.ndarray, Y: np.ndarray) -> Theta:
    """Simplified ADERF (Section 4.3): f1(w,x) = f_GE(w, Psi x), f2(w,y) = f_GE(w, Psi^-1 y)
    with Psi_ll = (mean_j y_l^2 / mean_i x_l^2)^(1/4), then the GERF fit on the
    rescaled sets.  The objective of Section 4.3 is a mean over all pairs (i, j);
    setting its derivative in Psi_ll to zero gives the ratio of the two per-set
    MEANS.  The section prints the ratio of sums because it takes both sets to
    have L elements; for sets of different sizes only the means form minimises
    the pairwise-mean objective."""
    X = np.asarray(X, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    psi = ((Y ** 2).mean(axis=0) / (X ** 2).mean(axis=0)) ** 0.25
    g = fit_gerf(X * psi, Y / psi)
    B = g.B1[0, 0]
    return Theta(A=g.A, B1=B * np.diag(psi), B2=B * np.diag(1.0 / psi),
                 C1=-0.5 * np.diag(psi ** 2), C2=-0.5 * np.diag(psi ** -2.0),
                 logD=g.logD, lbar=g.lbar, name="saderf")


def fit_aderf(X: np.ndarray, Y: np.ndarray) -> Theta:
    """Asymmetric DERF, closed-form optimum (Theorem on ADERF)."""
    M1, M2, mu4, mu5 = statistics(X, Y)
    d = M1.shape[0]
    mu3 = mu4 @ mu5 / d
    lam1, Q1 = np.linalg.eigh(M1)
    lam2, Q2 = np.linalg.eigh(M2)
    if lam1.min() <= 1e-12 * lam1.max() or lam2.min() <= 1e-12 * lam2.max():
        raise np.linalg.LinAlgError("ADERF needs nonsingular M1, M2")
    Z = np.diag(np.sqrt(lam1)) @ Q1.T @ Q2 @ np.diag(np.sqrt(lam2))
    U, sig, _Vt = np.linalg.svd(Z)
    phi = 2.0 * sig.sum() / d + 2.0 * mu3
    A = float(a_star(phi))
    s = np.sqrt(1.0 - 4.0 * A)
    B1 = s * np.diag(np.sqrt(sig)) @ U.T @ np.diag(lam1 ** -0.5) @ Q1.T
    B2 = s * np.diag(sig ** -0.5) @ U.T @ np.diag(lam1 ** 0.5) @ Q1.T
    C1 = -B1.T @ B1 / (2.0 * (1.0 - 4.0 * A))
    C2 = -B2.T @ B2 / (2.0 * (1.0 - 4.0 * A))
    lbar = d * (np.log(1.0 - 4.0 * A) - 0.5 * np.log(1.0 - 8.0 * A)
                + 2.0 / (1.0 - 8.0 * A) * (sig.sum() / d + mu3) + 2.0 * mu3)
    return Theta(A=np.full(d, A), B1=B1, B2=B2, C1=C1, C2=C2,
                 logD=0.25 * d * np.log(1.0 - 4.0 * A), lbar=float(lbar), name="aderf")


def fit_sderf(X: np.ndarray, Y: np.ndarray) -> Theta:
    """Symmetric DERF, closed-form optimum (Theorem on SDERF)."""
    M1, M2, mu4, mu5 = statistics(X, Y)
    d = M1.shape[0]
    N = M1 + np.outer(mu4, mu5) + np.outer(mu5, mu4) + M2
    lam, Q3 = np.linalg.eigh(N)
    order = np.argsort(-lam)                      # non-ascending eigenvalues
    lam, Q3 = np.maximum(lam[order], 0.0), Q3[:, order]
    A = a_star(lam)
    B = np.diag(np.sqrt(1.0 - 4.0 * A)) @ Q3.T
    eye = np.eye(d)
    lbar = (np.sum(np.log(1.0 - 4.0 * A) - 0.5 * np.log(1.0 - 8.0 * A)
                   + (1.0 + 1.0 / (1.0 - 8.0 * A)) * lam) - np.trace(M1) - np.trace(M2))
    return Theta(A=A, B1=B, B2=B.copy(), C1=-0.5 * eye, C2=-0.5 * eye,
                 logD=0.25 * float(np.sum(np.log(1.0 - 4.0 * A))), lbar=float(lbar), name="sderf")


def fit(variant: str, X: np.ndarray, Y: np.ndarray) -> Theta:
    variant = variant.lower()
    if variant == "posrf":
        return fit_posrf(np.asarray(X).shape[1])
    return {"gerf": fit_gerf, "saderf": fit_saderf, "aderf": fit_aderf, "sderf": fit_sderf}[variant](X, Y)


def validity_residuals(th: Theta) -> dict:
    """Residuals of the conditions under which DERFs are RFs for exp(x.y)
    (Theorem on DERF validity): 8A < I, B1^T (I-4A)^-1 B2 = I,
    Ck = -1/2 Bk^T (I-4A)^-1 Bk, D = det(I-4A)^(1/4)."""
    d = th.d
    inv = np.diag(1.0 / (1.0 - 4.0 * th.A))
    return {
        "max_8A": float(np.max(8.0 * th.A)),
        "cross": float(np.abs(th.B1.T @ inv @ th.B2 - np.eye(d)).max()),
        "C1": float(np.abs(th.C1 + 0.5 * th.B1.T @ inv @ th.B1).max()),
        "C2": float(np.abs(th.C2 + 0.5 * th.B2.T @ inv @ th.B2).max()),
        "logD": float(abs(th.logD - 0.25 * np.sum(np.log(1.0 - 4.0 * th.A)))),
    }


# --------------------------------------------------------------------------
# closed-form variance and the objective
# --------------------------------------------------------------------------
def second_moment_log(th: Theta, X: np.ndarray, Y: np.ndarray) -> np.ndarray:
    """log E[(f1(w,x) f2(w,y))^2] for every pair (i, j): the first term of the
    DERF variance formula (Theorem on DERF validity), in the log domain."""
    X = np.atleast_2d(np.asarray(X, dtype=np.float64))
    Y = np.atleast_2d(np.asarray(Y, dtype=np.float64))
    inv8 = np.diag(1.0 / (1.0 - 8.0 * th.A))
    Gx = th.C1 + th.B1.T @ inv8 @ th.B1
    Gy = th.C2 + th.B2.T @ inv8 @ th.B2
    Gxy = th.B1.T @ inv8 @ th.B2
    qx = np.einsum("ia,ab,ib->i", X, Gx, X)
    qy = np.einsum("ja,ab,jb->j", Y, Gy, Y)
    qxy = X @ Gxy @ Y.T
    const = 4.0 * th.logD - 0.5 * np.sum(np.log(1.0 - 8.0 * th.A))
    return const + 2.0 * qx[:, None] + 2.0 * qy[None, :] + 4.0 * qxy


def variance(th: Theta, X: np.ndarray, Y: np.ndarray) -> np.ndarray:
    """Var_w f1(w,x_i) f2(w,y_j) for all pairs (DERF variance formula)."""
    X = np.atleast_2d(np.asarray(X, dtype=np.float64))
    Y = np.atleast_2d(np.asarray(Y, dtype=np.float64))
    return np.exp(second_moment_log(th, X, Y)) - np.exp(2.0 * X @ Y.T)


def lbar_bruteforce(th: Theta, X: np.ndarray, Y: np.ndarray) -> float:
    """Shifted log-variance objective (Section 3.1) by its definition: the mean
    over all pairs of log(Var_ij + K(x_i,y_j)^2)."""
    X = np.asarray(X, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    var = variance(th, X, Y)
    return float(np.mean(np.log(var + np.exp(2.0 * X @ Y.T))))


# --------------------------------------------------------------------------
# features
# --------------------------------------------------------------------------
def log_features(th: Theta, Omega: np.ndarray, X: np.ndarray, side: int, alpha: float = 0.0) -> np.ndarray:
    """E[i, m] = log( M^-1/2 exp(alpha |x_i|^2) f^(side)(omega_m, x_i) ):
    the DERF exponent w^T A w + w^T B x + x^T C x + log D (Section 4), the
    factor turning softmax-kernel RFs into RFs for K^(alpha) (Section 2.3), and
    the M^-1/2 of the feature matrices P, S (Section 2.1)."""
    Omega = np.asarray(Omega, dtype=np.float64)
    X = np.atleast_2d(np.asarray(X, dtype=np.float64))
    B, C = (th.B1, th.C1) if side == 1 else (th.B2, th.C2)
    wAw = (Omega ** 2) @ th.A                         # (M,)
    wBx = X @ (Omega @ B).T                           # (L, M):  omega_m^T B x_i
    xCx = np.einsum("ia,ab,ib->i", X, C, X)           # (L,)
    sq = np.sum(X * X, axis=1)
    return (wBx + wAw[None, :] + (xCx + alpha * sq)[:, None]
            + th.logD - 0.5 * np.log(Omega.shape[0]))


def features(th: Theta, Omega: np.ndarray, X: np.ndarray, side: int, alpha: float = 0.0) -> np.ndarray:
    """Rows of P (side 1) or S (side 2) of Section 2.1, including M^-1/2."""
    return np.exp(log_features(th, Omega, X, side, alpha))


# --------------------------------------------------------------------------
# the operator and attention
# --------------------------------------------------------------------------
def kernel_matvec(th: Theta, Omega, X, Y, C, alpha: float = 0.0) -> np.ndarray:
    """Unbiased estimate K_hat C = P (S^T C) of K^(alpha)(X, Y) C, in the
    O(L M n) order of Section 2.1."""
    E1 = log_features(th, Omega, X, 1, alpha)
    E2 = log_features(th, Omega, Y, 2, alpha)
    s = E1.max(axis=1, keepdims=True)                 # inert shifts, multiplied back below
    t = E2.max()
    T = np.exp(E2 - t).T @ np.asarray(C, dtype=np.float64)
    return (np.exp(E1 - s) @ T) * np.exp(s + t)


def attention(th: Theta, Omega, Q, K, V, qk_scale: float, causal: bool = False) -> np.ndarray:
    """Self-attention with K_hat = P S^T in place of the softmax kernel matrix
    (Section 2.2, the attention equation), x = qk_scale*Q_i, y = qk_scale*K_j.

    Non-causal: P (S^T [V 1]) then the row-wise division (Section 2.1 order).
    Causal (sum restricted to j <= i, diagonal included): the same with a
    running prefix state T_i = T_{i-1} + S_i [V_i 1]^T, one row at a time.
    Shifts of the exponents (one per query row, one global for keys) cancel in
    the ratio; they only keep exp() in range.
    """
    X = qk_scale * np.asarray(Q, dtype=np.float64)
    Y = qk_scale * np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    E1 = log_features(th, Omega, X, 1)
    E2 = log_features(th, Omega, Y, 2)
    P = np.exp(E1 - E1.max(axis=1, keepdims=True))
    S = np.exp(E2 - E2.max())
    V1 = np.concatenate([V, np.ones((V.shape[0], 1))], axis=1)
    if not causal:
        T = S.T @ V1
        R = P @ T
        return R[:, :-1] / R[:, -1:]
    if X.shape[0] != Y.shape[0]:
        raise ValueError("causal attention needs as many queries as keys")
    out = np.empty((X.shape[0], V.shape[1]))
    T = np.zeros((S.shape[1], V1.shape[1]))
    for i in range(X.shape[0]):
        T += np.outer(S[i], V1[i])
        r = P[i] @ T
        out[i] = r[:-1] / r[-1]
    return out


def attention_khat_definition(th: Theta, Omega, Q, K, V, qk_scale: float, causal: bool = False,
                              rows=None) -> np.ndarray:
    """The same quantity straight from its definition: form the requested rows
    of K_hat = P S^T, zero the entries with j > i when causal, then
    diag(K_hat 1)^-1 K_hat V (Section 2.2).  O(L^2): for small inputs and for
    sampled rows of large ones."""
    X = qk_scale * np.asarray(Q, dtype=np.float64)
    Y = qk_scale * np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    rows = np.arange(X.shape[0]) if rows is None else np.asarray(rows)
    E1 = log_features(th, Omega, X[rows], 1)
    E2 = log_features(th, Omega, Y, 2)
    P = np.exp(E1 - E1.max(axis=1, keepdims=True))
    S = np.exp(E2 - E2.max())
    Khat = P @ S.T
    if causal:
        Khat = np.where(np.arange(Y.shape[0])[None, :] <= rows[:, None], Khat, 0.0)
    return (Khat @ V) / Khat.sum(axis=1, keepdims=True)


def attention_backward(th: Theta, Omega, Q, K, V, dY, qk_scale: float, causal: bool = False):
    """Gradients of the scalar  sum(Y * dY)  with respect to Q, K and V, where Y is `attention(...)` above
    (Section 2.2 with K_hat = P S^T) and theta, omega are held fixed (the paper fits theta from the data's statistics
    and then treats it as a set of constants of the feature map, Sections 3.1 and 4.3).

    Chain rule written out on the same quantities as the forward pass.  With V1 = [V 1], Yhat = P T (numerators and
    denominator) and T = S^T V1 (causal: T_i = sum_{j<=i} S_j V1_j^T):
      G1_i  = [dY_i / den_i, -(dY_i . Y_i) / den_i]                      (gradient of the row of Yhat)
      dP_im = G1_i . T_(i),m        dE1 = P * dP                          (P = exp(E1))
      R_j   = sum_{i (>= j when causal)} P_i^T G1_i                       (gradient of S_j V1_j^T)
      dV1_j = S_j R_j               dS_jm = V1_j . R_(j),m    dE2 = S * dS
      E1_im = omega_m^T B1 x_i + x_i^T C1 x_i + const_m   =>   dx_i = dE1_i (Omega B1) + sum_m dE1_im (C1 + C1^T) x_i
    and the same on the key side; x = qk_scale Q, so dQ = qk_scale dx.  Returns (dQ, dK, dV), float64."""
    Omega = np.asarray(Omega, dtype=np.float64)
    X = qk_scale * np.asarray(Q, dtype=np.float64)
    Y = qk_scale * np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    G = np.asarray(dY, dtype=np.float64)
    E1 = log_features(th, Omega, X, 1)
    E2 = log_features(th, Omega, Y, 2)
    P = np.exp(E1 - E1.max(axis=1, keepdims=True))    # inert shifts: they cancel in Y and hence in its gradient
    S = np.exp(E2 - E2.max())
    V1 = np.concatenate([V, np.ones((V.shape[0], 1))], axis=1)
    Lq, Lk = X.shape[0], Y.shape[0]
    if not causal:
        T = S.T @ V1
        R = P @ T
        den = R[:, -1]
        out = R[:, :-1] / den[:, None]
        G1 = np.concatenate([G / den[:, None], -(np.sum(G * out, axis=1) / den)[:, None]], axis=1)
        dP = G1 @ T.T
        Rk = P.T @ G1                                  # one R for every key
        dV1 = S @ Rk
        dS = V1 @ Rk.T
    else:
        if Lq != Lk:
            raise ValueError("causal attention needs as many queries as keys")
        Mf, n1 = S.shape[1], V1.shape[1]
        dP = np.empty_like(P)
        G1 = np.empty((Lq, n1))
        T = np.zeros((Mf, n1))
        for i in range(Lq):                            # forward sweep: prefix states
            T += np.outer(S[i], V1[i])
            r = P[i] @ T
            yi = r[:-1] / r[-1]
            G1[i] = np.concatenate([G[i] / r[-1], [-(G[i] @ yi) / r[-1]]])
            dP[i] = T @ G1[i]
        dV1 = np.empty_like(V1)
        dS = np.empty_like(S)
        Rk = np.zeros((Mf, n1))
        for j in range(Lk - 1, -1, -1):                # backward sweep: suffix sums
            Rk += np.outer(P[j], G1[j])
            dV1[j] = S[j] @ Rk
            dS[j] = Rk @ V1[j]
    dE1 = P * dP
    dE2 = S * dS
    dX = dE1 @ (Omega @ th.B1) + dE1.sum(axis=1, keepdims=True) * (X @ (th.C1 + th.C1.T))
    dYk = dE2 @ (Omega @ th.B2) + dE2.sum(axis=1, keepdims=True) * (Y @ (th.C2 + th.C2.T))
    return qk_scale * dX, qk_scale * dYk, dV1[:, :-1]


# --------------------------------------------------------------------------
# exact references (never compared with the GPU; they validate the above)
# --------------------------------------------------------------------------
def exact_kernel(X, Y, alpha: float = 0.0) -> np.ndarray:
    """K^(alpha)(x, y) = exp(alpha|x|^2 + x.y + alpha|y|^2) (Section 2.1)."""
    X = np.atleast_2d(np.asarray(X, dtype=np.float64))
    Y = np.atleast_2d(np.asarray(Y, dtype=np.float64))
    return np.exp(alpha * np.sum(X * X, 1)[:, None] + X @ Y.T + alpha * np.sum(Y * Y, 1)[None, :])


def exact_kernel_matvec(X, Y, C, alpha: float = 0.0) -> np.ndarray:
    return exact_kernel(X, Y, alpha) @ np.asarray(C, dtype=np.float64)


def exact_attention(Q, K, V, qk_scale: float, causal: bool = False) -> np.ndarray:
    """softmax over j of x_i.y_j (masked to j <= i when causal), times V."""
    X = qk_scale * np.asarray(Q, dtype=np.float64)
    Y = qk_scale * np.asarray(K, dtype=np.float64)
    Z = X @ Y.T
    if causal:
        Z = np.where(np.arange(Y.shape[0])[None, :] <= np.arange(X.shape[0])[:, None], Z, -np.inf)
    W = np.exp(Z - Z.max(axis=1, keepdims=True))
    return (W @ np.asarray(V, dtype=np.float64)) / W.sum(axis=1, keepdims=True)


def orthogonal_omega(gauss_dir, gauss_len):
    """Block-orthogonal random features: the appendix on the classification experiments uses orthogonal omegas and
    refers to the literature for the construction; this is the textbook one.  Rows are taken in blocks of d; the rows
    of `gauss_dir` in a block are orthonormalised in order (Gram-Schmidt = the QR factorisation of the transposed
    block with a positive diagonal of R), and row i is given the length |gauss_len[i]| (a chi_d variable), so that
    every omega_i is marginally N(0, I_d).  Shapes [M, d] -> [M, d], float64."""
    G = np.asarray(gauss_dir, dtype=np.float64)
    N = np.asarray(gauss_len, dtype=np.float64)
    M, d = G.shape
    out = np.empty_like(G)
    for r0 in range(0, M, d):
        blk = G[r0:r0 + d]
        Qm, R = np.linalg.qr(blk.T)                 # blk^T = Q R: column i of Q spans rows 0..i of blk
        sgn = np.sign(np.diag(R))
        sgn[sgn == 0] = 1.0
        dirs = (Qm * sgn).T[: blk.shape[0]]         # Gram-Schmidt directions (positive diagonal of R)
        out[r0:r0 + d] = np.linalg.norm(N[r0:r0 + d], axis=1)[:, None] * dirs
    return out

