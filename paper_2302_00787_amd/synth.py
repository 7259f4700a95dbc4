"""Seeded synthetic inputs with the shapes and statistics of the five workloads.

This module draws numbers and nothing else: it contains none of the method's
arithmetic (no features, no fits, no attention).  Both the HIP path and the CPU
oracle read the arrays it returns, so that parity is checked on identical
inputs and identical omega.

All arrays are float32.  For the bf16 workloads the values of Q, K, V are
rounded once, here, to bf16-representable numbers (round to nearest even), so
input rounding is not part of any error budget; `to_bf16_bits` gives the 16-bit
patterns for upload.

Workloads (numbering follows the configuration list of the benchmark file):
  c1  tiny non-causal attention, fp32:  B1 H1 L256 d16 M64, Q,K,V ~ N(0,1)
  c2  Gaussian-kernel operator, fp32:   N16384 d32 M512 n8, rows U[0,1] scaled to norm 2
  c3  encoder attention, bf16:          B8 H8 L4096 d64 M256, per-head N(mu, U diag(0.5^(i/8)) U^T)
  c4  causal speech-like, bf16:         B4 H8 L16384 d64 M256, N(0,1) + per-head mean of norm 0.5 (after scaling)
  c5  long causal, bf16:                B1 H16 L65536 d128 M512, eigenvalues i^-1.5, 5% rows x3
"""
from __future__ import annotations

import numpy as np

WORKLOADS = {
    "c1": dict(kind="attention", dtype="f32", causal=False, B=1, H=1, L=256, d=16, M=64, seed=0),
    "c2": dict(kind="matvec", dtype="f32", N=16384, d=32, M=512, n=8, alpha=-0.5, seed=2000),
    "c3": dict(kind="attention", dtype="bf16", causal=False, B=8, H=8, L=4096, d=64, M=256, seed=3000),
    "c4": dict(kind="attention", dtype="bf16", causal=True, B=4, H=8, L=16384, d=64, M=256, chunk=64, seed=4000),
    "c5": dict(kind="attention", dtype="bf16", causal=True, B=1, H=16, L=65536, d=128, M=512, chunk=64, seed=5000),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 -> nearest bf16 value (ties to even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """bf16-representable float32 array -> its uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def haar_orthogonal(rng: np.random.Generator, d: int) -> np.ndarray:
    """Haar-distributed orthogonal matrix: QR of a Gaussian matrix with the
    signs of R's diagonal made positive."""
    q, r = np.linalg.qr(rng.standard_normal((d, d)))
    return q * np.sign(np.diag(r))[None, :]


def _normal(rng, shape):
    return rng.standard_normal(shape, dtype=np.float32)


def make(name: str, **override) -> dict:
    """Build workload `name` ("c1".."c5"); keyword overrides shrink it (B, H, L, N, M, d, seed)."""
    cfg = dict(WORKLOADS[name])
    cfg.update(override)
    rng = np.random.default_rng(cfg["seed"])
    d, M = cfg["d"], cfg["M"]
    out = dict(cfg)
    out["name"] = name

    if cfg["kind"] == "matvec":
        N, n = cfg["N"], cfg["n"]
        X = rng.random((N, d), dtype=np.float32)
        X *= (2.0 / np.linalg.norm(X.astype(np.float64), axis=1))[:, None].astype(np.float32)
        out.update(X=X, Y=X, C=_normal(rng, (N, n)), Omega=_normal(rng, (1, M, d)), qk_scale=1.0)
        return out

    B, H, L = cfg["B"], cfg["H"], cfg["L"]
    out["qk_scale"] = float(d) ** -0.25
    Q = np.empty((B, H, L, d), dtype=np.float32)
    K = np.empty((B, H, L, d), dtype=np.float32)
    if name in ("c1", "c4"):
        for h in range(H):
            Q[:, h] = _normal(rng, (B, L, d))
            K[:, h] = _normal(rng, (B, L, d))
            if name == "c4":
                # mean offset of norm 0.5 in the scaled space x = d^-1/4 Q, one direction per head and side
                for T in (Q, K):
                    m = rng.standard_normal(d)
                    m *= 0.5 / np.linalg.norm(m)
                    T[:, h] += (m / out["qk_scale"]).astype(np.float32)
    elif name == "c3":
        lam = 0.5 ** (np.arange(d) / 8.0)
        for h in range(H):
            U = haar_orthogonal(rng, d)
            root = (U * np.sqrt(lam)[None, :]).T.astype(np.float32)     # g @ root ~ N(0, U diag(lam) U^T)
            for T in (Q, K):
                mu = (0.1 * rng.standard_normal(d)).astype(np.float32)
                T[:, h] = _normal(rng, (B, L, d)) @ root + mu
    elif name == "c5":
        lam = np.arange(1, d + 1, dtype=np.float64) ** -1.5
        for h in range(H):
            U = haar_orthogonal(rng, d)
            root = (U * np.sqrt(lam)[None, :]).T.astype(np.float32)
            for T in (Q, K):
                g = _normal(rng, (B, L, d)) @ root
                heavy = rng.random((B, L)) < 0.05
                g[heavy] *= 3.0
                T[:, h] = g
    else:
        raise KeyError(name)
    V = _normal(rng, (B, H, L, d))
    Omega = _normal(rng, (H, M, d))
    if cfg["dtype"] == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    out.update(Q=Q, K=K, V=V, Omega=Omega)
    return out


def clusters(seed: int = 6000, classes: int = 6, d: int = 32, n_train: int = 4096, n_test: int = 1024,
             spread: float = 0.55) -> dict:
    """Labelled points for the kernel-classification demo: `classes` Gaussian clusters in d dimensions with centres
    drawn on the unit sphere, two clusters per class (so classes are not linearly separable), isotropic noise
    `spread` / sqrt(d) per coordinate.  Returns float32 points, integer labels and one-hot label rows."""
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((2 * classes, d))
    centres /= np.linalg.norm(centres, axis=1, keepdims=True)

    def draw(n):
        which = rng.integers(0, 2 * classes, n)
        pts = centres[which] + spread / np.sqrt(d) * rng.standard_normal((n, d))
        return pts.astype(np.float32), (which % classes).astype(np.int64)

    Xtr, ytr = draw(n_train)
    Xte, yte = draw(n_test)
    onehot = np.zeros((n_train, classes), dtype=np.float32)
    onehot[np.arange(n_train), ytr] = 1.0
    return dict(train=Xtr, train_labels=ytr, train_onehot=onehot, test=Xte, test_labels=yte, classes=classes, d=d)
