"""Seeded sweeps over shapes that no other test names: every case draws its path (general-shape kernels, the two bf16
paths, the operator kernels), sizes (ragged, tiny, odd), parameter family and entry point from a generator seeded by
the case number, and is held to the oracle at the tolerance of its arithmetic (R13).  The cases are cheap; their value
is in the combinations (a sweep of this kind found the operator kernels' overflow on rows far outside the unit ball).
"""
import numpy as np
import pytest

from oracle import favorsharp_oracle as orc
from paper_2302_00787_amd import synth
from tests import util

pytestmark = pytest.mark.gpu

VARIANTS = ["posrf", "gerf", "sderf", "aderf", "saderf"]


@pytest.fixture(scope="module")
def fs():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2302_00787_amd import binding
    binding.lib()
    return binding


def _theta_per_head(variant, Q, K, s):
    """One oracle-fitted float32 parameter block per head, or None where the family is not defined (singular M1 / M2)."""
    H, d = Q.shape[1], Q.shape[3]
    out = []
    for h in range(H):
        X = s * Q[:, h].reshape(-1, d).astype(np.float64)
        Y = s * K[:, h].reshape(-1, d).astype(np.float64)
        try:
            out.append(util.theta_vec_from_oracle(orc.fit(variant, X, Y)))
        except Exception:
            return None
    return np.stack(out)


def _padded(a, dtype):
    """Device copy whose last dimension is padded to the alignment the boundary asks for (4 floats / 8 bf16 numbers),
    returned as the unpadded view."""
    import torch
    q = 8 if dtype == "bf16" else 4
    n = a.shape[-1]
    t = torch.zeros(a.shape[:-1] + ((n + q - 1) // q * q,), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32,
                    device="cuda")
    t[..., :n] = util.to_device(a, dtype)
    return t[..., :n]


def _compare(Yh, theta, Om, Q, K, V, s, causal, tol):
    assert np.isfinite(Yh).all()
    d = Q.shape[3]
    for b in range(Q.shape[0]):
        for h in range(Q.shape[1]):
            th = util.oracle_theta_from_vec(theta[h], d)
            ref = orc.attention(th, Om[h], Q[b, h], K[b, h], V[b, h], s, causal)
            fro, row = util.attention_errors(Yh[b, h], ref, V[b, h].astype(np.float64))
            assert fro <= tol and row <= 4 * tol, (b, h, fro, row)


@pytest.mark.parametrize("case", range(16))
def test_bf16_paths_random_shapes(fs, case):
    import torch
    rng = np.random.default_rng(7000 + case)
    name = str(rng.choice(["c3", "c4", "c5"]))
    causal = True if name == "c5" else bool(rng.integers(0, 2))
    B, H = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    L = int(rng.choice([1, 17, 63, 64, 65, 127, 129, 191, 300, 511, 513, 777, 1024, 1500, 2049]))
    variant = str(rng.choice(VARIANTS))
    prepared = bool(rng.integers(0, 2))
    w = synth.make(name, B=B, H=H, L=L, seed=int(rng.integers(1, 10 ** 6)))
    Q, K, V, Om, s = w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"]
    theta = _theta_per_head(variant, Q, K, s)
    if theta is None:          # the dense families need non-singular second moments: too few rows in this draw
        theta = _theta_per_head("sderf", Q, K, s)
    td, Od = torch.from_numpy(theta).cuda(), torch.from_numpy(Om).cuda()
    Qd, Kd, Vd = (util.to_device(a, "bf16") for a in (Q, K, V))
    if prepared:
        prep = fs.attention_prepare(td, Od, B, H, s)
        Y = fs.attention_prepared(prep, td, Qd, Kd, Vd, s, Od, causal=causal, out_dtype=torch.float32)
    else:
        Y = fs.attention(td, Qd, Kd, Vd, s, Od, causal=causal, out_dtype=torch.float32)
    _compare(util.to_host(Y), theta, Om, Q, K, V, s, causal, 2e-2)


@pytest.mark.parametrize("case", range(16))
def test_general_path_random_shapes(fs, case):
    import torch
    rng = np.random.default_rng(8000 + case)
    causal = bool(rng.integers(0, 2))
    B, H = int(rng.integers(1, 3)), int(rng.integers(1, 3))
    d = int(rng.choice([1, 3, 8, 16, 24, 33, 64, 100, 128]))
    dv = int(rng.choice([1, 5, 16, d, 64]))
    M = int(rng.choice([1, 7, 32, 45, 64, 130, 256]))
    Lq = int(rng.choice([1, 2, 31, 32, 33, 100, 257, 600]))
    Lk = Lq if causal else int(rng.choice([1, 2, 31, 33, 100, 257, 600]))
    dtype = str(rng.choice(["f32", "bf16"]))
    variant = str(rng.choice(VARIANTS))
    s = float(d ** -0.25)
    Q = rng.standard_normal((B, H, Lq, d)).astype(np.float32)
    K = (rng.standard_normal((B, H, Lk, d)) + 0.1).astype(np.float32)
    V = rng.standard_normal((B, H, Lk, dv)).astype(np.float32)
    if dtype == "bf16":
        Q, K, V = (synth.round_to_bf16(a) for a in (Q, K, V))
    Om = rng.standard_normal((H, M, d)).astype(np.float32)
    theta = _theta_per_head(variant, Q, K, s)
    if theta is None:          # the dense families need non-singular second moments: too few rows in this draw
        theta = _theta_per_head("sderf", Q, K, s)
    out = torch.zeros((B, H, Lq, (dv + 3) // 4 * 4), dtype=torch.float32, device="cuda")[..., :dv]
    fs.attention(torch.from_numpy(theta).cuda(), _padded(Q, dtype), _padded(K, dtype), _padded(V, dtype), s,
                 torch.from_numpy(Om).cuda(), causal=causal, out=out)
    # storage in bf16 changes the inputs, not the arithmetic (fp32 on this path): both sides read the rounded numbers
    _compare(util.to_host(out), theta, Om, Q, K, V, s, causal, 1e-4)


@pytest.mark.parametrize("case", range(10))
def test_operator_random_shapes(fs, case):
    """Kernel operator on random shapes: those with d a multiple of 4 up to 64, M a multiple of 16 and at most 16
    columns take the fp32 MFMA operator kernels, the others the general-shape kernels; row norms from inside the unit
    ball to far outside it."""
    import torch
    rng = np.random.default_rng(9000 + case)
    d = int(rng.choice([4, 12, 32, 48, 64, 6, 33]))
    M = int(rng.choice([16, 48, 64, 512, 40, 7]))
    n = int(rng.choice([1, 3, 8, 16, 17]))
    Nx, Ny = int(rng.choice([1, 63, 64, 65, 300, 1000])), int(rng.choice([2, 64, 129, 500, 1025]))
    radius = float(rng.choice([0.5, 1.0, 2.0, 4.0]))
    variant = str(rng.choice(["posrf", "gerf", "sderf", "aderf"]))
    alpha = float(rng.choice([0.0, -0.5]))
    X = rng.standard_normal((Nx, d))
    Yp = rng.standard_normal((Ny, d)) + 0.2
    X = (radius * X / np.linalg.norm(X, axis=1, keepdims=True) * rng.uniform(0.7, 1.0, (Nx, 1))).astype(np.float32)
    Yp = (radius * Yp / np.linalg.norm(Yp, axis=1, keepdims=True) * rng.uniform(0.7, 1.0, (Ny, 1))).astype(np.float32)
    C = rng.standard_normal((Ny, n)).astype(np.float32)
    Om = rng.standard_normal((M, d)).astype(np.float32)
    try:
        vec = util.theta_vec_from_oracle(orc.fit(variant, np.concatenate([X, Yp]).astype(np.float64), Yp.astype(np.float64)))
    except Exception:          # the dense families need non-singular second moments: too few rows in this draw
        vec = util.theta_vec_from_oracle(orc.fit("sderf", np.concatenate([X, Yp]).astype(np.float64), Yp.astype(np.float64)))
    th = util.oracle_theta_from_vec(vec, d)
    ref = orc.kernel_matvec(th, Om, X, Yp, C, alpha)
    out = util.to_host(fs.kernel_matvec(torch.from_numpy(vec).cuda(), _padded(X[None, None], "f32")[0, 0],
                                        _padded(Yp[None, None], "f32")[0, 0], 1.0, alpha, torch.from_numpy(Om).cuda(),
                                        torch.from_numpy(C).cuda()))
    assert np.isfinite(out).all()
    assert np.linalg.norm(out - ref) <= 1e-4 * np.linalg.norm(ref), np.linalg.norm(out - ref) / np.linalg.norm(ref)
