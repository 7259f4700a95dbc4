"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element, on the same seeded
inputs, the same omega and the same parameter block.

Tolerances (relative): 1e-4 for f32 inputs, 2e-2 for bf16 inputs with f32 accumulation.  For attention the
relative error is the Frobenius one per (b, h), plus a per-row bound |dY_i| <= 4 tol max_j |V_j| (rows of Y
can be close to zero, so an element-wise relative error would be ill-posed).
"""
import numpy as np
import pytest

from oracle import favorsharp_oracle as orc
from paper_2302_00787_amd import synth
from tests import util

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def fs():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2302_00787_amd import binding
    binding.lib()                      # raises if the HIP library was not built: there is no fallback
    return binding


def _fit_theta_block(variant, Q, K, scale, groups_shape):
    """Oracle fit per group (here: per head, rows pooled over the batch) -> float32 parameter blocks."""
    B, H, L, d = Q.shape
    vecs = []
    for h in range(H):
        X = scale * Q[:, h].reshape(-1, d).astype(np.float64)
        Y = scale * K[:, h].reshape(-1, d).astype(np.float64)
        vecs.append(util.theta_vec_from_oracle(orc.fit(variant, X, Y)))
    return np.stack(vecs)


def _check_attention(fs, Q, K, V, Omega, scale, causal, variant, dtype, chunk=0, heads_to_check=None):
    import torch
    B, H, Lq, d = Q.shape
    theta = _fit_theta_block(variant, Q, K, scale, None)
    Y = fs.attention(torch.from_numpy(theta).cuda(), util.to_device(Q, dtype), util.to_device(K, dtype),
                     util.to_device(V, dtype), scale, torch.from_numpy(Omega).cuda(), causal=causal, chunk=chunk)
    torch.cuda.synchronize()
    Yh = util.to_host(Y)
    assert np.isfinite(Yh).all()
    tol = TOL[dtype]
    worst = (0.0, 0.0)
    for b in range(B):
        for h in (range(H) if heads_to_check is None else heads_to_check):
            th = util.oracle_theta_from_vec(theta[h], d)
            ref = orc.attention(th, Omega[h], Q[b, h], K[b, h], V[b, h], scale, causal)
            fro, row = util.attention_errors(Yh[b, h], ref, V[b, h].astype(np.float64))
            worst = (max(worst[0], fro), max(worst[1], row))
            assert fro <= tol, (b, h, fro)
            assert row <= 4 * tol, (b, h, row)
    return worst


# ----------------------------------------------------------------------------- features
@pytest.mark.parametrize("variant", ["posrf", "gerf", "saderf", "aderf", "sderf"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_features_match_oracle(fs, variant, dtype):
    import torch
    rng = np.random.default_rng(11)
    n, d, M = 77, 24, 45                      # ragged in rows and in features
    X = (0.8 * rng.standard_normal((n, d)) + 0.1).astype(np.float32)
    Yk = (0.7 * rng.standard_normal((n, d)) - 0.1).astype(np.float32)
    if dtype == "bf16":
        X, Yk = synth.round_to_bf16(X), synth.round_to_bf16(Yk)
    Om = rng.standard_normal((M, d)).astype(np.float32)
    scale = 0.9
    vec = util.theta_vec_from_oracle(orc.fit(variant, scale * X.astype(np.float64), scale * Yk.astype(np.float64)))
    th = util.oracle_theta_from_vec(vec, d)
    tdev, odev = torch.from_numpy(vec).cuda(), torch.from_numpy(Om).cuda()
    for side, data, alpha in ((1, X, 0.0), (2, Yk, -0.5)):
        ref = orc.features(th, Om, scale * data.astype(np.float64), side, alpha)
        out = util.to_host(fs.features(tdev, side, util.to_device(data, dtype), scale, alpha, odev))
        np.testing.assert_allclose(out, ref, rtol=1e-4)
        out_s, rls = fs.features(tdev, side, util.to_device(data, dtype), scale, alpha, odev, stabilise=True)
        E = orc.log_features(th, Om, scale * data.astype(np.float64), side, alpha)
        np.testing.assert_allclose(util.to_host(rls), E.max(axis=1), rtol=0, atol=2e-5 * max(1.0, np.abs(E).max()))
        np.testing.assert_allclose(util.to_host(out_s), np.exp(E - E.max(axis=1, keepdims=True)), rtol=1e-4, atol=1e-30)


# ----------------------------------------------------------------------------- attention, small general shapes
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("variant", ["sderf", "aderf", "saderf", "gerf"])
def test_attention_f32_small_ragged(fs, causal, variant):
    rng = np.random.default_rng(21)
    B, H, L, d, dv, M = 2, 3, 203, 24, 20, 72          # several 32-row tiles plus a ragged tail; M not a tile multiple
    Q = (rng.standard_normal((B, H, L, d)) + 0.2).astype(np.float32)
    K = (rng.standard_normal((B, H, L, d)) - 0.1).astype(np.float32)
    V = rng.standard_normal((B, H, L, dv)).astype(np.float32)
    Om = rng.standard_normal((H, M, d)).astype(np.float32)
    _check_attention(fs, Q, K, V, Om, d ** -0.25, causal, variant, "f32")


def test_attention_noncausal_different_lengths_and_strides(fs):
    import torch
    rng = np.random.default_rng(22)
    B, H, Lq, Lk, d, M = 1, 2, 50, 131, 16, 64
    Q = rng.standard_normal((B, H, Lq, d)).astype(np.float32)
    K = rng.standard_normal((B, H, Lk, d)).astype(np.float32)
    V = rng.standard_normal((B, H, Lk, d)).astype(np.float32)
    Om = rng.standard_normal((H, M, d)).astype(np.float32)
    s = d ** -0.25
    theta = np.stack([util.theta_vec_from_oracle(orc.fit_sderf(s * Q[0, h].astype(np.float64), s * K[0, h].astype(np.float64)))
                      for h in range(H)])
    # keys and values interleaved in one buffer: [B, Lk, H, 2, d] viewed as two strided [B,H,Lk,d] tensors
    kv = torch.empty((B, Lk, H, 2, d), dtype=torch.float32, device="cuda")
    kv[:, :, :, 0] = torch.from_numpy(K).cuda().permute(0, 2, 1, 3)
    kv[:, :, :, 1] = torch.from_numpy(V).cuda().permute(0, 2, 1, 3)
    Kd, Vd = kv[:, :, :, 0].permute(0, 2, 1, 3), kv[:, :, :, 1].permute(0, 2, 1, 3)
    Y = fs.attention(torch.from_numpy(theta).cuda(), torch.from_numpy(Q).cuda(), Kd, Vd, s, torch.from_numpy(Om).cuda())
    Yh = util.to_host(Y)
    for h in range(H):
        ref = orc.attention(util.oracle_theta_from_vec(theta[h], d), Om[h], Q[0, h], K[0, h], V[0, h], s, False)
        fro, row = util.attention_errors(Yh[0, h], ref, V[0, h].astype(np.float64))
        assert fro <= 1e-4 and row <= 4e-4


def test_attention_group_modes(fs):
    """One parameter set / omega for everything, per head, and per (batch, head) all address the right block."""
    import torch
    rng = np.random.default_rng(23)
    B, H, L, d, M = 2, 2, 64, 16, 32
    Q = rng.standard_normal((B, H, L, d)).astype(np.float32)
    K = rng.standard_normal((B, H, L, d)).astype(np.float32)
    V = rng.standard_normal((B, H, L, d)).astype(np.float32)
    s = d ** -0.25
    for groups in (1, H, B * H):
        Om = rng.standard_normal((groups, M, d)).astype(np.float32)
        vecs = []
        for g in range(groups):
            sel = [(b, h) for b in range(B) for h in range(H) if (0 if groups == 1 else h if groups == H else b * H + h) == g]
            X = np.concatenate([s * Q[b, h] for b, h in sel]).astype(np.float64)
            Yk = np.concatenate([s * K[b, h] for b, h in sel]).astype(np.float64)
            vecs.append(util.theta_vec_from_oracle(orc.fit_sderf(X, Yk)))
        theta = np.stack(vecs)
        Y = util.to_host(fs.attention(torch.from_numpy(theta).cuda(), torch.from_numpy(Q).cuda(), torch.from_numpy(K).cuda(),
                                      torch.from_numpy(V).cuda(), s, torch.from_numpy(Om).cuda(), causal=True))
        for b in range(B):
            for h in range(H):
                g = 0 if groups == 1 else h if groups == H else b * H + h
                ref = orc.attention(util.oracle_theta_from_vec(theta[g], d), Om[g], Q[b, h], K[b, h], V[b, h], s, True)
                fro, row = util.attention_errors(Y[b, h], ref, V[b, h].astype(np.float64))
                assert fro <= 1e-4 and row <= 4e-4, (groups, b, h)


@pytest.mark.parametrize("L,M,d", [(1, 1, 4), (33, 16, 8), (64, 200, 128)])
def test_attention_degenerate_sizes(fs, L, M, d):
    rng = np.random.default_rng(24)
    Q = rng.standard_normal((1, 1, L, d)).astype(np.float32)
    K = rng.standard_normal((1, 1, L, d)).astype(np.float32)
    V = rng.standard_normal((1, 1, L, d)).astype(np.float32)
    Om = rng.standard_normal((1, M, d)).astype(np.float32)
    for causal in (False, True):
        _check_attention(fs, Q, K, V, Om, d ** -0.25, causal, "sderf", "f32")


def test_attention_empty_query_set_and_error_paths(fs):
    import torch
    d, M = 16, 32
    th = torch.from_numpy(util.theta_vec_from_oracle(orc.fit_posrf(d))[None]).cuda()
    Om = torch.randn(1, M, d, device="cuda")
    K = torch.randn(1, 1, 40, d, device="cuda")
    Y = fs.attention(th, torch.empty(1, 1, 0, d, device="cuda"), K, K, 0.5, Om)
    assert Y.shape == (1, 1, 0, d)
    with pytest.raises(fs.FavorSharpError) as e:
        fs.attention(th, K[:, :, :20], K, K, 0.5, Om, causal=True)            # causal needs Lq == Lk
    assert e.value.status == 2
    with pytest.raises(fs.FavorSharpError) as e:
        fs.attention(th, K, K, K, 0.5, Om, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 4


# ----------------------------------------------------------------------------- kernel operator
@pytest.mark.parametrize("variant", ["sderf", "aderf"])
def test_kernel_matvec_small(fs, variant):
    import torch
    rng = np.random.default_rng(31)
    Nx, Ny, d, M, n = 70, 121, 12, 56, 5
    X = rng.random((Nx, d)).astype(np.float32)
    Yp = rng.random((Ny, d)).astype(np.float32)
    C = rng.standard_normal((Ny, n)).astype(np.float32)
    Om = rng.standard_normal((M, d)).astype(np.float32)
    vec = util.theta_vec_from_oracle(orc.fit(variant, X.astype(np.float64), Yp.astype(np.float64)))
    th = util.oracle_theta_from_vec(vec, d)
    for alpha in (0.0, -0.5):
        ref = orc.kernel_matvec(th, Om, X, Yp, C, alpha)
        out = util.to_host(fs.kernel_matvec(torch.from_numpy(vec).cuda(), torch.from_numpy(X).cuda(),
                                            torch.from_numpy(Yp).cuda(), 1.0, alpha, torch.from_numpy(Om).cuda(),
                                            torch.from_numpy(C).cuda()))
        assert np.linalg.norm(out - ref) / np.linalg.norm(ref) <= 1e-4
        np.testing.assert_allclose(out, ref, rtol=1e-3, atol=1e-4 * np.abs(ref).max())


@pytest.mark.parametrize("variant", ["sderf", "aderf"])
@pytest.mark.parametrize("Nx,Ny,d,M,n", [(70, 121, 12, 64, 5), (333, 1000, 32, 512, 16), (129, 64, 64, 48, 1), (1, 257, 4, 16, 3)])
def test_kernel_matvec_on_the_operator_kernels(fs, variant, Nx, Ny, d, M, n):
    """Shapes that take the fp32 MFMA operator kernels (fp32 rows, d a multiple of 4 up to 64, M a multiple of 16, at
    most 16 right-hand sides): different and ragged set sizes, dense and isotropic quadratic forms, both exponents."""
    import torch
    rng = np.random.default_rng(1000 * d + M)
    X = (rng.random((Nx, d)) * 1.2 - 0.1).astype(np.float32)
    Yp = (rng.random((Ny, d)) * 0.9 + 0.05).astype(np.float32)
    C = rng.standard_normal((Ny, n)).astype(np.float32)
    Om = rng.standard_normal((M, d)).astype(np.float32)
    fitX = X if Nx >= d + 2 else np.concatenate([X, Yp[: d + 2]])      # the dense families need a non-singular M1
    vec = util.theta_vec_from_oracle(orc.fit(variant, fitX.astype(np.float64), Yp.astype(np.float64)))
    th = util.oracle_theta_from_vec(vec, d)
    for alpha in (0.0, -0.5):
        ref = orc.kernel_matvec(th, Om, X, Yp, C, alpha)
        out = util.to_host(fs.kernel_matvec(torch.from_numpy(vec).cuda(), torch.from_numpy(X).cuda(),
                                            torch.from_numpy(Yp).cuda(), 1.0, alpha, torch.from_numpy(Om).cuda(),
                                            torch.from_numpy(C).cuda()))
        assert np.isfinite(out).all()
        assert np.linalg.norm(out - ref) / np.linalg.norm(ref) <= 1e-4, (alpha, np.linalg.norm(out - ref) / np.linalg.norm(ref))
        np.testing.assert_allclose(out, ref, rtol=1e-3, atol=1e-4 * np.abs(ref).max())


# ----------------------------------------------------------------------------- fit
def _fit(fs, entry, variant, Qd, Kd, s, groups):
    """theta [groups, floats] on the host from either fit entry point."""
    if entry == "host":
        return util.to_host(fs.fit_params(variant, Qd, Kd, s, groups=groups))
    theta, status = fs.fit_params_device(variant, Qd, Kd, s, groups=groups)
    assert util.to_host(status).tolist() == [0] * groups
    return util.to_host(theta)


@pytest.mark.parametrize("entry", ["host", "device"])
@pytest.mark.parametrize("variant", ["posrf", "gerf", "saderf", "aderf", "sderf"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fit_params_invariants(fs, variant, dtype, entry):
    """Eigenvectors are unique only up to sign / rotation inside equal eigenvalues, so the fit is compared on what
    is unique: A, log D, the objective value, B^T B and B1^T B2, and the validity conditions of the DERF theorem.
    Both entry points (closed forms on the host, closed forms on the device) are held to the same oracle."""
    rng = np.random.default_rng(41)
    B, H, L, d = 2, 3, 300, 16
    sc = np.linspace(0.4, 1.3, d)
    Q = (rng.standard_normal((B, H, L, d)) * sc + 0.15).astype(np.float32)
    K = (rng.standard_normal((B, H, L, d)) * sc[::-1] - 0.1).astype(np.float32)
    if dtype == "bf16":
        Q, K = synth.round_to_bf16(Q), synth.round_to_bf16(K)
    s = d ** -0.25
    theta = _fit(fs, entry, variant, util.to_device(Q, dtype), util.to_device(K, dtype), s, H)
    for h in range(H):
        X = s * Q[:, h].reshape(-1, d).astype(np.float64)
        Yk = s * K[:, h].reshape(-1, d).astype(np.float64)
        ref = orc.fit(variant, X, Yk)
        got = util.oracle_theta_from_vec(theta[h], d)
        np.testing.assert_allclose(np.sort(got.A), np.sort(ref.A), atol=2e-5)
        assert got.logD == pytest.approx(ref.logD, abs=1e-4)
        if ref.lbar is not None:
            assert float(theta[h][1]) == pytest.approx(ref.lbar, abs=2e-4 * max(1.0, abs(ref.lbar)))
        np.testing.assert_allclose(got.B1.T @ got.B1, ref.B1.T @ ref.B1, atol=3e-4)
        np.testing.assert_allclose(got.B1.T @ got.B2, ref.B1.T @ ref.B2, atol=3e-4)
        np.testing.assert_allclose(got.C1, ref.C1, atol=3e-4)
        np.testing.assert_allclose(got.C2, ref.C2, atol=3e-4)
        r = orc.validity_residuals(got)
        assert r["max_8A"] < 1 and r["cross"] < 1e-4 and r["C1"] < 1e-4 and r["C2"] < 1e-4 and r["logD"] < 1e-4
        # the fitted parameters reach the oracle's optimum of the objective on the same data
        assert orc.lbar_bruteforce(got, X[:200], Yk[:200]) == pytest.approx(orc.lbar_bruteforce(ref, X[:200], Yk[:200]), abs=2e-4)


@pytest.mark.parametrize("entry", ["host", "device"])
@pytest.mark.parametrize("variant", ["posrf", "gerf", "saderf", "aderf", "sderf"])
def test_fit_params_sets_of_different_sizes(fs, variant, entry):
    """Lx != Ly: every statistic is a mean over its own set (Section 4.3's Psi is then the ratio of per-set means,
    not of sums), for all five families on both fit entry points."""
    rng = np.random.default_rng(43)
    B, H, Lx, Ly, d = 2, 2, 200, 520, 16
    sc = np.linspace(0.4, 1.3, d)
    Q = (rng.standard_normal((B, H, Lx, d)) * sc + 0.15).astype(np.float32)
    K = (rng.standard_normal((B, H, Ly, d)) * sc[::-1] - 0.1).astype(np.float32)
    s = d ** -0.25
    theta = _fit(fs, entry, variant, util.to_device(Q, "f32"), util.to_device(K, "f32"), s, H)
    for h in range(H):
        X = s * Q[:, h].reshape(-1, d).astype(np.float64)
        Yk = s * K[:, h].reshape(-1, d).astype(np.float64)
        ref = orc.fit(variant, X, Yk)
        got = util.oracle_theta_from_vec(theta[h], d)
        np.testing.assert_allclose(np.sort(got.A), np.sort(ref.A), atol=2e-5)
        assert got.logD == pytest.approx(ref.logD, abs=1e-4)
        if ref.lbar is not None:
            assert float(theta[h][1]) == pytest.approx(ref.lbar, abs=2e-4 * max(1.0, abs(ref.lbar)))
        np.testing.assert_allclose(got.B1.T @ got.B1, ref.B1.T @ ref.B1, atol=3e-4)
        np.testing.assert_allclose(got.B1.T @ got.B2, ref.B1.T @ ref.B2, atol=3e-4)
        np.testing.assert_allclose(got.C1, ref.C1, atol=3e-4)
        np.testing.assert_allclose(got.C2, ref.C2, atol=3e-4)
        assert orc.lbar_bruteforce(got, X[:150], Yk[:200]) == pytest.approx(orc.lbar_bruteforce(ref, X[:150], Yk[:200]), abs=2e-4)


@pytest.mark.parametrize("variant", ["sderf", "aderf"])
@pytest.mark.parametrize("d", [9, 64, 128])
def test_device_fit_dense_families_at_other_sizes(fs, variant, d):
    """The device-resident fit at an odd d (strided rows; the round-robin ordering gets a bye), at d = 64 (matrices in
    LDS) and at d = 128 (matrices in global memory), on anisotropic data with a mean, against the oracle's fit."""
    import torch
    rng = np.random.default_rng(300 + d)
    L, dpad = 700, (d + 3) // 4 * 4
    U, _ = np.linalg.qr(rng.standard_normal((d, d)))
    spec = np.linspace(1.2, 0.3, d)
    Q = np.zeros((1, 1, L, dpad), np.float32)
    K = np.zeros((1, 1, L, dpad), np.float32)
    Q[..., :d] = (rng.standard_normal((L, d)) * spec) @ U.T + 0.1
    K[..., :d] = (rng.standard_normal((L, d)) * spec[::-1]) @ U.T - 0.05
    s = d ** -0.25
    Qd, Kd = torch.from_numpy(Q).cuda()[..., :d], torch.from_numpy(K).cuda()[..., :d]
    theta = _fit(fs, "device", variant, Qd, Kd, s, 1)
    X = s * Q[0, 0, :, :d].astype(np.float64)
    Yk = s * K[0, 0, :, :d].astype(np.float64)
    ref = orc.fit(variant, X, Yk)
    got = util.oracle_theta_from_vec(theta[0], d)
    np.testing.assert_allclose(np.sort(got.A), np.sort(ref.A), atol=2e-5)
    assert got.logD == pytest.approx(ref.logD, abs=1e-4 * max(1.0, abs(ref.logD)))
    assert float(theta[0][1]) == pytest.approx(ref.lbar, abs=2e-4 * max(1.0, abs(ref.lbar)))
    np.testing.assert_allclose(got.B1.T @ got.B1, ref.B1.T @ ref.B1, atol=3e-4)
    np.testing.assert_allclose(got.B1.T @ got.B2, ref.B1.T @ ref.B2, atol=3e-4)
    np.testing.assert_allclose(got.C1, ref.C1, atol=3e-4)
    np.testing.assert_allclose(got.C2, ref.C2, atol=3e-4)
    r = orc.validity_residuals(got)
    assert r["max_8A"] < 1 and r["cross"] < 1e-4 and r["C1"] < 1e-4 and r["C2"] < 1e-4 and r["logD"] < 1e-4
    # and the host entry point agrees on the same invariants
    host = util.oracle_theta_from_vec(_fit(fs, "host", variant, Qd, Kd, s, 1)[0], d)
    np.testing.assert_allclose(np.sort(got.A), np.sort(host.A), atol=2e-5)
    np.testing.assert_allclose(got.B1.T @ got.B2, host.B1.T @ host.B2, atol=3e-4)


@pytest.mark.parametrize("entry", ["host", "device"])
@pytest.mark.parametrize("d", [64, 128])
def test_fit_on_bf16_rows_scanned_by_the_mfma_statistics_kernels(fs, d, entry):
    """bf16 rows of 64 and of 128 numbers take the MFMA statistics kernels.  Packed [B, L, H, d] storage (row stride
    H d), a length that is neither a multiple of the 64-row tile nor of the scan's row chunk, one parameter set per
    head: the fit is held to the oracle's on the same (bf16-rounded) numbers."""
    import torch
    rng = np.random.default_rng(500 + d)
    B, H, L = 2, 2, 1333
    U, _ = np.linalg.qr(rng.standard_normal((d, d)))
    spec = np.linspace(1.2, 0.3, d)
    Q = synth.round_to_bf16(((rng.standard_normal((B, H, L, d)) * spec) @ U.T + 0.1).astype(np.float32))
    K = synth.round_to_bf16(((rng.standard_normal((B, H, L, d)) * spec[::-1]) @ U.T - 0.05).astype(np.float32))
    s = d ** -0.25
    packed = torch.empty((B, L, H, 2, d), dtype=torch.bfloat16, device="cuda")
    packed[:, :, :, 0] = util.to_device(Q, "bf16").permute(0, 2, 1, 3)
    packed[:, :, :, 1] = util.to_device(K, "bf16").permute(0, 2, 1, 3)
    Qd, Kd = packed[:, :, :, 0].permute(0, 2, 1, 3), packed[:, :, :, 1].permute(0, 2, 1, 3)
    theta = _fit(fs, entry, "sderf", Qd, Kd, s, H)
    for h in range(H):
        X = s * Q[:, h].reshape(-1, d).astype(np.float64)
        Yk = s * K[:, h].reshape(-1, d).astype(np.float64)
        ref = orc.fit("sderf", X, Yk)
        got = util.oracle_theta_from_vec(theta[h], d)
        np.testing.assert_allclose(np.sort(got.A), np.sort(ref.A), atol=2e-5)
        assert got.logD == pytest.approx(ref.logD, abs=1e-4 * max(1.0, abs(ref.logD)))
        assert float(theta[h][1]) == pytest.approx(ref.lbar, abs=2e-4 * max(1.0, abs(ref.lbar)))
        np.testing.assert_allclose(got.B1.T @ got.B1, ref.B1.T @ ref.B1, atol=3e-4)
        np.testing.assert_allclose(got.B1.T @ got.B2, ref.B1.T @ ref.B2, atol=3e-4)
        np.testing.assert_allclose(got.C2, ref.C2, atol=3e-4)


def test_device_fit_reports_singular_statistics_per_group(fs):
    """ADERF needs nonsingular second moments: a head whose queries miss one coordinate gets FS_ERR_NOT_PD in its own
    status word, the other head is fitted; the host entry point returns the same code for the call."""
    import torch
    rng = np.random.default_rng(77)
    B, H, L, d = 1, 2, 200, 8
    Q = rng.standard_normal((B, H, L, d)).astype(np.float32)
    K = rng.standard_normal((B, H, L, d)).astype(np.float32)
    Q[:, 1, :, 3] = 0.0
    Qd, Kd = torch.from_numpy(Q).cuda(), torch.from_numpy(K).cuda()
    s = d ** -0.25
    theta, status = fs.fit_params_device("aderf", Qd, Kd, s, groups=H)
    assert util.to_host(status).tolist() == [0, 3]
    ref = orc.fit("aderf", s * Q[0, 0].astype(np.float64), s * K[0, 0].astype(np.float64))
    got = util.oracle_theta_from_vec(util.to_host(theta)[0], d)
    np.testing.assert_allclose(got.B1.T @ got.B2, ref.B1.T @ ref.B2, atol=3e-4)
    with pytest.raises(fs.FavorSharpError) as err:
        fs.fit_params("aderf", Qd, Kd, s, groups=H)
    assert err.value.status == 3


def test_device_fit_then_attention_without_host_round_trip(fs):
    """Fit on the device and attention enqueued right behind it on the same stream; the parameter block is
    downloaded afterwards and handed to the oracle, so the whole path is checked on one theta."""
    import torch
    w = synth.make("c4", B=1, H=2, L=640)
    Q, K, V, Om, s = w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"]
    Qd, Kd, Vd = (util.to_device(a, "bf16") for a in (Q, K, V))
    theta, status = fs.fit_params_device("sderf", Qd, Kd, s, groups=2)
    Y = util.to_host(fs.attention(theta, Qd, Kd, Vd, s, torch.from_numpy(Om).cuda(), causal=True, chunk=64))
    assert util.to_host(status).tolist() == [0, 0]
    th_host = util.to_host(theta)
    for h in range(2):
        th = util.oracle_theta_from_vec(th_host[h].astype(np.float32), w["d"])
        ref = orc.attention(th, Om[h], Q[0, h], K[0, h], V[0, h], s, True)
        fro, row = util.attention_errors(Y[0, h], ref, V[0, h].astype(np.float64))
        assert fro <= 2e-2 and row <= 8e-2


def test_fit_then_attention_end_to_end(fs):
    """theta fitted by the library, downloaded and handed to the oracle: the whole path on one parameter block."""
    import torch
    w = synth.make("c1")
    Q, K, V, Om, s = w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"]
    Qd, Kd, Vd = (torch.from_numpy(a).cuda() for a in (Q, K, V))
    theta = fs.fit_params("sderf", Qd, Kd, s, groups=1)
    Y = util.to_host(fs.attention(theta, Qd, Kd, Vd, s, torch.from_numpy(Om).cuda()))
    th = util.oracle_theta_from_vec(util.to_host(theta)[0].astype(np.float32), w["d"])
    ref = orc.attention(th, Om[0], Q[0, 0], K[0, 0], V[0, 0], s, False)
    fro, row = util.attention_errors(Y[0, 0], ref, V[0, 0].astype(np.float64))
    assert fro <= 1e-4 and row <= 4e-4


# ----------------------------------------------------------------------------- the five workloads
def test_c1_full(fs):
    w = synth.make("c1")
    _check_attention(fs, w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"], False, "sderf", "f32")


def test_c2_full(fs):
    import torch
    w = synth.make("c2")
    X, C, Om = w["X"], w["C"], w["Omega"][0]
    vec = util.theta_vec_from_oracle(orc.fit_sderf(X.astype(np.float64), X.astype(np.float64)))
    th = util.oracle_theta_from_vec(vec, w["d"])
    Xd = torch.from_numpy(X).cuda()
    out = util.to_host(fs.kernel_matvec(torch.from_numpy(vec).cuda(), Xd, Xd, 1.0, w["alpha"], torch.from_numpy(Om).cuda(),
                                        torch.from_numpy(C).cuda()))
    ref = orc.kernel_matvec(th, Om, X, X, C, w["alpha"])
    assert np.linalg.norm(out - ref) / np.linalg.norm(ref) <= 1e-4
    assert np.abs(out - ref).max() <= 1e-4 * np.abs(ref).max() * 4


@pytest.mark.parametrize("name,over", [
    ("c3", dict(B=2, H=2, L=704)),
    ("c4", dict(B=1, H=2, L=1216)),
    ("c5", dict(B=1, H=2, L=832)),
])
def test_bf16_workloads_reduced(fs, name, over):
    """The bf16 workloads at their real d, M and statistics, shortened so the oracle finishes in seconds; the
    lengths are not multiples of 128 so several tiles and a ragged tail are covered."""
    w = synth.make(name, **over)
    _check_attention(fs, w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"], w["causal"], "sderf", "bf16",
                     chunk=w.get("chunk", 0))


# ----------------------------------------------------------------------------- bf16 MFMA path (d = 64, M = 256)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("L", [64, 100, 1000])
@pytest.mark.parametrize("variant", ["sderf", "aderf"])
def test_bf16_path_lengths_and_variants(fs, causal, L, variant):
    """Chunk-exact, ragged and multi-segment lengths; ADERF exercises the dense key-side quadratic form."""
    w = synth.make("c4", B=2, H=2, L=L, seed=77 + L)
    worst = _check_attention(fs, w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"], causal, variant, "bf16", chunk=64)
    print(f"bf16 path causal={causal} L={L} {variant}: worst frobenius {worst[0]:.2e}, worst row {worst[1]:.2e}")


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("H,L", [(1, 4096), (1, 5000), (2, 8209)])
def test_bf16_path_few_sequences_many_slots(fs, causal, H, L):
    """One or two sequences cut into 64 and more slots: the slot reduction then runs range by range (totals per range,
    a scan over them, and for causal calls a walk over every range), in another summation order than the one-kernel
    form: whole sequences against the oracle, chunk-exact and ragged lengths, one and two slots per segment."""
    w = synth.make("c4", B=1, H=H, L=L, seed=401 + L)
    worst = _check_attention(fs, w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"], causal, "sderf", "bf16", chunk=64)
    print(f"bf16 path, ranges, causal={causal} H={H} L={L}: worst frobenius {worst[0]:.2e}, worst row {worst[1]:.2e}")


def test_bf16_path_few_sequences_many_slots_late_outlier(fs):
    """The running shifts survive the range form: a key with a huge bound late in a single sequence of 64 slots leaves
    the rows of all earlier segments within tolerance (as in the late-key test, which has too few slots for ranges)."""
    import torch
    L = 4096
    w = synth.make("c4", B=1, H=1, L=L, seed=419)
    Q, K, V, s, d = w["Q"], w["K"].copy(), w["V"], w["qk_scale"], w["d"]
    Om = (2.2 * w["Omega"]).astype(np.float32)
    longest = float(np.linalg.norm(Om[0], axis=1).max())
    late = L - 300
    K[0, 0, late] *= (longest / s) / np.linalg.norm(K[0, 0, late])
    K = synth.round_to_bf16(K)
    vec = util.theta_vec_from_oracle(orc.fit_posrf(d))
    th = util.oracle_theta_from_vec(vec, d)
    Y = fs.attention(torch.from_numpy(vec[None]).cuda(), util.to_device(Q, "bf16"), util.to_device(K, "bf16"),
                     util.to_device(V, "bf16"), s, torch.from_numpy(Om).cuda(), causal=True, out_dtype=torch.float32)
    Yh = util.to_host(Y)[0, 0]
    assert np.isfinite(Yh).all()
    ref = orc.attention(th, Om[0], Q[0, 0], K[0, 0], V[0, 0], s, True)
    safe = (late // 64) * 64
    fro, row = util.attention_errors(Yh[:safe], ref[:safe], V[0, 0, :safe].astype(np.float64))
    assert fro <= 2e-2 and row <= 8e-2, (fro, row)


@pytest.mark.parametrize("variant,B,H,Lq,Lk", [("sderf", 64, 8, 300, 300), ("gerf", 64, 8, 70, 333), ("aderf", 1, 2, 128, 128),
                                               ("saderf", 2, 2, 200, 64), ("posrf", 1, 1, 1, 1), ("sderf", 1, 3, 64, 256),
                                               ("aderf", 1, 2, 256, 190)])
def test_bf16_path_non_causal_whole_sequences_per_workgroup(fs, variant, B, H, Lq, Lk):
    """Non-causal calls with many sequences (B*H >= 512) or short ones (at most four chunks) run one workgroup per
    sequence, the state staying in registers between the key rows and the query rows: equal and different numbers
    of queries and keys, ragged tails, a single token, isotropic and dense key-side quadratic forms."""
    w = synth.make("c3", B=B, H=H, L=max(Lq, Lk), seed=431 + Lq + Lk)
    worst = _check_attention(fs, w["Q"][:, :, :Lq], w["K"][:, :, :Lk], w["V"][:, :, :Lk], w["Omega"], w["qk_scale"],
                             False, variant, "bf16")
    print(f"bf16 path, whole sequences, B={B} H={H} Lq={Lq} Lk={Lk} {variant}: worst frobenius {worst[0]:.2e}, "
          f"worst row {worst[1]:.2e}")


@pytest.mark.parametrize("variant,L", [("sderf", 128), ("aderf", 100), ("gerf", 333)])
def test_bf16_path_causal_many_short_sequences(fs, variant, L):
    """Causal calls with 256 sequences or more are one segment per sequence: no state pass and no reduction run, the
    causal kernel starts every sequence from nothing (and must not read a prefix state that nobody wrote: the
    workspace is filled with NaN bit patterns first)."""
    import torch
    w = synth.make("c4", B=32, H=8, L=L, seed=443 + L)
    Q, K, V, Om, s, d = w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"], w["d"]
    theta = _fit_theta_block(variant, Q, K, s, None)
    ws = torch.full((fs.attention_workspace_bytes(32, 8, L, L, d, d, Om.shape[1], True, 8, Om.shape[0]),), 0xFF,
                    dtype=torch.uint8, device="cuda")
    Y = fs.attention(torch.from_numpy(theta).cuda(), util.to_device(Q, "bf16"), util.to_device(K, "bf16"),
                     util.to_device(V, "bf16"), s, torch.from_numpy(Om).cuda(), causal=True, chunk=64, workspace=ws)
    assert fs.attention_flushed_rows(ws) == 0
    Yh = util.to_host(Y)
    assert np.isfinite(Yh).all()
    worst = (0.0, 0.0)
    for b in range(0, 32, 5):
        for h in range(8):
            ref = orc.attention(util.oracle_theta_from_vec(theta[h], d), Om[h], Q[b, h], K[b, h], V[b, h], s, True)
            fro, row = util.attention_errors(Yh[b, h], ref, V[b, h].astype(np.float64))
            worst = (max(worst[0], fro), max(worst[1], row))
            assert fro <= 2e-2 and row <= 8e-2, (b, h, fro, row)
    print(f"bf16 path, causal, 256 sequences of {L} {variant}: worst frobenius {worst[0]:.2e}, worst row {worst[1]:.2e}")


# ----------------------------------------------------------------------------- bf16 MFMA path (d = 128, M = 512)
@pytest.mark.parametrize("variant,L", [("posrf", 1), ("sderf", 64), ("sderf", 100), ("sderf", 1000), ("aderf", 200),
                                       ("aderf", 1000)])
def test_bf16_wide_path_lengths_and_variants(fs, L, variant):
    """The long-context shape (causal, d = dv = 128, M = 512: two feature halves x two column halves per call) on
    single-token, chunk-exact, ragged and multi-slot lengths; ADERF (fitted on more than d rows, so that its
    statistics are nonsingular) exercises the dense key-side quadratic form."""
    w = synth.make("c5", B=1, H=2, L=L, seed=177 + L)
    worst = _check_attention(fs, w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"], True, variant, "bf16", chunk=64)
    print(f"bf16 wide path L={L} {variant}: worst frobenius {worst[0]:.2e}, worst row {worst[1]:.2e}")


@pytest.mark.parametrize("variant,L", [("posrf", 1), ("sderf", 64), ("sderf", 100), ("sderf", 1000), ("aderf", 200),
                                       ("aderf", 1000), ("gerf", 333)])
def test_bf16_wide_path_non_causal(fs, L, variant):
    """The same shape without the mask (the query pass of the walk on the sum of all slot states, no key tiles in
    it): single-token, chunk-exact, ragged and multi-slot lengths, isotropic and dense key-side quadratic forms."""
    w = synth.make("c5", B=1, H=2, L=L, seed=277 + L)
    worst = _check_attention(fs, w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"], False, variant, "bf16")
    print(f"bf16 wide path, non-causal, L={L} {variant}: worst frobenius {worst[0]:.2e}, worst row {worst[1]:.2e}")


@pytest.mark.parametrize("variant,Lq,Lk", [("sderf", 300, 200), ("sderf", 64, 1000), ("aderf", 1000, 200),
                                           ("gerf", 1, 500), ("posrf", 700, 1), ("saderf", 130, 131)])
def test_bf16_wide_path_non_causal_other_numbers_of_queries_than_keys(fs, variant, Lq, Lk):
    """Without the mask the queries and the keys are cut into slots separately (state kernel and reduction over the
    keys' slots, the query pass over the queries'): more queries than keys, fewer, a single query, a single key."""
    w = synth.make("c5", B=1, H=2, L=max(Lq, Lk), seed=291 + Lq + Lk)
    worst = _check_attention(fs, w["Q"][:, :, :Lq], w["K"][:, :, :Lk], w["V"][:, :, :Lk], w["Omega"], w["qk_scale"],
                             False, variant, "bf16")
    print(f"bf16 wide path, non-causal, Lq={Lq} Lk={Lk} {variant}: worst frobenius {worst[0]:.2e}, worst row {worst[1]:.2e}")


@pytest.mark.parametrize("Lk", [300, 200])
def test_bf16_wide_path_non_causal_runs_on_the_wide_kernels(fs, Lk):
    """Non-causal calls take the d = 128 kernels, with as many queries as keys and with other numbers: query rows 120
    times longer than the data's flush on their bound-based shifts and are counted (the general-shape kernels, with
    exact maxima, never flush a query)."""
    import torch
    w = synth.make("c5", B=1, H=2, L=300, seed=281)
    Q, K, V, Om, s, d = w["Q"].copy(), w["K"][:, :, :Lk], w["V"][:, :, :Lk], w["Omega"], w["qk_scale"], w["d"]
    Q[:, :, [7, 150]] *= 120.0
    Q = synth.round_to_bf16(Q)
    vec = util.theta_vec_from_oracle(orc.fit_posrf(d))
    thd, Omd = torch.from_numpy(vec[None]).cuda(), torch.from_numpy(Om).cuda()
    ws = torch.empty(fs.attention_workspace_bytes(1, 2, 300, Lk, d, d, Om.shape[1], False, 1, Om.shape[0]),
                     dtype=torch.uint8, device="cuda")
    Y = fs.attention(thd, util.to_device(Q, "bf16"), util.to_device(K, "bf16"), util.to_device(V, "bf16"), s, Omd,
                     causal=False, workspace=ws, out_dtype=torch.float32)
    assert fs.attention_flushed_rows(ws) == 4
    Yh = util.to_host(Y)
    assert np.isfinite(Yh).all()
    assert (Yh[:, :, [7, 150]] == 0).all()
    th = util.oracle_theta_from_vec(vec, d)
    keep = np.setdiff1d(np.arange(300), [7, 150])
    for h in range(2):
        ref = orc.attention(th, Om[h], Q[0, h], K[0, h], V[0, h], s, False)
        fro, row = util.attention_errors(Yh[0, h][keep], ref[keep], V[0, h].astype(np.float64))
        assert fro <= 2e-2 and row <= 8e-2, (h, fro, row)


@pytest.mark.parametrize("variant,L,causal", [("sderf", 200, True), ("aderf", 320, True), ("saderf", 200, False)])
def test_bf16_wide_path_one_slot_per_sequence(fs, variant, L, causal):
    """Calls of the d = 128 shape with 128 sequences or more have one slot per sequence.  Causal: no state is computed
    or scanned, the walks start from a block of zeros and only the key shift of each sequence is computed beforehand.
    Non-causal: the state of the only slot is the total, no reduction runs.  (NaN bit patterns in the workspace:
    nothing unwritten may be read; every third batch entry against the oracle.)"""
    import torch
    w = synth.make("c5", B=16, H=8, L=L, seed=457 + L)
    Q, K, V, Om, s, d = w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"], w["d"]
    theta = _fit_theta_block(variant, Q, K, s, None)
    ws = torch.full((fs.attention_workspace_bytes(16, 8, L, L, d, d, Om.shape[1], causal, 8, Om.shape[0]),), 0xFF,
                    dtype=torch.uint8, device="cuda")
    Y = fs.attention(torch.from_numpy(theta).cuda(), util.to_device(Q, "bf16"), util.to_device(K, "bf16"),
                     util.to_device(V, "bf16"), s, torch.from_numpy(Om).cuda(), causal=causal, chunk=64 if causal else 0,
                     workspace=ws)
    assert fs.attention_flushed_rows(ws) == 0
    Yh = util.to_host(Y)
    assert np.isfinite(Yh).all()
    worst = (0.0, 0.0)
    for b in range(0, 16, 3):
        for h in range(8):
            ref = orc.attention(util.oracle_theta_from_vec(theta[h], d), Om[h], Q[b, h], K[b, h], V[b, h], s, causal)
            fro, row = util.attention_errors(Yh[b, h], ref, V[b, h].astype(np.float64))
            worst = (max(worst[0], fro), max(worst[1], row))
            assert fro <= 2e-2 and row <= 8e-2, (b, h, fro, row)
    print(f"bf16 wide path, causal={causal}, 128 sequences of {L} {variant}: worst frobenius {worst[0]:.2e}, "
          f"worst row {worst[1]:.2e}")


def test_bf16_wide_path_f32_output_and_strided_inputs(fs):
    import torch
    w = synth.make("c5", B=2, H=2, L=320)
    Q, K, V, Om, s, d = w["Q"], w["K"], w["V"], w["Omega"], w["qk_scale"], w["d"]
    qkv = torch.empty((2, 320, 2, 3, d), dtype=torch.bfloat16, device="cuda")          # packed [B, L, H, 3, d]
    for i, a in enumerate((Q, K, V)):
        qkv[:, :, :, i] = util.to_device(a, "bf16").permute(0, 2, 1, 3)
    Qd, Kd, Vd = (qkv[:, :, :, i].permute(0, 2, 1, 3) for i in range(3))
    theta = fs.fit_params("sderf", Qd, Kd, s, groups=2)
    th_host = util.to_host(theta).astype(np.float32)
    Y = fs.attention(theta, Qd, Kd, Vd, s, torch.from_numpy(Om).cuda(), causal=True, out_dtype=torch.float32)
    assert Y.dtype == torch.float32
    Yh = util.to_host(Y)
    for b in range(2):
        for h in range(2):
            ref = orc.attention(util.oracle_theta_from_vec(th_host[h], d), Om[h], Q[b, h], K[b, h], V[b, h], s, True)
            fro, row = util.attention_errors(Yh[b, h], ref, V[b, h].astype(np.float64))
            assert fro <= 2e-2 and row <= 8e-2, (b, h, fro, row)


def test_bf16_wide_path_shared_parameters_and_extreme_scales(fs):
    """One parameter set and one omega for all heads (groups = 1), key rows 20x larger than the rest late in the
    sequence and query rows 3x larger: shifts that are bounds over all 512 features keep the four partial walks on
    one scale and everything finite."""
    import torch
    w = synth.make("c5", B=1, H=2, L=576, seed=311)
    Q, K, V, s, d = w["Q"].copy(), w["K"].copy(), w["V"], w["qk_scale"], w["d"]
    K[0, 1, 400:404] *= 20.0
    Q[0, 0, 100:102] *= 3.0
    Q, K = synth.round_to_bf16(Q), synth.round_to_bf16(K)
    Om = w["Omega"][:1]
    vec = util.theta_vec_from_oracle(orc.fit_posrf(d))
    th = util.oracle_theta_from_vec(vec, d)
    Y = fs.attention(torch.from_numpy(vec[None]).cuda(), util.to_device(Q, "bf16"), util.to_device(K, "bf16"),
                     util.to_device(V, "bf16"), s, torch.from_numpy(Om).cuda(), causal=True, out_dtype=torch.float32)
    Yh = util.to_host(Y)
    assert np.isfinite(Yh).all()
    for h in range(2):
        ref = orc.attention(th, Om[0], Q[0, h], K[0, h], V[0, h], s, True)
        fro, row = util.attention_errors(Yh[0, h], ref, V[0, h].astype(np.float64))
        assert fro <= 2e-2 and row <= 8e-2, (h, fro, row)


@pytest.mark.parametrize("causal", [False, True])
def test_attention_with_block_orthogonal_omega(fs, causal):
    """Orthogonal random features only change omega: the library's host-side generator and the oracle's build the same
    omega from the same Gaussian draws, and the attention kernels run on it unchanged."""
    w = synth.make("c4", B=1, H=2, L=384, seed=91)
    rng = np.random.default_rng(92)
    G = rng.standard_normal(w["Omega"].shape).astype(np.float32)
    N = rng.standard_normal(w["Omega"].shape).astype(np.float32)
    Om_lib = fs.orthogonal_omega(G, N)
    Om_ref = np.stack([orc.orthogonal_omega(G[h].astype(np.float64), N[h].astype(np.float64)) for h in range(G.shape[0])])
    assert np.max(np.abs(Om_lib - Om_ref)) <= 2e-6 * np.max(np.abs(Om_ref))
    _check_attention(fs, w["Q"], w["K"], w["V"], Om_lib, w["qk_scale"], causal, "sderf", "bf16", chunk=64)


def test_bf16_path_f32_output_strided_inputs_and_shared_parameters(fs):
    import torch
    w = synth.make("c3", B=2, H=2, L=320)
    Q, K, V, Om, s, d = w["Q"], w["K"], w["V"], w["Omega"][:1], w["qk_scale"], w["d"]
    X = np.concatenate([s * Q[b, h] for b in range(2) for h in range(2)]).astype(np.float64)
    Yk = np.concatenate([s * K[b, h] for b in range(2) for h in range(2)]).astype(np.float64)
    vec = util.theta_vec_from_oracle(orc.fit_sderf(X, Yk))
    th = util.oracle_theta_from_vec(vec, d)
    qkv = torch.empty((2, 320, 2, 3, d), dtype=torch.bfloat16, device="cuda")          # packed [B, L, H, 3, d]
    for i, a in enumerate((Q, K, V)):
        qkv[:, :, :, i] = util.to_device(a, "bf16").permute(0, 2, 1, 3)
    Qd, Kd, Vd = (qkv[:, :, :, i].permute(0, 2, 1, 3) for i in range(3))
    for causal in (False, True):
        Y = fs.attention(torch.from_numpy(vec[None]).cuda(), Qd, Kd, Vd, s, torch.from_numpy(Om).cuda(), causal=causal,
                         out_dtype=torch.float32)
        assert Y.dtype == torch.float32
        Yh = util.to_host(Y)
        for b in range(2):
            for h in range(2):
                ref = orc.attention(th, Om[0], Q[b, h], K[b, h], V[b, h], s, causal)
                fro, row = util.attention_errors(Yh[b, h], ref, V[b, h].astype(np.float64))
                assert fro <= 2e-2 and row <= 8e-2, (causal, b, h, fro, row)


def test_bf16_path_extreme_scales_stay_finite(fs):
    """Key rows 30x larger than the rest (late in the sequence: their features vanish, the running shift must not
    follow them) and query rows 3x larger (their own shift grows) leave the result finite and within tolerance."""
    w = synth.make("c4", B=1, H=1, L=512, seed=5)
    Q, K = w["Q"].copy(), w["K"].copy()
    K[0, 0, 300:304] *= 30.0
    Q[0, 0, 100:102] *= 3.0
    Q, K = synth.round_to_bf16(Q), synth.round_to_bf16(K)
    _check_attention(fs, Q, K, w["V"], w["Omega"], w["qk_scale"], True, "posrf", "bf16")


@pytest.mark.parametrize("name,L,stretch", [("c4", 1024, 2.2), ("c5", 2048, 1.7)])
def test_bf16_causal_late_key_with_a_huge_bound_leaves_earlier_rows_intact(fs, name, L, stretch):
    """The key shift follows a Cauchy-Schwarz bound over all features (the bound less 120 binary orders); for a key
    whose norm matches the longest omega it is far above the key's actual features.  Omega is stretched here so that
    this shift exceeds 2^200 for one key late in the sequence (its own features stay negligible): on a shift common
    to the whole sequence the states of every earlier segment would leave the fp32 range.  The prefix states are kept on running shifts instead, so every
    row in a segment before the outlier's must stay within tolerance; the rows behind it are beyond the documented
    range of the shifts (their state is rescaled by the bound) and are only required to be finite."""
    import torch
    w = synth.make(name, B=1, H=1, L=L, seed=17)
    Q, K, V, s, d = w["Q"], w["K"].copy(), w["V"], w["qk_scale"], w["d"]
    Om = (stretch * w["Omega"]).astype(np.float32)
    longest = float(np.linalg.norm(Om[0], axis=1).max())
    late = L - 100
    K[0, 0, late] *= (longest / s) / np.linalg.norm(K[0, 0, late])
    K = synth.round_to_bf16(K)
    vec = util.theta_vec_from_oracle(orc.fit_posrf(d))
    th = util.oracle_theta_from_vec(vec, d)
    shift_log2 = (longest * longest / 2.0) / np.log(2.0) - 120.0
    assert shift_log2 > 200.0, shift_log2
    ws = torch.empty(fs.attention_workspace_bytes(1, 1, L, L, d, d, Om.shape[1], True, 1, 1), dtype=torch.uint8, device="cuda")
    Y = fs.attention(torch.from_numpy(vec[None]).cuda(), util.to_device(Q, "bf16"), util.to_device(K, "bf16"),
                     util.to_device(V, "bf16"), s, torch.from_numpy(Om).cuda(), causal=True, out_dtype=torch.float32,
                     workspace=ws)
    Yh = util.to_host(Y)[0, 0]
    assert np.isfinite(Yh).all()
    # whatever the rows behind the outlier lose is reported: the counter is the number of rows written as zeros
    assert fs.attention_flushed_rows(ws) == int((np.abs(Yh).max(axis=1) == 0).sum())
    ref = orc.attention(th, Om[0], Q[0, 0], K[0, 0], V[0, 0], s, True)
    safe = (late // 64) * 64           # segments and slots are whole chunks of 64 rows
    fro, row = util.attention_errors(Yh[:safe], ref[:safe], V[0, 0, :safe].astype(np.float64))
    assert fro <= 2e-2 and row <= 8e-2, (fro, row)


@pytest.mark.parametrize("name,L,causal,dtype", [("c4", 1000, True, "bf16"), ("c3", 1000, False, "bf16"),
                                                 ("c3", 200, False, "bf16"), ("c5", 1000, True, "bf16"),
                                                 ("c1", 300, True, "f32"), ("c1", 300, False, "f32")])
def test_rows_with_a_zero_normaliser_are_written_as_zeros_and_counted(fs, name, L, causal, dtype):
    """Denominator guard (Section 2.2).  On the bf16 kernels the shift of a query row is a Cauchy-Schwarz bound over
    all features: a query 40 times longer than the data's has every actual feature more than 2^126 below it, all of
    them flush, and the row's normaliser is exactly 0.  Such rows (four or five per (b, h), one of them in the ragged
    last chunk; the sequence of 200 rows runs in the kernel that takes a whole sequence per workgroup) must come out as zeros, the counter must report exactly their number, every other row must still agree
    with the oracle, and a call without such rows on the same workspace must put the counter back to 0.  The
    general-shape kernels shift a query row by its exact maximum, so no query can flush there: the count stays 0
    and all rows agree with the oracle."""
    import torch
    w = synth.make(name, B=1, H=2, L=L, seed=23)
    Q0, K, V, s, d, Om = w["Q"], w["K"], w["V"], w["qk_scale"], w["d"], w["Omega"]
    if dtype == "bf16":
        Q0, K, V = synth.round_to_bf16(Q0), synth.round_to_bf16(K), synth.round_to_bf16(V)
    Q = Q0.copy()
    rows = [r for r in (3, 64, 150, 257) if r < L - 2] + [L - 2]
    Q[:, :, rows] *= 120.0 if name == "c5" else 40.0
    if dtype == "bf16":
        Q = synth.round_to_bf16(Q)
    vec = util.theta_vec_from_oracle(orc.fit_posrf(d))
    th = util.oracle_theta_from_vec(vec, d)
    thd, Omd = torch.from_numpy(vec[None]).cuda(), torch.from_numpy(Om).cuda()
    B, H = Q.shape[:2]
    groups, og = 1, Om.shape[0]
    nbytes = fs.attention_workspace_bytes(B, H, L, L, d, V.shape[-1], Om.shape[-2], causal, groups, og)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    Kd, Vd = util.to_device(K, dtype), util.to_device(V, dtype)
    Y = fs.attention(thd, util.to_device(Q, dtype), Kd, Vd, s, Omd, causal=causal, out_dtype=torch.float32, workspace=ws)
    count = fs.attention_flushed_rows(ws)
    Yh = util.to_host(Y)
    assert np.isfinite(Yh).all()
    zero_rows = int((np.abs(Yh).max(axis=-1) == 0).sum())
    assert count == zero_rows, (count, zero_rows)
    on_fast_kernels = dtype == "bf16"
    assert count == (B * H * len(rows) if on_fast_kernels else 0), count
    keep = np.ones(L, bool)
    keep[rows] = False             # (the long rows themselves are outside the tolerances' range of exponents)
    if on_fast_kernels:
        assert (Yh[:, :, rows] == 0).all()
    tol = (2e-2, 8e-2) if dtype == "bf16" else (1e-4, 1e-3)
    for h in range(H):
        ref = orc.attention(th, Om[h % og], Q[0, h], K[0, h], V[0, h], s, causal)
        fro, row = util.attention_errors(Yh[0, h][keep], ref[keep], V[0, h].astype(np.float64))
        assert fro <= tol[0] and row <= tol[1], (h, fro, row)
    fs.attention(thd, util.to_device(Q0, dtype), Kd, Vd, s, Omd, causal=causal, out_dtype=torch.float32, workspace=ws)
    assert fs.attention_flushed_rows(ws) == 0


@pytest.mark.parametrize("causal", [False, True])
def test_bf16_path_ragged_tail_with_uniformly_large_keys(fs, causal):
    """Every key rescaled to the norm 21 (in the scaled space), so that the key shift (dominated by -|y|^2/2) is
    below -128 in the log2 domain while the Cauchy-Schwarz bounds stay inside the documented range, and a last chunk
    of 36 valid rows: the rows past the end must contribute exactly zero (not exp2(0 - shift) = inf times a zero
    value).  All keys have one norm because a causal row only sees the keys before it: keys of one chunk whose row
    terms differ by more than the fp32 exponent range cannot share a scale."""
    w = synth.make("c4", B=1, H=2, L=100, seed=91)
    K = w["K"].astype(np.float64)
    K *= (21.0 / w["qk_scale"]) / np.linalg.norm(K, axis=-1, keepdims=True)
    _check_attention(fs, w["Q"], synth.round_to_bf16(K.astype(np.float32)), w["V"], w["Omega"], w["qk_scale"], causal,
                     "posrf", "bf16", chunk=64)


@pytest.mark.parametrize("name,variant", [("c3", "sderf"), ("c4", "sderf"), ("c5", "sderf"), ("c3", "aderf"),
                                          ("c4", "aderf"), ("c5", "aderf"), ("c5", "saderf")])
def test_bf16_workloads_full_size_sampled_rows(fs, name, variant):
    """The full workload in the launch configuration the benchmark times; the oracle evaluates sampled output rows
    one by one from the definition (rows of K_hat, masked when causal): sequence start, segment and chunk
    boundaries, the end, and random rows, for three (b, h) pairs.  SDERF as the benchmark has it, and the families
    with a dense key-side quadratic form (row-term kernel over all keys, different projections for the two sides)."""
    import torch
    w = synth.make(name)
    B, H, L, d = w["B"], w["H"], w["L"], w["d"]
    s, causal = w["qk_scale"], w["causal"]
    Qd, Kd, Vd = (util.to_device(w[k], "bf16") for k in ("Q", "K", "V"))
    theta = fs.fit_params(variant, Qd, Kd, s, groups=H)
    Y = fs.attention(theta, Qd, Kd, Vd, s, torch.from_numpy(w["Omega"]).cuda(), causal=causal, chunk=w.get("chunk", 0))
    torch.cuda.synchronize()
    th_host = util.to_host(theta).astype(np.float32)
    rng = np.random.default_rng(9)
    fixed = [0, 1, 31, 32, 33, 63, 64, 65, 2047, 2048, 2049, L // 2 - 1, L // 2, L - 2, L - 1]
    for b, h in [(0, 0), (B - 1, H - 1), (B // 2, H // 2)]:
        rows = np.unique(np.concatenate([fixed, rng.integers(0, L, 52)]))
        th = util.oracle_theta_from_vec(th_host[h], d)
        ref = orc.attention_khat_definition(th, w["Omega"][h], w["Q"][b, h], w["K"][b, h], w["V"][b, h], s, causal, rows=rows)
        got = util.to_host(Y[b, h][torch.from_numpy(rows).cuda()])
        assert np.isfinite(got).all()
        fro, row = util.attention_errors(got, ref, w["V"][b, h].astype(np.float64))
        print(f"{name} {variant} full size (b={b}, h={h}): {len(rows)} sampled rows, frobenius {fro:.2e}, worst row {row:.2e}")
        assert fro <= 2e-2 and row <= 8e-2
    assert torch.isfinite(Y.float()).all().item()


@pytest.mark.parametrize("name,over,prepared,variant", [
    ("c1", {}, False, "sderf"), ("c4", dict(B=1, H=2, L=1216), False, "sderf"), ("c5", dict(B=1, H=2, L=832), False, "sderf"),
    ("c4", dict(B=1, H=2, L=1216), True, "sderf"), ("c2", {}, False, "sderf"),
    ("c4", dict(B=1, H=2, L=1216), True, "aderf"), ("c5", dict(B=1, H=2, L=832), False, "aderf"),
    ("c4", dict(B=1, H=1, L=4100), False, "sderf"), ("c3", dict(B=1, H=1, L=4100), True, "sderf"),
    ("c3", dict(B=1, H=2, L=200), False, "aderf")])
def test_attention_call_replays_from_a_hip_graph(fs, name, over, prepared, variant):
    """The entry point only enqueues kernels on the caller's stream (no synchronisation, no allocation, no memset
    nodes), so a caller may capture it: the graph is replayed three times, with eager work and synchronisations in
    between, and every replay must reproduce the eager result bit for bit (general path, both bf16 paths, the call
    on prepared projection constants, the kernel operator on its fp32 MFMA kernels, parameter sets with a dense
    quadratic form, which add the row-term kernel, a single sequence of 65 slots, whose slot reduction is the
    three-kernel form, and short sequences that take a workgroup each)."""
    import torch
    if name == "c2":
        _operator_graph_replay(fs)
        return
    w = synth.make(name, **over)
    dt = w.get("dtype", "f32")
    Q, K, V = (util.to_device(w[k], dt) for k in "QKV")
    Om, s, causal = torch.from_numpy(w["Omega"]).cuda(), w["qk_scale"], bool(w["causal"])
    theta = fs.fit_params(variant, Q, K, s, groups=w["H"])
    B, H, L, d = Q.shape
    ws = torch.empty(fs.attention_workspace_bytes(B, H, L, L, d, V.shape[-1], Om.shape[-2], causal, H, H), dtype=torch.uint8,
                     device="cuda")
    Y = torch.empty_like(V)

    prep = fs.attention_prepare(theta, Om, B, H, s) if prepared else None

    def call():
        if prepared:
            fs.attention_prepared(prep, theta, Q, K, V, s, Om, causal=causal, chunk=w.get("chunk", 0), out=Y, workspace=ws)
        else:
            fs.attention(theta, Q, K, V, s, Om, causal=causal, chunk=w.get("chunk", 0), out=Y, workspace=ws)

    _replay_and_compare(call, Y, name)


def _operator_graph_replay(fs):
    """favorsharp_kernel_matvec on the fp32 MFMA operator kernels (a reduced c2), captured and replayed."""
    import torch
    w = synth.make("c2", N=2048 + 37)
    X, C, Om = w["X"], w["C"], w["Omega"][0]
    Xd, Cd, Od = torch.from_numpy(X).cuda(), torch.from_numpy(C).cuda(), torch.from_numpy(Om).cuda()
    theta = fs.fit_params("sderf", Xd[None, None], Xd[None, None], 1.0, groups=1)
    N, d = X.shape
    ws = torch.empty(fs.kernel_matvec_workspace_bytes(N, N, d, Om.shape[0], C.shape[1]), dtype=torch.uint8, device="cuda")
    ref = fs.kernel_matvec(theta, Xd, Xd, 1.0, w["alpha"], Od, Cd, workspace=ws).clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fs.kernel_matvec(theta, Xd, Xd, 1.0, w["alpha"], Od, Cd, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        res = fs.kernel_matvec(theta, Xd, Xd, 1.0, w["alpha"], Od, Cd, workspace=ws)
    for rep in range(3):
        res.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(res, ref), rep
        _ = torch.randn(1 << 20, device="cuda").sum().item()


def _replay_and_compare(call, Y, name):
    import torch
    call()
    torch.cuda.synchronize()
    ref = Y.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):           # warm-up on a side stream, as graph capture asks for
        call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(3):
        Y.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, ref), (name, rep)
        _ = torch.randn(1 << 20, device="cuda").sum().item()


@pytest.mark.parametrize("name,over", [("c1", {}), ("c3", dict(B=2, H=2, L=704)), ("c4", dict(B=1, H=2, L=1216)),
                                       ("c5", dict(B=1, H=2, L=832)), ("c3", dict(B=2, H=2, L=128)),
                                       ("c4", dict(B=32, H=8, L=128))])
def test_attention_timed_gives_the_same_result_and_a_kernel_time(fs, name, over):
    """favorsharp_attention_timed: the two events bracket the main kernel (attached to its dispatch on the bf16 paths,
    recorded around it on the general path); the result is that of favorsharp_attention bit for bit, and the time
    between the events is positive and no longer than the whole call."""
    import ctypes
    import time
    import torch
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    w = synth.make(name, **over)
    dt = w.get("dtype", "f32")
    Q, K, V = (util.to_device(w[k], dt) for k in "QKV")
    Om, s, causal = torch.from_numpy(w["Omega"]).cuda(), w["qk_scale"], bool(w["causal"])
    theta = fs.fit_params("sderf", Q, K, s, groups=w["H"])
    ref = fs.attention(theta, Q, K, V, s, Om, causal=causal, chunk=w.get("chunk", 0))
    ev = [ctypes.c_void_p(), ctypes.c_void_p()]
    for e in ev:
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    Y = fs.attention(theta, Q, K, V, s, Om, causal=causal, chunk=w.get("chunk", 0), events=(ev[0].value, ev[1].value))
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    assert hip.hipEventSynchronize(ev[1]) == 0
    ms = ctypes.c_float()
    assert hip.hipEventElapsedTime(ctypes.byref(ms), ev[0], ev[1]) == 0
    for e in ev:
        hip.hipEventDestroy(e)
    assert torch.equal(Y, ref)
    assert 0.0 < ms.value <= wall_ms, (ms.value, wall_ms)


@pytest.mark.parametrize("name,over,variant", [("c4", dict(B=2, H=2, L=1216), "sderf"), ("c4", dict(B=1, H=2, L=333), "aderf"),
                                               ("c3", dict(B=2, H=2, L=712), "sderf"), ("c5", dict(B=1, H=2, L=832), "sderf"),
                                               ("c5", dict(B=1, H=2, L=200), "aderf"), ("c3", dict(B=2, H=2, L=200), "aderf"),
                                               ("c4", dict(B=32, H=8, L=100), "sderf")])
def test_prepared_constants_give_the_same_bits(fs, name, over, variant):
    """favorsharp_attention_prepare + favorsharp_attention_prepared against favorsharp_attention: the projection
    constants are the same numbers, so the outputs agree bit for bit; a second prepared call on other data of the
    same shapes reuses the buffer (dense C2: the key row terms are recomputed per call)."""
    import torch
    w = synth.make(name, **over)
    s, causal = w["qk_scale"], bool(w["causal"])
    theta = torch.from_numpy(_fit_theta_block(variant, w["Q"], w["K"], s, None)).cuda()
    Om = torch.from_numpy(w["Omega"]).cuda()
    prepared = fs.attention_prepare(theta, Om, w["B"], w["H"], s)
    assert prepared[1] == (1 if variant == "aderf" else 0)
    for seed in (w["seed"], w["seed"] + 7):
        w2 = synth.make(name, **dict(over, seed=seed))
        Qd, Kd, Vd = (util.to_device(w2[k], "bf16") for k in ("Q", "K", "V"))
        want = fs.attention(theta, Qd, Kd, Vd, s, Om, causal=causal, chunk=64 if causal else 0)
        got = fs.attention_prepared(prepared, theta, Qd, Kd, Vd, s, Om, causal=causal, chunk=64 if causal else 0)
        torch.cuda.synchronize()
        assert torch.isfinite(want.float()).all().item()
        assert torch.equal(got, want), (name, variant, seed)


@pytest.mark.parametrize("name", ["c3", "c4", "c5"])
def test_bf16_path_is_bitwise_reproducible(fs, name):
    """The kernels use no atomics and every LDS region is ordered by workgroup barriers, so two runs on the same
    inputs must agree bit for bit; a race in the producer / consumer hand-over or in the cross-workgroup scan would
    show up here (five repetitions at the benchmark's full size, other work in between)."""
    import torch
    w = synth.make(name)
    s, causal = w["qk_scale"], w["causal"]
    Qd, Kd, Vd = (util.to_device(w[k], "bf16") for k in ("Q", "K", "V"))
    Om = torch.from_numpy(w["Omega"]).cuda()
    theta = fs.fit_params("sderf", Qd, Kd, s, groups=w["H"])
    first = fs.attention(theta, Qd, Kd, Vd, s, Om, causal=causal, chunk=w.get("chunk", 0)).clone()
    for rep in range(5):
        scratch = torch.randn(1 << 22, device="cuda").sum().item()      # unrelated work in between
        again = fs.attention(theta, Qd, Kd, Vd, s, Om, causal=causal, chunk=w.get("chunk", 0))
        assert torch.equal(first.view(torch.int16), again.view(torch.int16)), (name, rep, scratch)
