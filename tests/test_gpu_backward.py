"""GPU parity of favorsharp_attention_backward against the oracle's attention_backward (non-causal and causal).

Tolerance: the kernels accumulate in fp32, the oracle in fp64; the gradients are sums of products of the same
quantities as the forward pass plus one more contraction, so they are held to the forward bar per (b, h): relative
Frobenius error <= 1e-4 times a factor 3 for the extra chain of contractions (f32 inputs) and the same for bf16
inputs on the general-shape kernels (the oracle sees the rounded inputs; all arithmetic of that path is fp32).  The
bf16 MFMA gradient kernels (bf16 rows, d = dv = 64, M = 256) round their operands, features, states and G1 rows to
bf16 and are held to the bf16 bar of the forward pass, 2e-2, whatever dtype the gradients are stored in.
Next to the Frobenius bound every gradient row is bounded: |dg_i| <= 4 tol max_j |g_ref,j| (a few wrong rows at a
slot or chunk boundary of a long tensor would pass the Frobenius bound alone)."""
import numpy as np
import pytest

from oracle import favorsharp_oracle as orc
from paper_2302_00787_amd import synth
from tests import util

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fs():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2302_00787_amd import binding
    binding.lib()
    return binding


def _theta_block(variant, Q, K, scale):
    vecs = []
    for h in range(Q.shape[1]):
        d = Q.shape[-1]
        th = orc.fit(variant, scale * Q[:, h].reshape(-1, d).astype(np.float64), scale * K[:, h].reshape(-1, d).astype(np.float64))
        vecs.append(util.theta_vec_from_oracle(th))
    return np.stack(vecs)


def _assert_grads(got, ref, tol, where, floor=0.0):
    """Frobenius and per-row bounds for (dQ, dK, dV) of one (b, h).  A gradient that is zero by construction (a
    single key: Y = V_0 whatever Q and K are) is measured against `floor`, a small multiple of the scale of the
    output gradient, instead of against 0."""
    errs = [util.gradient_errors(g, r, floor) for g, r in zip(got, ref)]
    assert max(e[0] for e in errs) <= tol, (where, "frobenius", errs)
    assert max(e[1] for e in errs) <= 4 * tol, (where, "row", errs)
    return max(e[0] for e in errs), max(e[1] for e in errs)


def _check_backward(fs, Q, K, V, dY, Omega, scale, variant, dtype, tol, grad_dtype=None, causal=False):
    import torch
    B, H, Lq, d = Q.shape
    theta = _theta_block(variant, Q, K, scale)
    gQ, gK, gV = fs.attention_backward(torch.from_numpy(theta).cuda(), util.to_device(Q, dtype), util.to_device(K, dtype),
                                       util.to_device(V, dtype), util.to_device(dY, dtype), scale,
                                       torch.from_numpy(Omega).cuda(), causal=causal, grad_dtype=grad_dtype)
    torch.cuda.synchronize()
    gQ, gK, gV = util.to_host(gQ), util.to_host(gK), util.to_host(gV)
    assert np.isfinite(gQ).all() and np.isfinite(gK).all() and np.isfinite(gV).all()
    worst = 0.0
    for b in range(B):
        for h in range(H):
            th = util.oracle_theta_from_vec(theta[h], d)
            rq, rk, rv = orc.attention_backward(th, Omega[h], Q[b, h], K[b, h], V[b, h], dY[b, h], scale, causal)
            floor = max(0.5 * tol, 1e-3) * float(np.linalg.norm(dY[b, h]))   # scale for a gradient that is zero by construction
            fro, _ = _assert_grads((gQ[b, h], gK[b, h], gV[b, h]), (rq, rk, rv), tol, (b, h), floor)
            worst = max(worst, fro)
    return worst


@pytest.mark.parametrize("variant", ["sderf", "aderf", "saderf", "gerf"])
def test_backward_f32_small_ragged_different_lengths(fs, variant):
    rng = np.random.default_rng(61)
    B, H, Lq, Lk, d, dv, M = 2, 2, 70, 45, 12, 20, 50      # row starts must be 16-byte aligned: d, dv multiples of 4
    Q = (rng.standard_normal((B, H, Lq, d)) * np.linspace(0.5, 1.2, d) + 0.1).astype(np.float32)
    K = (rng.standard_normal((B, H, Lk, d)) * np.linspace(1.1, 0.6, d) - 0.05).astype(np.float32)
    V = rng.standard_normal((B, H, Lk, dv)).astype(np.float32)
    dY = rng.standard_normal((B, H, Lq, dv)).astype(np.float32)
    Om = rng.standard_normal((H, M, d)).astype(np.float32)
    _check_backward(fs, Q, K, V, dY, Om, d ** -0.25, variant, "f32", 3e-4)


@pytest.mark.parametrize("L,M,d,dv", [(1, 1, 4, 4), (33, 16, 8, 4), (64, 200, 128, 128)])
def test_backward_degenerate_and_maximum_sizes(fs, L, M, d, dv):
    rng = np.random.default_rng(62)
    Q = (0.7 * rng.standard_normal((1, 1, L, d))).astype(np.float32)
    K = (0.7 * rng.standard_normal((1, 1, L, d))).astype(np.float32)
    V = rng.standard_normal((1, 1, L, dv)).astype(np.float32)
    dY = rng.standard_normal((1, 1, L, dv)).astype(np.float32)
    Om = rng.standard_normal((1, M, d)).astype(np.float32)
    _check_backward(fs, Q, K, V, dY, Om, d ** -0.25, "sderf" if L > 1 else "posrf", "f32", 3e-4)


def test_backward_c3_shape_bf16_inputs(fs):
    """The non-causal bf16 workload at its real d, M and statistics, shortened so the oracle finishes in seconds.
    This shape runs on the bf16 MFMA kernels (bf16 operands, fp32 accumulation): the bar is the bf16 one, 2e-2, for
    fp32 and for bf16 gradients.  The length is not a multiple of the tile sizes (ragged tails in every kernel)."""
    w = synth.make("c3", B=2, H=2, L=712)
    rng = np.random.default_rng(63)
    dY = synth.round_to_bf16(rng.standard_normal(w["V"].shape).astype(np.float32))
    import torch
    worst = _check_backward(fs, w["Q"], w["K"], w["V"], dY, w["Omega"], w["qk_scale"], "sderf", "bf16", 2e-2,
                            grad_dtype=torch.float32)
    assert worst > 0.0
    _check_backward(fs, w["Q"], w["K"], w["V"], dY, w["Omega"], w["qk_scale"], "sderf", "bf16", 2e-2)


@pytest.mark.parametrize("variant", ["aderf", "saderf", "gerf"])
def test_backward_bf16_path_other_families_and_lengths(fs, variant):
    """Dense C (ADERF: row terms from the precomputed table, dense derivative of the row term), diagonal C (SADERF)
    and the scalar family on the bf16 kernels, with different numbers of queries and keys."""
    import torch
    rng = np.random.default_rng(65)
    B, H, Lq, Lk, d, M = 1, 2, 200, 333, 64, 256
    sc = np.linspace(0.6, 1.1, d)
    Q = synth.round_to_bf16((rng.standard_normal((B, H, Lq, d)) * sc + 0.05).astype(np.float32))
    K = synth.round_to_bf16((rng.standard_normal((B, H, Lk, d)) * sc[::-1] - 0.05).astype(np.float32))
    V = synth.round_to_bf16(rng.standard_normal((B, H, Lk, d)).astype(np.float32))
    dY = synth.round_to_bf16(rng.standard_normal((B, H, Lq, d)).astype(np.float32))
    Om = rng.standard_normal((H, M, d)).astype(np.float32)
    _check_backward(fs, Q, K, V, dY, Om, d ** -0.25, variant, "bf16", 2e-2, grad_dtype=torch.float32)


@pytest.mark.parametrize("variant,B,H,Lq,Lk,f32", [("sderf", 1, 2, 128, 128, True), ("aderf", 1, 2, 100, 120, True),
                                                   ("saderf", 2, 2, 64, 190, False), ("gerf", 48, 8, 300, 200, False),
                                                   ("aderf", 64, 8, 70, 333, True), ("posrf", 1, 3, 1, 190, True)])
def test_backward_bf16_path_whole_sequences_per_workgroup(fs, variant, B, H, Lq, Lk, f32):
    """Non-causal calls with many sequences (B*H >= 384) or short ones (at most four chunks of queries and keys
    together) run the whole backward pass of a sequence in one workgroup, both states staying on chip: equal and
    different numbers of queries and keys, ragged tails, isotropic and dense key-side quadratic forms, fp32 output
    gradients into fp32 gradients and bf16 into bf16 (every seventh batch entry against the oracle)."""
    import torch
    rng = np.random.default_rng(67 + Lq + Lk)
    d, M = 64, 256
    sc = np.linspace(0.6, 1.1, d)
    Q = synth.round_to_bf16((rng.standard_normal((B, H, Lq, d)) * sc + 0.05).astype(np.float32))
    K = synth.round_to_bf16((rng.standard_normal((B, H, Lk, d)) * sc[::-1] - 0.05).astype(np.float32))
    V = synth.round_to_bf16(rng.standard_normal((B, H, Lk, d)).astype(np.float32))
    dY = rng.standard_normal((B, H, Lq, d)).astype(np.float32)
    if not f32:
        dY = synth.round_to_bf16(dY)
    Om = rng.standard_normal((H, M, d)).astype(np.float32)
    scale = d ** -0.25
    theta = _theta_block(variant, Q[::7], K[::7], scale)
    gQ, gK, gV = fs.attention_backward(torch.from_numpy(theta).cuda(), util.to_device(Q, "bf16"), util.to_device(K, "bf16"),
                                       util.to_device(V, "bf16"), util.to_device(dY, "f32" if f32 else "bf16"), scale,
                                       torch.from_numpy(Om).cuda(), causal=False,
                                       grad_dtype=torch.float32 if f32 else torch.bfloat16)
    torch.cuda.synchronize()
    gQ, gK, gV = util.to_host(gQ), util.to_host(gK), util.to_host(gV)
    assert np.isfinite(gQ).all() and np.isfinite(gK).all() and np.isfinite(gV).all()
    worst = (0.0, 0.0)
    for b in range(0, B, 7):
        for h in range(H):
            th = util.oracle_theta_from_vec(theta[h], d)
            ref = orc.attention_backward(th, Om[h], Q[b, h], K[b, h], V[b, h], dY[b, h], scale, False)
            floor = 1e-2 * float(np.linalg.norm(dY[b, h]))
            e = _assert_grads((gQ[b, h], gK[b, h], gV[b, h]), ref, 2e-2, (b, h), floor)
            worst = (max(worst[0], e[0]), max(worst[1], e[1]))
    print(f"backward, whole sequences, B={B} H={H} Lq={Lq} Lk={Lk} {variant}: worst frobenius {worst[0]:.2e}, "
          f"worst row {worst[1]:.2e}")


def test_backward_whole_sequences_per_workgroup_is_bitwise_reproducible(fs):
    """The one-workgroup backward pass reuses one LDS region for six loops and a transposition, ordered by workgroup
    barriers only, and reads back rows of G1 that the same workgroup wrote to memory: a missing barrier would show up
    as run-to-run differences (512 sequences of 200 rows, five repetitions, other work in between), and the forward
    call of the same shape must be reproducible too."""
    import torch
    torch.manual_seed(5)
    B, H, L, d, M = 64, 8, 200, 64, 256
    Q, K, V, dY = (torch.randn(B, H, L, d, device="cuda").to(torch.bfloat16) for _ in range(4))
    Om = torch.randn(H, M, d, device="cuda")
    s = d ** -0.25
    theta = fs.fit_params("aderf", Q, K, s, groups=H)
    first = [g.clone() for g in fs.attention_backward(theta, Q, K, V, dY, s, Om, causal=False)]
    y0 = fs.attention(theta, Q, K, V, s, Om, causal=False).clone()
    assert all(torch.isfinite(g.float()).all().item() for g in first)
    for rep in range(5):
        scratch = torch.randn(1 << 22, device="cuda").sum().item()
        again = fs.attention_backward(theta, Q, K, V, dY, s, Om, causal=False)
        for a, b in zip(first, again):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), (rep, scratch)
        assert torch.equal(y0.view(torch.int16), fs.attention(theta, Q, K, V, s, Om, causal=False).view(torch.int16))


def test_backward_value_gradients_sum_to_output_gradients_at_full_c3_size(fs):
    """At the full size of the non-causal workload the oracle cannot run; what holds at any size: the attention
    weights of a row sum to one, so sum_j dV_j = sum_i dY_i per (b, h); and sampled rows of dV against the oracle's
    weights W^T dY restricted to a subset of the queries' contribution is not available, so only the invariant is
    checked here."""
    import torch
    w = synth.make("c3")
    rng = np.random.default_rng(64)
    dY = synth.round_to_bf16(rng.standard_normal(w["V"].shape).astype(np.float32))
    theta = _theta_block("sderf", w["Q"][:1], w["K"][:1], w["qk_scale"])
    gQ, gK, gV = fs.attention_backward(torch.from_numpy(theta).cuda(), util.to_device(w["Q"], "bf16"),
                                       util.to_device(w["K"], "bf16"), util.to_device(w["V"], "bf16"),
                                       util.to_device(dY, "bf16"), w["qk_scale"], torch.from_numpy(w["Omega"]).cuda(),
                                       grad_dtype=torch.float32)
    torch.cuda.synchronize()
    gV = util.to_host(gV).astype(np.float64)
    assert np.isfinite(util.to_host(gQ)).all() and np.isfinite(util.to_host(gK)).all()
    want = dY.astype(np.float64).sum(axis=2)
    got = gV.sum(axis=2)
    scale = np.abs(dY).astype(np.float64).sum(axis=2).max()
    # bf16 kernels: every dV row carries a relative rounding error of about 2^-9; the column sums of 4096 of them
    # against the sum of absolute values
    assert np.abs(got - want).max() <= 1e-3 * scale


@pytest.mark.parametrize("variant", ["sderf", "aderf", "saderf", "gerf"])
def test_backward_causal_f32_small_ragged(fs, variant):
    """Causal variant: several segments, several 32-row steps per segment and a ragged tail."""
    rng = np.random.default_rng(71)
    B, H, L, d, dv, M = 2, 2, 333, 12, 20, 50
    Q = (rng.standard_normal((B, H, L, d)) * np.linspace(0.5, 1.2, d) + 0.1).astype(np.float32)
    K = (rng.standard_normal((B, H, L, d)) * np.linspace(1.1, 0.6, d) - 0.05).astype(np.float32)
    V = rng.standard_normal((B, H, L, dv)).astype(np.float32)
    dY = rng.standard_normal((B, H, L, dv)).astype(np.float32)
    Om = rng.standard_normal((H, M, d)).astype(np.float32)
    _check_backward(fs, Q, K, V, dY, Om, d ** -0.25, variant, "f32", 3e-4, causal=True)


@pytest.mark.parametrize("L,M,d,dv", [(1, 1, 4, 4), (33, 16, 8, 4), (64, 200, 128, 128)])
def test_backward_causal_degenerate_and_maximum_sizes(fs, L, M, d, dv):
    rng = np.random.default_rng(72)
    Q = (0.7 * rng.standard_normal((1, 1, L, d))).astype(np.float32)
    K = (0.7 * rng.standard_normal((1, 1, L, d))).astype(np.float32)
    V = rng.standard_normal((1, 1, L, dv)).astype(np.float32)
    dY = rng.standard_normal((1, 1, L, dv)).astype(np.float32)
    Om = rng.standard_normal((1, M, d)).astype(np.float32)
    _check_backward(fs, Q, K, V, dY, Om, d ** -0.25, "sderf" if L > 1 else "posrf", "f32", 3e-4, causal=True)


def test_backward_causal_c4_shape_bf16_inputs(fs):
    """The causal bf16 workload at its real d, M and statistics, shortened so the oracle finishes in seconds: bf16
    MFMA kernels, bar 2e-2.  Several slots per sequence, several chunks per slot and a ragged tail."""
    import torch
    w = synth.make("c4", B=1, H=2, L=1216)
    rng = np.random.default_rng(73)
    dY = synth.round_to_bf16(rng.standard_normal(w["V"].shape).astype(np.float32))
    _check_backward(fs, w["Q"], w["K"], w["V"], dY, w["Omega"], w["qk_scale"], "sderf", "bf16", 2e-2,
                    grad_dtype=torch.float32, causal=True)
    _check_backward(fs, w["Q"], w["K"], w["V"], dY, w["Omega"], w["qk_scale"], "sderf", "bf16", 2e-2, causal=True)


@pytest.mark.parametrize("variant,L", [("aderf", 333), ("saderf", 64), ("gerf", 100)])
def test_backward_causal_bf16_path_other_families_and_lengths(fs, variant, L):
    import torch
    rng = np.random.default_rng(75)
    B, H, d, M = 1, 2, 64, 256
    sc = np.linspace(0.6, 1.1, d)
    Q = synth.round_to_bf16((rng.standard_normal((B, H, L, d)) * sc + 0.05).astype(np.float32))
    K = synth.round_to_bf16((rng.standard_normal((B, H, L, d)) * sc[::-1] - 0.05).astype(np.float32))
    V = synth.round_to_bf16(rng.standard_normal((B, H, L, d)).astype(np.float32))
    dY = synth.round_to_bf16(rng.standard_normal((B, H, L, d)).astype(np.float32))
    Om = rng.standard_normal((H, M, d)).astype(np.float32)
    _check_backward(fs, Q, K, V, dY, Om, d ** -0.25, variant, "bf16", 2e-2, grad_dtype=torch.float32, causal=True)


@pytest.mark.parametrize("variant,L", [("sderf", 200), ("aderf", 128), ("gerf", 333)])
def test_backward_causal_one_slot_per_sequence(fs, variant, L):
    """Causal calls with 256 sequences or more give every sequence one slot: no prefix and no suffix states exist, the
    walks start from a block of zeros and only the key shift of each sequence is computed beforehand (the workspace
    is filled with NaN bit patterns first: nothing that was not written may be read; every fifth batch entry against
    the oracle)."""
    import torch
    rng = np.random.default_rng(79 + L)
    B, H, d, M = 32, 8, 64, 256
    sc = np.linspace(0.6, 1.1, d)
    Q = synth.round_to_bf16((rng.standard_normal((B, H, L, d)) * sc + 0.05).astype(np.float32))
    K = synth.round_to_bf16((rng.standard_normal((B, H, L, d)) * sc[::-1] - 0.05).astype(np.float32))
    V = synth.round_to_bf16(rng.standard_normal((B, H, L, d)).astype(np.float32))
    dY = synth.round_to_bf16(rng.standard_normal((B, H, L, d)).astype(np.float32))
    Om = rng.standard_normal((H, M, d)).astype(np.float32)
    scale = d ** -0.25
    theta = _theta_block(variant, Q[::5], K[::5], scale)
    ws = torch.full((fs.attention_backward_workspace_bytes(B, H, L, L, d, d, M, True, H, H),), 0xFF, dtype=torch.uint8,
                    device="cuda")
    grads = fs.attention_backward(torch.from_numpy(theta).cuda(), util.to_device(Q, "bf16"), util.to_device(K, "bf16"),
                                  util.to_device(V, "bf16"), util.to_device(dY, "bf16"), scale, torch.from_numpy(Om).cuda(),
                                  causal=True, grad_dtype=torch.float32, workspace=ws)
    assert fs.attention_flushed_rows(ws) == 0
    gQ, gK, gV = (util.to_host(g) for g in grads)
    assert np.isfinite(gQ).all() and np.isfinite(gK).all() and np.isfinite(gV).all()
    worst = (0.0, 0.0)
    for b in range(0, B, 5):
        for h in range(H):
            th = util.oracle_theta_from_vec(theta[h], d)
            ref = orc.attention_backward(th, Om[h], Q[b, h], K[b, h], V[b, h], dY[b, h], scale, True)
            e = _assert_grads((gQ[b, h], gK[b, h], gV[b, h]), ref, 2e-2, (b, h))
            worst = (max(worst[0], e[0]), max(worst[1], e[1]))
    print(f"backward, causal, 256 sequences of {L} {variant}: worst frobenius {worst[0]:.2e}, worst row {worst[1]:.2e}")


@pytest.mark.parametrize("causal", [False, True])
def test_backward_bf16_path_single_token(fs, causal):
    """One query and one key: Y = V_0 whatever Q and K are, so dQ = dK = 0 and dV = dY.  On the bf16 kernels the zero
    is a cancellation of terms of size |dY| |V| that were rounded to bf16 on the way, so it is held to 2e-2 of that
    size; dV to the bf16 bar."""
    import torch
    rng = np.random.default_rng(76)
    d, M = 64, 256
    Q, K, V, dY = (synth.round_to_bf16(rng.standard_normal((1, 2, 1, d)).astype(np.float32)) for _ in range(4))
    Om = rng.standard_normal((2, M, d)).astype(np.float32)
    theta = np.stack([util.theta_vec_from_oracle(orc.fit_posrf(d))] * 2)
    gQ, gK, gV = fs.attention_backward(torch.from_numpy(theta).cuda(), util.to_device(Q, "bf16"), util.to_device(K, "bf16"),
                                       util.to_device(V, "bf16"), util.to_device(dY, "bf16"), d ** -0.25,
                                       torch.from_numpy(Om).cuda(), causal=causal, grad_dtype=torch.float32)
    torch.cuda.synchronize()
    gQ, gK, gV = util.to_host(gQ), util.to_host(gK), util.to_host(gV)
    for h in range(2):
        size = float(np.linalg.norm(dY[0, h]) * np.linalg.norm(V[0, h]))
        assert np.linalg.norm(gQ[0, h]) <= 2e-2 * size and np.linalg.norm(gK[0, h]) <= 2e-2 * size
        assert np.linalg.norm(gV[0, h] - dY[0, h]) <= 2e-2 * np.linalg.norm(dY[0, h])


@pytest.mark.parametrize("causal", [False, True])
def test_backward_bf16_path_strided_inputs_and_shared_parameters(fs, causal):
    """Q, K, V packed as [B, L, H, 3, d] and dY as [B, L, H, d] (row strides 3 H d and H d), one parameter set and
    one omega for all heads, two batches: strides, batch offsets and parameter groups on the bf16 kernels."""
    import torch
    w = synth.make("c4", B=2, H=2, L=448, seed=83)
    Q, K, V, s, d = w["Q"], w["K"], w["V"], w["qk_scale"], w["d"]
    Om = w["Omega"][:1]
    rng = np.random.default_rng(84)
    dY = synth.round_to_bf16(rng.standard_normal(V.shape).astype(np.float32))
    X = np.concatenate([s * Q[b, h] for b in range(2) for h in range(2)]).astype(np.float64)
    Yk = np.concatenate([s * K[b, h] for b in range(2) for h in range(2)]).astype(np.float64)
    vec = util.theta_vec_from_oracle(orc.fit_sderf(X, Yk))
    th = util.oracle_theta_from_vec(vec, d)
    qkv = torch.empty((2, 448, 2, 3, d), dtype=torch.bfloat16, device="cuda")
    for i, a in enumerate((Q, K, V)):
        qkv[:, :, :, i] = util.to_device(a, "bf16").permute(0, 2, 1, 3)
    Qd, Kd, Vd = (qkv[:, :, :, i].permute(0, 2, 1, 3) for i in range(3))
    dYd = util.to_device(dY, "bf16").permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    gQ, gK, gV = fs.attention_backward(torch.from_numpy(vec[None]).cuda(), Qd, Kd, Vd, dYd, s, torch.from_numpy(Om).cuda(),
                                       causal=causal, grad_dtype=torch.float32)
    torch.cuda.synchronize()
    gQ, gK, gV = util.to_host(gQ), util.to_host(gK), util.to_host(gV)
    for b in range(2):
        for h in range(2):
            rq, rk, rv = orc.attention_backward(th, Om[0], Q[b, h], K[b, h], V[b, h], dY[b, h], s, causal)
            _assert_grads((gQ[b, h], gK[b, h], gV[b, h]), (rq, rk, rv), 2e-2, (b, h))


@pytest.mark.parametrize("name", ["c3", "c4"])
def test_backward_bf16_path_is_bitwise_reproducible(fs, name):
    """No atomics, every LDS region ordered by workgroup barriers: repeated calls at the benchmark's full size must
    agree bit for bit; a race in a producer / consumer hand-over or between the walks of a call would show up here."""
    import torch
    w = synth.make(name)
    s, causal = w["qk_scale"], bool(w["causal"])
    Qd, Kd, Vd = (util.to_device(w[k], "bf16") for k in ("Q", "K", "V"))
    rng = np.random.default_rng(85)
    dYd = util.to_device(synth.round_to_bf16(rng.standard_normal(w["V"].shape).astype(np.float32)), "bf16")
    Om = torch.from_numpy(w["Omega"]).cuda()
    theta = fs.fit_params("sderf", Qd, Kd, s, groups=w["H"])
    first = [g.clone() for g in fs.attention_backward(theta, Qd, Kd, Vd, dYd, s, Om, causal=causal)]
    for rep in range(4):
        scratch = torch.randn(1 << 22, device="cuda").sum().item()      # unrelated work in between
        again = fs.attention_backward(theta, Qd, Kd, Vd, dYd, s, Om, causal=causal)
        torch.cuda.synchronize()
        for a, b in zip(first, again):
            assert torch.equal(a, b), (name, rep)
    assert all(torch.isfinite(g.float()).all().item() for g in first)


@pytest.mark.parametrize("name", ["c3", "c4"])
def test_backward_full_size_against_the_oracle_on_two_heads(fs, name):
    """The bf16 workloads at their full size, in the launch configuration the benchmark times (c4: 32 sequences of
    16384 tokens, eight slots of 32 chunks each); the oracle evaluates two whole (b, h) sequences (first and last)
    and every gradient row of them is compared."""
    import torch
    w = synth.make(name)
    B, H, L, d = w["B"], w["H"], w["L"], w["d"]
    s, causal = w["qk_scale"], bool(w["causal"])
    rng = np.random.default_rng(86)
    dY = synth.round_to_bf16(rng.standard_normal(w["V"].shape).astype(np.float32))
    Qd, Kd, Vd, dYd = (util.to_device(a, "bf16") for a in (w["Q"], w["K"], w["V"], dY))
    Om = torch.from_numpy(w["Omega"]).cuda()
    theta = fs.fit_params("sderf", Qd, Kd, s, groups=H)
    gQ, gK, gV = fs.attention_backward(theta, Qd, Kd, Vd, dYd, s, Om, causal=causal, grad_dtype=torch.float32)
    torch.cuda.synchronize()
    th_host = util.to_host(theta).astype(np.float32)
    for b, h in [(0, 0), (B - 1, H - 1)]:
        th = util.oracle_theta_from_vec(th_host[h], d)
        rq, rk, rv = orc.attention_backward(th, w["Omega"][h], w["Q"][b, h], w["K"][b, h], w["V"][b, h], dY[b, h], s, causal)
        fro, row = _assert_grads(tuple(util.to_host(g[b, h]) for g in (gQ, gK, gV)), (rq, rk, rv), 2e-2, (b, h))
        print(f"{name} backward full size (b={b}, h={h}): worst relative Frobenius error {fro:.2e}, worst row error {row:.2e}")


@pytest.mark.parametrize("causal", [False, True])
def test_forward_and_backward_bf16_path_one_parameter_set_per_sequence(fs, causal):
    """groups = omega_groups = B*H: every (b, h) sequence has its own fitted parameters and its own omega."""
    import torch
    w = synth.make("c4", B=2, H=2, L=320, seed=87)
    Q, K, V, s, d, M = w["Q"], w["K"], w["V"], w["qk_scale"], w["d"], w["M"]
    rng = np.random.default_rng(88)
    dY = synth.round_to_bf16(rng.standard_normal(V.shape).astype(np.float32))
    Om = rng.standard_normal((4, M, d)).astype(np.float32)
    ths = [orc.fit_sderf(s * Q[b, h].astype(np.float64), s * K[b, h].astype(np.float64)) for b in range(2) for h in range(2)]
    theta = torch.from_numpy(np.stack([util.theta_vec_from_oracle(t) for t in ths])).cuda()
    Qd, Kd, Vd, dYd = (util.to_device(a, "bf16") for a in (Q, K, V, dY))
    Y = util.to_host(fs.attention(theta, Qd, Kd, Vd, s, torch.from_numpy(Om).cuda(), causal=causal, out_dtype=torch.float32))
    gQ, gK, gV = (util.to_host(g) for g in fs.attention_backward(theta, Qd, Kd, Vd, dYd, s, torch.from_numpy(Om).cuda(),
                                                                  causal=causal, grad_dtype=torch.float32))
    for b in range(2):
        for h in range(2):
            g = 2 * b + h
            th = util.oracle_theta_from_vec(util.theta_vec_from_oracle(ths[g]), d)
            ref = orc.attention(th, Om[g], Q[b, h], K[b, h], V[b, h], s, causal)
            fro, row = util.attention_errors(Y[b, h], ref, V[b, h].astype(np.float64))
            assert fro <= 2e-2 and row <= 8e-2, (b, h, fro, row)
            rq, rk, rv = orc.attention_backward(th, Om[g], Q[b, h], K[b, h], V[b, h], dY[b, h], s, causal)
            _assert_grads((gQ[b, h], gK[b, h], gV[b, h]), (rq, rk, rv), 2e-2, (b, h))


@pytest.mark.parametrize("causal", [False, True])
def test_backward_gradient_tensors_with_huge_row_strides(fs, causal):
    """Gradient tensors whose row stride does not fit the 32-bit offsets of the bf16 kernels (2^23 elements and
    more): the call must take the general-shape kernels instead of wrapping offsets, and stay correct."""
    import torch
    w = synth.make("c4", B=1, H=1, L=40, seed=93)
    Q, K, V, s, d = w["Q"], w["K"], w["V"], w["qk_scale"], w["d"]
    rng = np.random.default_rng(94)
    dY = synth.round_to_bf16(rng.standard_normal(V.shape).astype(np.float32))
    vec = util.theta_vec_from_oracle(orc.fit_sderf(s * Q[0, 0].astype(np.float64), s * K[0, 0].astype(np.float64)))
    th = util.oracle_theta_from_vec(vec, d)
    big = 1 << 23
    wide = [torch.zeros((1, 1, 40, big), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    gK = wide[0][..., :d]
    dYd = wide[1][..., :d]
    dYd.copy_(util.to_device(dY, "bf16"))
    gQ = torch.empty((1, 1, 40, d), dtype=torch.bfloat16, device="cuda")
    gV = torch.empty((1, 1, 40, d), dtype=torch.bfloat16, device="cuda")
    fs.attention_backward(torch.from_numpy(vec[None]).cuda(), util.to_device(Q, "bf16"), util.to_device(K, "bf16"),
                          util.to_device(V, "bf16"), dYd, s, torch.from_numpy(w["Omega"]).cuda(), causal=causal,
                          grads=(gQ, gK, gV))
    torch.cuda.synchronize()
    ref = orc.attention_backward(th, w["Omega"][0], Q[0, 0], K[0, 0], V[0, 0], dY[0, 0], s, causal)
    _assert_grads(tuple(util.to_host(g[0, 0]) for g in (gQ, gK, gV)), ref, 2e-2, "huge strides")
    assert float(wide[0][..., d:d + 64].abs().max()) == 0.0          # nothing written beside the rows


@pytest.mark.parametrize("causal,L", [(False, 300), (True, 300), (False, 120)])
def test_backward_counts_rows_with_a_zero_normaliser_and_drops_their_terms(fs, causal, L):
    """Denominator guard in the backward pass (bf16 gradient kernels): a query row whose features all flush (40
    times the data's length: its Cauchy-Schwarz shift is more than 2^126 above every actual feature) has the
    normaliser 0, so its G1 row is 0: it gets a zero dQ row and adds nothing to dK and dV, which is what the oracle
    computes when that row of dY is zero.  The counter in the workspace's first word must report exactly these
    rows, and 0 again after a call without them (120 rows: the kernel that takes a whole sequence per workgroup)."""
    import torch
    w = synth.make("c4", B=1, H=2, L=L, seed=29)
    Q0, K, V, s, d, Om = w["Q"], w["K"], w["V"], w["qk_scale"], w["d"], w["Omega"]
    rows = [2, 64, min(200, L - 20), L - 1]
    Q = Q0.copy()
    Q[:, :, rows] *= 40.0
    Q = synth.round_to_bf16(Q)
    rng = np.random.default_rng(30)
    dY = synth.round_to_bf16(rng.standard_normal(V.shape).astype(np.float32))
    dY_seen = dY.copy()
    dY_seen[:, :, rows] = 0.0
    vec = util.theta_vec_from_oracle(orc.fit_posrf(d))
    th = util.oracle_theta_from_vec(vec, d)
    thd, Omd = torch.from_numpy(vec[None]).cuda(), torch.from_numpy(Om).cuda()
    nbytes = fs.attention_backward_workspace_bytes(1, 2, L, L, d, d, Om.shape[1], causal, 1, Om.shape[0])
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    Kd, Vd, dYd = (util.to_device(t, "bf16") for t in (K, V, dY))
    grads = fs.attention_backward(thd, util.to_device(Q, "bf16"), Kd, Vd, dYd, s, Omd, causal=causal, workspace=ws)
    assert fs.attention_flushed_rows(ws) == 2 * len(rows)
    gQ, gK, gV = (util.to_host(g) for g in grads)
    assert np.isfinite(gQ).all() and np.isfinite(gK).all() and np.isfinite(gV).all()
    assert (gQ[:, :, rows] == 0).all()
    for h in range(2):
        ref = orc.attention_backward(th, Om[h], Q[0, h], K[0, h], V[0, h], dY_seen[0, h], s, causal)
        _assert_grads((gQ[0, h], gK[0, h], gV[0, h]), ref, 2e-2, h)
    fs.attention_backward(thd, util.to_device(Q0, "bf16"), Kd, Vd, dYd, s, Omd, causal=causal, workspace=ws)
    assert fs.attention_flushed_rows(ws) == 0


@pytest.mark.parametrize("causal", [False, True])
def test_backward_bf16_kernels_take_an_fp32_output_gradient(fs, causal):
    """dY in fp32 next to bf16 Q, K, V (a caller that asked for an fp32 Y): the bf16 gradient kernels read it as it is
    (it stays fp32 until the G1 rows are rounded), so the result must agree with the oracle on the UNROUNDED dY to the
    bf16 bar, and must not be the result for the bf16-rounded dY bit for bit."""
    import torch
    w = synth.make("c4", B=1, H=2, L=333, seed=97)
    Q, K, V, s, d, Om = w["Q"], w["K"], w["V"], w["qk_scale"], w["d"], w["Omega"]
    rng = np.random.default_rng(98)
    dY = rng.standard_normal(V.shape).astype(np.float32)
    theta = _theta_block("sderf", Q, K, s)
    thd, Omd = torch.from_numpy(theta).cuda(), torch.from_numpy(Om).cuda()
    Qd, Kd, Vd = (util.to_device(t, "bf16") for t in (Q, K, V))
    got = fs.attention_backward(thd, Qd, Kd, Vd, util.to_device(dY, "f32"), s, Omd, causal=causal, grad_dtype=torch.float32)
    got = [util.to_host(g) for g in got]
    rounded = fs.attention_backward(thd, Qd, Kd, Vd, util.to_device(synth.round_to_bf16(dY), "bf16"), s, Omd, causal=causal,
                                    grad_dtype=torch.float32)
    assert any(not np.array_equal(a, util.to_host(b)) for a, b in zip(got, rounded))
    for h in range(2):
        th = util.oracle_theta_from_vec(theta[h], d)
        ref = orc.attention_backward(th, Om[h], Q[0, h], K[0, h], V[0, h], dY[0, h], s, causal)
        _assert_grads(tuple(g[0, h] for g in got), ref, 2e-2, h)


@pytest.mark.parametrize("name,over,variant", [("c3", dict(B=2, H=2, L=712), "sderf"), ("c4", dict(B=1, H=2, L=1216), "aderf"),
                                               ("c3", dict(B=2, H=2, L=128), "aderf"), ("c4", dict(B=32, H=8, L=100), "sderf"),
                                               ("c5", dict(B=1, H=2, L=96), "sderf")])
def test_backward_on_prepared_constants_gives_the_same_bits(fs, name, over, variant):
    """favorsharp_attention_backward_prepared against favorsharp_attention_backward: the projection constants are the
    same numbers, so the gradients agree bit for bit (separate kernels, the one-workgroup form, the causal form with
    and without slots; parameter sets with a dense C2 still compute their key row terms per call; the d = 128 shape
    runs on kernels that keep no constants and must simply ignore the buffer)."""
    import torch
    w = synth.make(name, **over)
    s, causal = w["qk_scale"], bool(w["causal"])
    Qd, Kd, Vd = (util.to_device(w[k], "bf16") for k in ("Q", "K", "V"))
    dY = torch.randn(Vd.shape, device="cuda", generator=torch.Generator(device="cuda").manual_seed(3)).to(torch.bfloat16)
    Om = torch.from_numpy(w["Omega"]).cuda()
    theta = fs.fit_params(variant, Qd, Kd, s, groups=w["H"])
    prepared = fs.attention_prepare(theta, Om, w["B"], w["H"], s)
    want = fs.attention_backward(theta, Qd, Kd, Vd, dY, s, Om, causal=causal)
    got = fs.attention_backward(theta, Qd, Kd, Vd, dY, s, Om, causal=causal, prepared=prepared)
    torch.cuda.synchronize()
    for a, b in zip(want, got):
        assert torch.isfinite(a.float()).all().item()
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), (name, variant)


@pytest.mark.parametrize("name,over,prepared", [("c3", dict(B=2, H=2, L=712), False), ("c4", dict(B=1, H=2, L=1216), True),
                                                ("c3", dict(B=2, H=2, L=128), True), ("c4", dict(B=32, H=8, L=100), False),
                                                ("c1", {}, False)])
def test_backward_call_replays_from_a_hip_graph(fs, name, over, prepared):
    """The backward entry points only enqueue kernels on the caller's stream (no synchronisation, no allocation, no
    memset nodes): captured in a HIP graph and replayed three times, with eager work and synchronisations in between,
    every replay reproduces the eager gradients bit for bit (separate non-causal kernels, the causal kernels with
    slots, the one-workgroup form, the causal form with one slot per sequence, the general-shape kernels)."""
    import torch
    w = synth.make(name, **over)
    dt = w.get("dtype", "f32")
    Q, K, V = (util.to_device(w[k], dt) for k in "QKV")
    dY = torch.randn(V.shape, device="cuda", generator=torch.Generator(device="cuda").manual_seed(7)).to(V.dtype)
    Om, s, causal = torch.from_numpy(w["Omega"]).cuda(), w["qk_scale"], bool(w["causal"])
    theta = fs.fit_params("aderf" if name == "c3" else "sderf", Q, K, s, groups=w["H"])
    B, H, L, d = Q.shape
    ws = torch.empty(fs.attention_backward_workspace_bytes(B, H, L, L, d, V.shape[-1], Om.shape[-2], causal, H, H),
                     dtype=torch.uint8, device="cuda")
    grads = tuple(torch.empty_like(t) for t in (Q, K, V))
    prep = fs.attention_prepare(theta, Om, B, H, s) if prepared else None

    def call():
        fs.attention_backward(theta, Q, K, V, dY, s, Om, causal=causal, workspace=ws, grads=grads, prepared=prep)

    call()
    torch.cuda.synchronize()
    ref = [g.clone() for g in grads]
    assert all(torch.isfinite(g.float()).all().item() for g in ref)
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
        for g in grads:
            g.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for g, r in zip(grads, ref):
            assert torch.equal(g, r), (name, rep)
        _ = torch.randn(1 << 20, device="cuda").sum().item()


def test_backward_error_paths(fs):
    import torch
    Q = torch.zeros((1, 1, 8, 8), device="cuda")
    K = torch.zeros((1, 1, 12, 8), device="cuda")
    th = torch.from_numpy(util.theta_vec_from_oracle(orc.fit_posrf(8))[None]).cuda()
    Om = torch.zeros((1, 4, 8), device="cuda")
    with pytest.raises(fs.FavorSharpError) as err:          # causal needs as many queries as keys
        fs.attention_backward(th, Q, K, K, Q, 1.0, Om, causal=True)
    assert err.value.status in (2, 4)       # unsupported (the workspace query already says so with 0 bytes)
