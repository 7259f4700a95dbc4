"""favorsharp_attention_noalloc (the entry point for callers that cannot allocate: it runs on a scratch array the
library owns) against favorsharp_attention with a caller-owned workspace: same kernels, same launch plan, so the
outputs must agree bit for bit, on two calls in a row of which the second is smaller (the array then still holds the
first call's states)."""
import numpy as np
import pytest

from paper_2302_00787_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fs():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2302_00787_amd import binding
    binding.lib()
    return binding


def _case(fs, name, causal, **over):
    import torch
    w = synth.make(name, **over)
    dtype = "bf16" if w["dtype"] == "bf16" else "f32"
    Q, K, V = (fs.to_device(w[k], dtype) for k in ("Q", "K", "V"))
    Om = torch.from_numpy(w["Omega"]).cuda()
    theta = fs.fit_params("sderf", Q, K, w["qk_scale"], groups=w["H"])
    want = fs.attention(theta, Q, K, V, w["qk_scale"], Om, causal=causal, chunk=64 if causal else 0)
    got = torch.full_like(want, float("nan"))
    fs.attention_noalloc(theta, Q, K, V, w["qk_scale"], Om, got, causal=causal, chunk=64 if causal else 0)
    torch.cuda.synchronize()
    assert torch.isfinite(want.float()).all().item()
    assert torch.equal(got, want), (name, causal, over)


def test_noalloc_attention_two_calls_in_a_row_second_smaller(fs):
    _case(fs, "c4", True, B=2, H=4, L=4096)          # bf16 kernels, 256 segment states in the array
    _case(fs, "c4", True, B=1, H=2, L=1000)          # smaller, ragged: stale states beside the ones in use
    _case(fs, "c3", False, B=1, H=2, L=712)          # non-causal bf16 kernels
    _case(fs, "c1", False)                           # general-shape kernels, f32
    _case(fs, "c1", True)


def test_noalloc_attention_counts_zero_normalisers_in_its_own_array(fs):
    """The counter of rows with a zero normaliser is the first word of the scratch array for these calls: four query
    rows 40 times longer than the data's flush on the bf16 kernels and are counted; the next, ordinary call puts the
    counter back to 0.  Both calls must still agree bit for bit with the calls on a caller-owned workspace."""
    import torch
    w = synth.make("c4", B=1, H=2, L=500, seed=41)
    Q0, K, V = (fs.to_device(w[k], "bf16") for k in ("Q", "K", "V"))
    Om = torch.from_numpy(w["Omega"]).cuda()
    theta = fs.fit_params("sderf", Q0, K, w["qk_scale"], groups=2)
    Q = Q0.clone()
    Q[:, :, [5, 100, 333, 499]] *= 40.0
    for q, expect in ((Q, 8), (Q0, 0)):
        want = fs.attention(theta, q, K, V, w["qk_scale"], Om, causal=True, chunk=64)
        got = torch.full_like(want, float("nan"))
        fs.attention_noalloc(theta, q, K, V, w["qk_scale"], Om, got, causal=True, chunk=64)
        assert fs.attention_flushed_rows(None) == expect
        assert torch.equal(got, want)


def test_noalloc_attention_rejects_what_does_not_fit(fs):
    import torch
    w = synth.make("c5", B=1, H=1, L=64)
    Q = torch.zeros((1, 16, 65536, 128), dtype=torch.bfloat16, device="cuda")
    th = torch.zeros((16, fs.theta_floats(128)), device="cuda")
    Om = torch.zeros((16, 512, 128), device="cuda")
    with pytest.raises(fs.FavorSharpError) as err:
        fs.attention_noalloc(th, Q, Q, Q, w["qk_scale"], Om, torch.empty_like(Q), causal=True, chunk=64)
    assert err.value.status == 6
