"""The C-ABI library loads, exports every symbol the header declares, and its pure-host entry points answer.
No kernel is launched here (there is no GPU on the build machine)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "favorsharp.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2302_00787_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2302_00787_amd import build
        build.build(verbose=False)
    return binding.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(favorsharp_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"favorsharp_fit_params", "favorsharp_features", "favorsharp_attention",
            "favorsharp_kernel_matvec"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_host_only_queries(lib):
    assert lib.favorsharp_theta_floats(64) == 8 + 64 + 4 * 64 * 64
    assert lib.favorsharp_theta_floats(0) == 0
    assert lib.favorsharp_status_string(0) == b"ok"
    assert b"workspace" in lib.favorsharp_status_string(4)
    assert b"gfx950" in lib.favorsharp_version()
    assert lib.favorsharp_attention_workspace_bytes(4, 8, 16384, 16384, 64, 64, 256, 1, 8, 8) > 0
    assert lib.favorsharp_attention_workspace_bytes(4, 8, 16384, 16384, 129, 64, 256, 1, 8, 8) == 0     # d > 128
    assert lib.favorsharp_attention_workspace_bytes(4, 8, 16384, 16384, 64, 64, 256, 1, 3, 8) == 0      # bad groups
    # the sequences are a grid dimension of the kernels: at most 65535 of them
    assert lib.favorsharp_attention_workspace_bytes(65535, 1, 64, 64, 64, 64, 256, 0, 1, 1) > 0
    assert lib.favorsharp_attention_workspace_bytes(8192, 8, 64, 64, 64, 64, 256, 0, 1, 1) == 0
    assert lib.favorsharp_attention_backward_workspace_bytes(8192, 8, 64, 64, 64, 64, 256, 0, 1, 1) == 0
    assert lib.favorsharp_fit_workspace_bytes(8192, 8, 64, 64, 64, 1) == 0
    assert lib.favorsharp_kernel_matvec_workspace_bytes(16384, 16384, 32, 512, 8) > 0
    # room for both sides' projection matrices (fp32 and bf16 copies) and biases
    assert lib.favorsharp_features_workspace_bytes(100, 16, 64) >= 2 * 64 * 16 * (4 + 2) + 2 * 64 * 4
    assert lib.favorsharp_fit_workspace_bytes(4, 8, 16384, 16384, 64, 8) > 0


def test_argument_errors_are_reported_before_any_device_work(lib):
    from paper_2302_00787_amd.binding import FsTensor
    t = FsTensor(None, 0, 0, 0, 64)
    P = ctypes.byref
    # null tensors / parameters -> invalid argument
    assert lib.favorsharp_attention(None, 1, P(t), P(t), P(t), 1, 1, 64, 64, 64, 64, 1.0, None, 1, 64, 0, 0, P(t),
                                    None, 0, None) == 1
    # causal with different query / key lengths, d too large -> unsupported
    assert lib.favorsharp_attention(None, 1, P(t), P(t), P(t), 1, 1, 32, 64, 64, 64, 1.0, None, 1, 64, 1, 0, P(t),
                                    None, 0, None) == 2
    assert lib.favorsharp_attention(None, 1, P(t), P(t), P(t), 1, 1, 64, 64, 256, 64, 1.0, None, 1, 64, 0, 0, P(t),
                                    None, 0, None) == 2
    # more than 65535 sequences -> unsupported
    assert lib.favorsharp_attention(None, 1, P(t), P(t), P(t), 8192, 8, 64, 64, 64, 64, 1.0, None, 1, 64, 0, 0, P(t),
                                    None, 0, None) == 2
    assert lib.favorsharp_fit_params(1, P(t), P(t), 8192, 8, 8, 8, 8, 1.0, 1, 0.0, None, None, 0, None) == 2
    assert lib.favorsharp_fit_params(9, P(t), P(t), 1, 1, 8, 8, 8, 1.0, 1, 0.0, None, None, 0, None) == 1
    assert lib.favorsharp_attention_flushed_rows(None, None, None) == 1
    assert lib.favorsharp_features(None, 3, P(t), 8, 8, 1.0, 0.0, None, 8, None, None, None, 0, None) == 1
    assert lib.favorsharp_kernel_matvec(None, P(t), P(t), 8, 8, 8, 1.0, 0.0, None, 8, None, 200, None, None, 0,
                                        None) == 2


def test_noalloc_entry_point_rejects_sizes_beyond_its_scratch_array_before_any_device_work(lib):
    from paper_2302_00787_amd.binding import FsTensor, NOALLOC_SCRATCH_BYTES
    t = FsTensor(None, 1, 0, 0, 128)
    P = ctypes.byref
    # the long-context workload needs far more than the fixed array
    assert lib.favorsharp_attention_workspace_bytes(1, 16, 65536, 65536, 128, 128, 512, 1, 16, 16) > NOALLOC_SCRATCH_BYTES
    assert lib.favorsharp_attention_noalloc(None, 16, P(t), P(t), P(t), 1, 16, 65536, 65536, 128, 128, 1.0, None, 16, 512,
                                            1, 64, P(t), None) == 6
    assert b"scratch" in lib.favorsharp_status_string(6)
    # invalid shapes are still reported as such
    assert lib.favorsharp_attention_noalloc(None, 3, P(t), P(t), P(t), 1, 16, 64, 64, 128, 128, 1.0, None, 16, 512, 1, 64,
                                            P(t), None) == 1


def test_prepared_entry_points_validate_before_any_device_work(lib):
    from paper_2302_00787_amd.binding import FsTensor
    t = FsTensor(None, 1, 0, 0, 64)
    P = ctypes.byref
    assert lib.favorsharp_prepared_bytes(4, 8, 64, 256, 8, 8) > 2 * 8 * 2 * 256 * 64
    assert lib.favorsharp_prepared_bytes(1, 16, 128, 512, 16, 16) > 0
    assert lib.favorsharp_prepared_bytes(1, 1, 16, 64, 1, 1) == 0          # no constants are kept for this shape
    dense = ctypes.c_int(7)
    assert lib.favorsharp_attention_prepare(None, 8, None, 8, 4, 8, 64, 256, 1.0, None, 0, ctypes.byref(dense), None) == 1
    assert lib.favorsharp_attention_prepared(None, 0, 0, None, 8, P(t), P(t), P(t), 4, 8, 64, 64, 64, 64, 1.0, None, 8, 256,
                                             1, 64, P(t), None, 0, None) == 1
    assert dense.value == 7


def test_backward_prepared_entry_point_validates_before_any_device_work(lib):
    from paper_2302_00787_amd.binding import FsTensor
    t = FsTensor(None, 0, 0, 0, 64)
    P = ctypes.byref
    tail = (None, 1, P(t), P(t), P(t), P(t), 1, 1, 64, 64, 64, 64, 1.0, None, 1, 256, 0, P(t), P(t), P(t), None, 0, None)
    assert lib.favorsharp_attention_backward_prepared(None, 0, 0, *tail) == 1                    # no buffer
    buf = ctypes.create_string_buffer(16)
    assert lib.favorsharp_attention_backward_prepared(buf, 16, 2, *tail) == 1                    # dense_c2 not 0 / 1
    assert lib.favorsharp_attention_backward_prepared(buf, 16, 0, *tail) == 4                    # buffer too small
    other = (None, 1, P(t), P(t), P(t), P(t), 1, 1, 64, 64, 32, 32, 1.0, None, 1, 64, 0, P(t), P(t), P(t), None, 0, None)
    assert lib.favorsharp_attention_backward_prepared(buf, 16, 0, *other) == 2                   # no constants for d = 32


def test_pack_and_unpack_theta_roundtrip():
    import numpy as np
    from paper_2302_00787_amd import binding
    d = 5
    rng = np.random.default_rng(0)
    B = rng.standard_normal((d, d))
    vec = binding.pack_theta(-rng.random(d), B, B, -0.5 * np.eye(d), -0.5 * np.eye(d), 0.3, 1.5, 4)
    u = binding.unpack_theta(vec, d)
    assert u["flags"] == 3 and u["variant"] == 4 and abs(u["logD"] - 0.3) < 1e-6
    np.testing.assert_allclose(u["B2"], B.astype(np.float32))
    assert len(vec) == 8 + d + 4 * d * d


def test_orthogonal_omega_matches_the_oracle_and_reports_rank_deficiency():
    """Host-only entry point: runs without a GPU.  Compared element by element with the oracle's QR-based routine."""
    import numpy as np
    from oracle import favorsharp_oracle as orc
    from paper_2302_00787_amd import binding as fs
    rng = np.random.default_rng(21)
    groups, M, d = 3, 150, 64                   # two full blocks and a ragged one per group
    G = rng.standard_normal((groups, M, d)).astype(np.float32)
    N = rng.standard_normal((groups, M, d)).astype(np.float32)
    out = fs.orthogonal_omega(G, N)
    assert out.shape == (groups, M, d) and out.dtype == np.float32
    for g in range(groups):
        ref = orc.orthogonal_omega(G[g].astype(np.float64), N[g].astype(np.float64))
        assert np.max(np.abs(out[g] - ref)) <= 2e-6 * np.max(np.abs(ref))
    # 2-D input = one group; M < d = one short block
    small = fs.orthogonal_omega(G[0, :5], N[0, :5])
    assert np.allclose(small, orc.orthogonal_omega(G[0, :5].astype(np.float64), N[0, :5].astype(np.float64)), atol=1e-5)
    # a repeated row has no direction of its own left
    bad = G[0, :8].copy()
    bad[3] = bad[1]
    try:
        fs.orthogonal_omega(bad, N[0, :8])
        raise AssertionError("rank deficiency not reported")
    except fs.FavorSharpError as e:
        assert "NOT_PD" in str(e).upper() or "singular" in str(e).lower(), str(e)
