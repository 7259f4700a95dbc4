"""Helpers shared by the tests: moving data between numpy (oracle side) and the device (HIP side)."""
import numpy as np

from oracle import favorsharp_oracle as orc
from paper_2302_00787_amd import synth


def theta_vec_from_oracle(th) -> np.ndarray:
    from paper_2302_00787_amd import binding
    variant = binding.VARIANTS.get(th.name, 4)
    return binding.pack_theta(th.A, th.B1, th.B2, th.C1, th.C2, th.logD, th.lbar, variant)


def oracle_theta_from_vec(vec, d):
    """The float32 parameter block, read back as the oracle's Theta, so both sides see identical numbers."""
    from paper_2302_00787_amd import binding
    u = binding.unpack_theta(vec, d)
    f = lambda a: np.asarray(a, dtype=np.float64)
    return orc.Theta(A=f(u["A"]), B1=f(u["B1"]), B2=f(u["B2"]), C1=f(u["C1"]), C2=f(u["C2"]), logD=float(u["logD"]))


def to_device(a: np.ndarray, dtype: str):
    from paper_2302_00787_amd import binding
    return binding.to_device(a, dtype)


def to_host(t) -> np.ndarray:
    from paper_2302_00787_amd import binding
    return binding.to_host(t)


def attention_errors(Y_gpu: np.ndarray, Y_ref: np.ndarray, V: np.ndarray):
    """(relative Frobenius error, worst row error relative to the largest value-row norm) for one (b, h)."""
    diff = Y_gpu - Y_ref
    fro = np.linalg.norm(diff) / max(np.linalg.norm(Y_ref), 1e-300)
    row = np.linalg.norm(diff, axis=1).max() / np.linalg.norm(V, axis=1).max()
    return float(fro), float(row)


def gradient_errors(g_gpu: np.ndarray, g_ref: np.ndarray, floor: float = 0.0):
    """(relative Frobenius error, worst row error relative to the largest row norm of the reference) for one
    gradient tensor of one (b, h); `floor` stands in for a reference that is zero by construction."""
    diff = g_gpu - g_ref
    fro = np.linalg.norm(diff) / max(np.linalg.norm(g_ref), floor, 1e-300)
    row = np.linalg.norm(diff, axis=1).max() / max(np.linalg.norm(g_ref, axis=1).max(), floor, 1e-300)
    return float(fro), float(row)
