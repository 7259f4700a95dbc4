"""Thin ctypes binding over libfavorsharp.so: argument marshalling only.

Function names mirror the C ABI (include/favorsharp.h).  PyTorch supplies device
memory and the current stream; every step of the computation runs in the HIP
kernels of the library.  There is no fallback: if the library has not been built
the import of `lib()` raises.
"""
from __future__ import annotations

import ctypes
import math
import os
from ctypes import c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfavorsharp.so")

VARIANTS = {"posrf": 0, "gerf": 1, "saderf": 2, "aderf": 3, "sderf": 4}
FS_F32, FS_BF16 = 0, 1
THETA_HEADER = 8


class FsTensor(ctypes.Structure):
    _fields_ = [("ptr", c_void_p), ("dtype", c_int32), ("stride_b", c_int64), ("stride_h", c_int64),
                ("stride_l", c_int64)]


class FavorSharpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().favorsharp_status_string(status).decode()} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2302_00787_amd.build` "
                              "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        P = ctypes.POINTER(FsTensor)
        L.favorsharp_theta_floats.restype = c_size_t
        L.favorsharp_theta_floats.argtypes = [c_int]
        L.favorsharp_status_string.restype = c_char_p
        L.favorsharp_status_string.argtypes = [c_int]
        L.favorsharp_version.restype = c_char_p
        L.favorsharp_version.argtypes = []
        L.favorsharp_orthogonal_omega.restype = c_int
        L.favorsharp_orthogonal_omega.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_void_p]
        L.favorsharp_fit_workspace_bytes.restype = c_size_t
        L.favorsharp_fit_workspace_bytes.argtypes = [c_int] * 6
        L.favorsharp_fit_params.restype = c_int
        L.favorsharp_fit_params.argtypes = [c_int, P, P, c_int, c_int, c_int, c_int, c_int, c_float, c_int, c_float,
                                            c_void_p, c_void_p, c_size_t, c_void_p]
        L.favorsharp_fit_device_workspace_bytes.restype = c_size_t
        L.favorsharp_fit_device_workspace_bytes.argtypes = [c_int] * 6
        L.favorsharp_fit_params_device.restype = c_int
        L.favorsharp_fit_params_device.argtypes = [c_int, P, P, c_int, c_int, c_int, c_int, c_int, c_float, c_int, c_float,
                                                   c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
        L.favorsharp_features_workspace_bytes.restype = c_size_t
        L.favorsharp_features_workspace_bytes.argtypes = [c_int] * 3
        L.favorsharp_features.restype = c_int
        L.favorsharp_features.argtypes = [c_void_p, c_int, P, c_int, c_int, c_float, c_float, c_void_p, c_int,
                                          c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
        L.favorsharp_attention_workspace_bytes.restype = c_size_t
        L.favorsharp_attention_workspace_bytes.argtypes = [c_int] * 10
        L.favorsharp_attention.restype = c_int
        L.favorsharp_attention.argtypes = [c_void_p, c_int, P, P, P, c_int, c_int, c_int, c_int, c_int, c_int, c_float,
                                           c_void_p, c_int, c_int, c_int, c_int, P, c_void_p, c_size_t, c_void_p]
        L.favorsharp_attention_timed.restype = c_int
        L.favorsharp_attention_timed.argtypes = L.favorsharp_attention.argtypes + [c_void_p, c_void_p]
        L.favorsharp_prepared_bytes.restype = c_size_t
        L.favorsharp_prepared_bytes.argtypes = [c_int] * 6
        L.favorsharp_attention_prepare.restype = c_int
        L.favorsharp_attention_prepare.argtypes = [c_void_p, c_int, c_void_p, c_int, c_int, c_int, c_int, c_int, c_float,
                                                   c_void_p, c_size_t, ctypes.POINTER(c_int), c_void_p]
        L.favorsharp_attention_prepared.restype = c_int
        L.favorsharp_attention_prepared.argtypes = [c_void_p, c_size_t, c_int] + L.favorsharp_attention.argtypes
        L.favorsharp_attention_noalloc.restype = c_int
        L.favorsharp_attention_noalloc.argtypes = L.favorsharp_attention.argtypes[:18] + [c_void_p]
        L.favorsharp_attention_flushed_rows.restype = c_int
        L.favorsharp_attention_flushed_rows.argtypes = [c_void_p, ctypes.POINTER(c_int), c_void_p]
        L.favorsharp_attention_backward_workspace_bytes.restype = c_size_t
        L.favorsharp_attention_backward_workspace_bytes.argtypes = [c_int] * 10
        L.favorsharp_attention_backward.restype = c_int
        L.favorsharp_attention_backward.argtypes = [c_void_p, c_int, P, P, P, P, c_int, c_int, c_int, c_int, c_int, c_int,
                                                    c_float, c_void_p, c_int, c_int, c_int, P, P, P, c_void_p, c_size_t,
                                                    c_void_p]
        L.favorsharp_attention_backward_prepared.restype = c_int
        L.favorsharp_attention_backward_prepared.argtypes = [c_void_p, c_size_t, c_int] + L.favorsharp_attention_backward.argtypes
        L.favorsharp_kernel_matvec_workspace_bytes.restype = c_size_t
        L.favorsharp_kernel_matvec_workspace_bytes.argtypes = [c_int] * 5
        L.favorsharp_kernel_matvec.restype = c_int
        L.favorsharp_kernel_matvec.argtypes = [c_void_p, P, P, c_int, c_int, c_int, c_float, c_float, c_void_p, c_int,
                                               c_void_p, c_int, c_void_p, c_void_p, c_size_t, c_void_p]
        _lib = L
    return _lib


# ------------------------------------------------------------------ marshalling helpers
def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FS_F32
    if t.dtype == torch.bfloat16:
        return FS_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _desc4(t: torch.Tensor) -> FsTensor:
    """[B, H, L, d] (or [L, d]) CUDA tensor -> fs_tensor."""
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if t.dim() == 2:
        sb = sh = 0
        sl, sd = t.stride()
    elif t.dim() == 4:
        sb, sh, sl, sd = t.stride()
    else:
        raise ValueError("expected a [B,H,L,d] or [L,d] tensor")
    if sd != 1 and t.shape[-1] > 1:
        raise ValueError("innermost stride must be 1")
    return FsTensor(t.data_ptr(), _dtype_code(t), sb, sh, sl)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _workspace(nbytes: int, device, workspace: torch.Tensor | None) -> torch.Tensor:
    if workspace is not None:
        if workspace.dtype != torch.uint8 or not workspace.is_cuda:
            raise ValueError("workspace must be a CUDA uint8 tensor")
        return workspace
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _check(status: int, where: str):
    if status != 0:
        raise FavorSharpError(status, where)


def theta_floats(d: int) -> int:
    return int(lib().favorsharp_theta_floats(d))


def pack_theta(A, B1, B2, C1, C2, logD, lbar=float("nan"), variant=4) -> np.ndarray:
    """Lay one parameter set out as the library expects it (float32 vector)."""
    A = np.asarray(A, dtype=np.float64)
    d = A.shape[0]
    C1, C2 = np.asarray(C1, dtype=np.float64), np.asarray(C2, dtype=np.float64)
    B1, B2 = np.asarray(B1, dtype=np.float64), np.asarray(B2, dtype=np.float64)
    flags = 0
    if np.array_equal(C1, -0.5 * np.eye(d)) and np.array_equal(C2, -0.5 * np.eye(d)):
        flags |= 1
    if np.array_equal(B1, B2):
        flags |= 2
    head = np.zeros(THETA_HEADER)
    head[0], head[1], head[2], head[3] = logD, lbar if lbar is not None else float("nan"), flags, variant
    return np.concatenate([head, A, B1.ravel(), B2.ravel(), C1.ravel(), C2.ravel()]).astype(np.float32)


def unpack_theta(vec: np.ndarray, d: int) -> dict:
    vec = np.asarray(vec, dtype=np.float32)
    o = THETA_HEADER
    dd = d * d
    return dict(logD=float(vec[0]), lbar=float(vec[1]), flags=int(vec[2]), variant=int(vec[3]),
                A=vec[o:o + d].copy(), B1=vec[o + d:o + d + dd].reshape(d, d).copy(),
                B2=vec[o + d + dd:o + d + 2 * dd].reshape(d, d).copy(),
                C1=vec[o + d + 2 * dd:o + d + 3 * dd].reshape(d, d).copy(),
                C2=vec[o + d + 3 * dd:o + d + 4 * dd].reshape(d, d).copy())


def to_device(a: np.ndarray, dtype: str) -> torch.Tensor:
    """Host array -> device tensor, float32 ("f32") or bfloat16 ("bf16": the values must already be representable,
    as the input generators leave them; their upper 16 bits are uploaded)."""
    if dtype == "bf16":
        from . import synth
        bits = synth.to_bf16_bits(a)
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> float64 host array."""
    return t.detach().float().cpu().numpy().astype(np.float64)


# ------------------------------------------------------------------ entry points
def fit_workspace_bytes(B, H, Lx, Ly, d, groups) -> int:
    return int(lib().favorsharp_fit_workspace_bytes(B, H, Lx, Ly, d, groups))


def fit_params(variant, X: torch.Tensor, Y: torch.Tensor, qk_scale: float, groups: int = 1, eig_ridge: float = 0.0,
               workspace: torch.Tensor | None = None) -> torch.Tensor:
    """favorsharp_fit_params: X [B,H,Lx,d], Y [B,H,Ly,d] -> theta [groups, theta_floats(d)] (float32, device)."""
    v = VARIANTS[variant] if isinstance(variant, str) else int(variant)
    if X.dim() == 2:
        X, Y = X[None, None], Y[None, None]
    B, H, Lx, d = X.shape
    Ly = Y.shape[2]
    theta = torch.empty((groups, theta_floats(d)), dtype=torch.float32, device=X.device)
    nbytes = fit_workspace_bytes(B, H, Lx, Ly, d, groups)
    ws = _workspace(nbytes, X.device, workspace)
    dx, dy = _desc4(X), _desc4(Y)
    st = lib().favorsharp_fit_params(v, ctypes.byref(dx), ctypes.byref(dy), B, H, Lx, Ly, d, qk_scale, groups,
                                     eig_ridge, theta.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    _check(st, "favorsharp_fit_params")
    return theta


def fit_device_workspace_bytes(B, H, Lx, Ly, d, groups) -> int:
    return int(lib().favorsharp_fit_device_workspace_bytes(B, H, Lx, Ly, d, groups))


def fit_params_device(variant, X: torch.Tensor, Y: torch.Tensor, qk_scale: float, groups: int = 1,
                      eig_ridge: float = 0.0, workspace: torch.Tensor | None = None):
    """favorsharp_fit_params_device: as fit_params, without a host round trip.  Returns (theta, status), both on the
    device; status [groups] int32 is valid once the stream has run the call (no synchronisation happens here)."""
    v = VARIANTS[variant] if isinstance(variant, str) else int(variant)
    if X.dim() == 2:
        X, Y = X[None, None], Y[None, None]
    B, H, Lx, d = X.shape
    Ly = Y.shape[2]
    theta = torch.empty((groups, theta_floats(d)), dtype=torch.float32, device=X.device)
    status = torch.empty((groups,), dtype=torch.int32, device=X.device)
    nbytes = fit_device_workspace_bytes(B, H, Lx, Ly, d, groups)
    ws = _workspace(nbytes, X.device, workspace)
    dx, dy = _desc4(X), _desc4(Y)
    st = lib().favorsharp_fit_params_device(v, ctypes.byref(dx), ctypes.byref(dy), B, H, Lx, Ly, d, qk_scale, groups,
                                            eig_ridge, theta.data_ptr(), status.data_ptr(), ws.data_ptr(), ws.numel(),
                                            _stream())
    _check(st, "favorsharp_fit_params_device")
    return theta, status


def features_workspace_bytes(n, d, M) -> int:
    return int(lib().favorsharp_features_workspace_bytes(n, d, M))


def features(theta: torch.Tensor, side: int, X: torch.Tensor, qk_scale: float, alpha: float, Omega: torch.Tensor,
             stabilise: bool = False, workspace: torch.Tensor | None = None):
    """favorsharp_features: X [n,d] -> out [n,M] float32 (and row_logscale [n] when stabilise)."""
    n, d = X.shape
    M = Omega.shape[-2]
    out = torch.empty((n, M), dtype=torch.float32, device=X.device)
    rls = torch.empty((n,), dtype=torch.float32, device=X.device) if stabilise else None
    ws = _workspace(features_workspace_bytes(n, d, M), X.device, workspace)
    dx = _desc4(X)
    st = lib().favorsharp_features(theta.data_ptr(), side, ctypes.byref(dx), n, d, qk_scale, alpha, Omega.data_ptr(), M,
                                   out.data_ptr(), rls.data_ptr() if stabilise else None, ws.data_ptr(), ws.numel(),
                                   _stream())
    _check(st, "favorsharp_features")
    return (out, rls) if stabilise else out


def attention_workspace_bytes(B, H, Lq, Lk, d, dv, M, causal, groups, omega_groups) -> int:
    return int(lib().favorsharp_attention_workspace_bytes(B, H, Lq, Lk, d, dv, M, int(causal), groups, omega_groups))


def attention(theta: torch.Tensor, Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, qk_scale: float,
              Omega: torch.Tensor, causal: bool = False, chunk: int = 0, out: torch.Tensor | None = None,
              out_dtype=None, workspace: torch.Tensor | None = None, events=None) -> torch.Tensor:
    """favorsharp_attention: Q [B,H,Lq,d], K [B,H,Lk,d], V [B,H,Lk,dv], theta [groups,*], Omega [og,M,d] -> Y."""
    B, H, Lq, d = Q.shape
    Lk, dv = K.shape[2], V.shape[3]
    groups = theta.shape[0] if theta.dim() == 2 else 1
    og, M = (Omega.shape[0], Omega.shape[1]) if Omega.dim() == 3 else (1, Omega.shape[0])
    if out is None:
        out = torch.empty((B, H, Lq, dv), dtype=out_dtype or Q.dtype, device=Q.device)
    nbytes = attention_workspace_bytes(B, H, Lq, Lk, d, dv, M, causal, groups, og)
    ws = _workspace(nbytes, Q.device, workspace)
    dq, dk, dvv, dy = _desc4(Q), _desc4(K), _desc4(V), _desc4(out)
    args = (theta.data_ptr(), groups, ctypes.byref(dq), ctypes.byref(dk), ctypes.byref(dvv),
            B, H, Lq, Lk, d, dv, qk_scale, Omega.data_ptr(), og, M, int(causal), chunk,
            ctypes.byref(dy), ws.data_ptr(), ws.numel(), _stream())
    if events is None:
        st = lib().favorsharp_attention(*args)
    else:       # (hipEvent_t begin, hipEvent_t end) as integers: favorsharp_attention_timed
        st = lib().favorsharp_attention_timed(*args, events[0], events[1])
    _check(st, "favorsharp_attention")
    return out


def prepared_bytes(B, H, d, M, groups, omega_groups) -> int:
    return int(lib().favorsharp_prepared_bytes(B, H, d, M, groups, omega_groups))


def attention_prepare(theta: torch.Tensor, Omega: torch.Tensor, B: int, H: int, qk_scale: float):
    """favorsharp_attention_prepare: the projection constants of (theta, Omega) -> (prepared buffer, dense_c2)."""
    groups = theta.shape[0] if theta.dim() == 2 else 1
    og, M, d = (Omega.shape[0], Omega.shape[1], Omega.shape[2]) if Omega.dim() == 3 else (1, Omega.shape[0], Omega.shape[1])
    buf = torch.empty(max(prepared_bytes(B, H, d, M, groups, og), 256), dtype=torch.uint8, device=theta.device)
    dense = c_int(0)
    st = lib().favorsharp_attention_prepare(theta.data_ptr(), groups, Omega.data_ptr(), og, B, H, d, M, qk_scale,
                                            buf.data_ptr(), buf.numel(), ctypes.byref(dense), _stream())
    _check(st, "favorsharp_attention_prepare")
    return buf, int(dense.value)


def attention_prepared(prepared, theta: torch.Tensor, Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, qk_scale: float,
                       Omega: torch.Tensor, causal: bool = False, chunk: int = 0, out: torch.Tensor | None = None,
                       out_dtype=None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """favorsharp_attention_prepared: `prepared` = what attention_prepare returned for the same theta, Omega, qk_scale."""
    buf, dense = prepared
    B, H, Lq, d = Q.shape
    Lk, dv = K.shape[2], V.shape[3]
    groups = theta.shape[0] if theta.dim() == 2 else 1
    og, M = (Omega.shape[0], Omega.shape[1]) if Omega.dim() == 3 else (1, Omega.shape[0])
    if out is None:
        out = torch.empty((B, H, Lq, dv), dtype=out_dtype or Q.dtype, device=Q.device)
    ws = _workspace(attention_workspace_bytes(B, H, Lq, Lk, d, dv, M, causal, groups, og), Q.device, workspace)
    dq, dk, dvv, dy = _desc4(Q), _desc4(K), _desc4(V), _desc4(out)
    st = lib().favorsharp_attention_prepared(buf.data_ptr(), buf.numel(), dense, theta.data_ptr(), groups, ctypes.byref(dq),
                                             ctypes.byref(dk), ctypes.byref(dvv), B, H, Lq, Lk, d, dv, qk_scale,
                                             Omega.data_ptr(), og, M, int(causal), chunk, ctypes.byref(dy), ws.data_ptr(),
                                             ws.numel(), _stream())
    _check(st, "favorsharp_attention_prepared")
    return out


NOALLOC_SCRATCH_BYTES = 64 << 20


def attention_noalloc(theta: torch.Tensor, Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, qk_scale: float,
                      Omega: torch.Tensor, out: torch.Tensor, causal: bool = False, chunk: int = 0) -> torch.Tensor:
    """favorsharp_attention_noalloc: as `attention`, on the library's own scratch array; `out` is required (nothing
    is allocated here either)."""
    B, H, Lq, d = Q.shape
    Lk, dv = K.shape[2], V.shape[3]
    groups = theta.shape[0] if theta.dim() == 2 else 1
    og, M = (Omega.shape[0], Omega.shape[1]) if Omega.dim() == 3 else (1, Omega.shape[0])
    dq, dk, dvv, dy = _desc4(Q), _desc4(K), _desc4(V), _desc4(out)
    st = lib().favorsharp_attention_noalloc(theta.data_ptr(), groups, ctypes.byref(dq), ctypes.byref(dk), ctypes.byref(dvv),
                                            B, H, Lq, Lk, d, dv, qk_scale, Omega.data_ptr(), og, M, int(causal), chunk,
                                            ctypes.byref(dy), _stream())
    _check(st, "favorsharp_attention_noalloc")
    return out


def attention_flushed_rows(workspace: torch.Tensor | None = None) -> int:
    """favorsharp_attention_flushed_rows: how many output rows of the last attention call on `workspace` (None: the
    scratch array of `attention_noalloc`) had a zero normaliser and were written as zeros.  Waits for the stream."""
    n = c_int(0)
    st = lib().favorsharp_attention_flushed_rows(None if workspace is None else workspace.data_ptr(), ctypes.byref(n),
                                                 _stream())
    _check(st, "favorsharp_attention_flushed_rows")
    return int(n.value)


def attention_backward_workspace_bytes(B, H, Lq, Lk, d, dv, M, causal, groups, omega_groups) -> int:
    return int(lib().favorsharp_attention_backward_workspace_bytes(B, H, Lq, Lk, d, dv, M, int(causal), groups,
                                                                    omega_groups))


def attention_backward(theta: torch.Tensor, Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, dY: torch.Tensor,
                       qk_scale: float, Omega: torch.Tensor, causal: bool = False, grad_dtype=None,
                       workspace: torch.Tensor | None = None, grads=None, prepared=None):
    """favorsharp_attention_backward: gradients of sum(Y * dY) -> (dQ, dK, dV), shaped like Q, K, V
    (`grads`: three preallocated tensors to write into, any row strides; `prepared`: what attention_prepare returned
    for the same theta, Omega, qk_scale: favorsharp_attention_backward_prepared)."""
    B, H, Lq, d = Q.shape
    Lk, dv = K.shape[2], V.shape[3]
    groups = theta.shape[0] if theta.dim() == 2 else 1
    og, M = (Omega.shape[0], Omega.shape[1]) if Omega.dim() == 3 else (1, Omega.shape[0])
    gd = grad_dtype or Q.dtype
    if grads is not None:
        gQ, gK, gV = grads
    else:
        gQ = torch.empty((B, H, Lq, d), dtype=gd, device=Q.device)
        gK = torch.empty((B, H, Lk, d), dtype=gd, device=Q.device)
        gV = torch.empty((B, H, Lk, dv), dtype=gd, device=Q.device)
    nbytes = attention_backward_workspace_bytes(B, H, Lq, Lk, d, dv, M, causal, groups, og)
    ws = _workspace(nbytes, Q.device, workspace)
    descs = [_desc4(t) for t in (Q, K, V, dY, gQ, gK, gV)]
    args = (theta.data_ptr(), groups, ctypes.byref(descs[0]), ctypes.byref(descs[1]), ctypes.byref(descs[2]),
            ctypes.byref(descs[3]), B, H, Lq, Lk, d, dv, qk_scale, Omega.data_ptr(), og, M, int(causal),
            ctypes.byref(descs[4]), ctypes.byref(descs[5]), ctypes.byref(descs[6]), ws.data_ptr(), ws.numel(), _stream())
    if prepared is None:
        _check(lib().favorsharp_attention_backward(*args), "favorsharp_attention_backward")
    else:
        buf, dense = prepared
        _check(lib().favorsharp_attention_backward_prepared(buf.data_ptr(), buf.numel(), dense, *args),
               "favorsharp_attention_backward_prepared")
    return gQ, gK, gV


def orthogonal_omega(gauss_dir: np.ndarray, gauss_len: np.ndarray) -> np.ndarray:
    """favorsharp_orthogonal_omega (host): [groups, M, d] or [M, d] Gaussian draws -> block-orthogonal omega, float32."""
    g = np.ascontiguousarray(gauss_dir, dtype=np.float32)
    n = np.ascontiguousarray(gauss_len, dtype=np.float32)
    if g.shape != n.shape or g.ndim not in (2, 3):
        raise ValueError("gauss_dir and gauss_len must have the same shape [groups, M, d] or [M, d]")
    groups = 1 if g.ndim == 2 else g.shape[0]
    M, d = g.shape[-2], g.shape[-1]
    out = np.empty_like(g)
    _check(lib().favorsharp_orthogonal_omega(g.ctypes.data_as(c_void_p), n.ctypes.data_as(c_void_p), groups, M, d,
                                             out.ctypes.data_as(c_void_p)), "favorsharp_orthogonal_omega")
    return out


def kernel_matvec_workspace_bytes(Nx, Ny, d, M, n) -> int:
    return int(lib().favorsharp_kernel_matvec_workspace_bytes(Nx, Ny, d, M, n))


def kernel_matvec(theta: torch.Tensor, X: torch.Tensor, Y: torch.Tensor, qk_scale: float, alpha: float,
                  Omega: torch.Tensor, C: torch.Tensor, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """favorsharp_kernel_matvec: X [Nx,d], Y [Ny,d], C [Ny,n] float32 -> out [Nx,n] float32."""
    Nx, d = X.shape
    Ny, n = C.shape
    M = Omega.shape[-2]
    if C.dtype != torch.float32 or not C.is_contiguous():
        raise ValueError("C must be contiguous float32")
    out = torch.empty((Nx, n), dtype=torch.float32, device=X.device)
    ws = _workspace(kernel_matvec_workspace_bytes(Nx, Ny, d, M, n), X.device, workspace)
    dx, dy = _desc4(X), _desc4(Y)
    st = lib().favorsharp_kernel_matvec(theta.data_ptr(), ctypes.byref(dx), ctypes.byref(dy), Nx, Ny, d, qk_scale,
                                        alpha, Omega.data_ptr(), M, C.data_ptr(), n, out.data_ptr(), ws.data_ptr(),
                                        ws.numel(), _stream())
    _check(st, "favorsharp_kernel_matvec")
    return out
