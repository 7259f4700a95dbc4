#!/usr/bin/env python3
"""Benchmark of the FAVOR# hot path on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4] [--only] [--no-cpu-baseline]

One "step" is one attention call on the metric workload (causal, bf16, B=4 H=8 L=16384 d=64 M=256, chunk 64):
both feature maps (fused, never stored) and the causal prefix-state contraction, with Q, K, V, omega, the fitted
parameters and the projection constants derived from them (favorsharp_attention_prepare, once per parameter set)
already resident in HBM; `ms_per_step_unprepared` is the same call with the constants rebuilt inside it.  The closed-form fit
(statistics scan on the GPU + d x d algebra on the host) is timed separately and reported as `fit_ms`, the
device-resident variant of the same fit as `fit_device_ms`.
Inputs rotate over three distinct sets so the 256 MB last-level cache cannot hold a set across steps.

Timing: `ms_per_step` is the mean wall-clock time of K back-to-back calls between two device synchronisations (it
includes every launch gap of a call); `main_kernel_ms` is the mean, over K more calls made right after the timed
ones, of the time between two HIP events that the library attaches to the dispatch of the dominant kernel (its own
begin and end on the stream the library launches on).

Prints ONE JSON line.  Headline fields: the metric workload.  `roofline`: the dominant kernel of the metric workload
(`frac`) and the whole call (`call_frac`) against the tighter of the HBM / MFMA bounds on the algorithmic counts.
`workloads`: the same measurements for the other four workloads and the two backward-pass workloads, taken in the
same run (unless --only), plus `many_short_sequences` (4096 sequences of 128 tokens on the d = 64 kernels, forward
and backward, outside the five configurations).  `families_ms` (headline, c3, c5): ms per call of the same workload with GERF, SADERF and
ADERF parameters instead of SDERF (the last two have a dense key-side quadratic form and B1 != B2).  `parity`: measured errors of the library's results against the CPU oracle on the same
inputs and the same float32 parameter block (computed in the CPU-baseline leg, which is the only part of this
script that touches the oracle).  `cpu_baseline`: the oracle timed on a bounded sample of the metric workload.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
MFMA_F32_PEAK_TFLOPS = 157.3
# HBM bytes per launch of the dominant kernel and per call, from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE`
# runs of this script (--only --calibrate-copy --workload <name>), each counter scaled by what it reads for the
# 256 MiB copy; figures, factors and commands in the file named beside the values.
MEASURED_TRAFFIC_BYTES = {
    "c4": (294.1e6, 508e6, "profiles/hbm_traffic_c2_c3_c4_c5.md"),
    "c3": (111.5e6, 270e6, "profiles/hbm_traffic_c2_c3_c4_c5.md"),
    "c5": (3.04e9, 3.71e9, "profiles/hbm_traffic_c2_c3_c4_c5.md"),
}
TOL = {"f32": 1e-4, "bf16": 2e-2}


class HipEvents:
    """hipEvent_t pairs created straight from the HIP runtime (the library records them on its own stream)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]

    def create(self) -> int:
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed ({rc})")
        return ev.value

    def elapsed_ms(self, a: int, b: int) -> float:
        self.hip.hipEventSynchronize(b)
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(ms.value)

    def destroy(self, ev: int):
        self.hip.hipEventDestroy(ev)


def algorithmic_counts(cfg: dict) -> dict:
    """Per-launch algorithmic work of the attention workloads: per head-token, bytes = 3 d e_in + d e_out,
    flops = 2 projections (2 d M each) + state update and state read (2 M (d+1) each) + the causal
    intra-chunk part ((T+1)/2 (2M + 2(d+1)))."""
    B, H, L, d, M = cfg["B"], cfg["H"], cfg["L"], cfg["d"], cfg["M"]
    esz = 2 if cfg["dtype"] == "bf16" else 4
    ht = B * H * L
    flops = 4 * d * M + 4 * M * (d + 1)
    if cfg["causal"]:
        T = cfg.get("chunk", 64)
        flops += (T + 1) / 2 * (2 * M + 2 * (d + 1))
    # the dominant kernel of a causal call does the whole method on its tokens; the query-side kernel of a non-causal
    # call reads Q, writes Y and does the query-side projection and the state read (the key side is another kernel)
    main_bytes = ht * 4 * d * esz if cfg["causal"] else ht * 2 * d * esz
    main_flops = ht * flops if cfg["causal"] else ht * (2 * d * M + 2 * M * (d + 1))
    return dict(head_tokens=ht, bytes=ht * 4 * d * esz, flops=ht * flops, main_bytes=main_bytes, main_flops=main_flops)


def host_cores() -> int:
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def timed(step, steps: int, warmup: int, torch) -> float:
    """Mean wall-clock milliseconds of `steps` back-to-back calls after `warmup` untimed ones."""
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3


# ---------------------------------------------------------------------------------------------- attention workloads
def run_attention(name: str, steps: int, warmup: int, fs, synth, torch, nsets: int = 3, with_fit: bool = False,
                  calibrate_copy: bool = False) -> dict:
    """Times favorsharp_attention on workload `name`; returns the measurements, the first input set (host and
    device) and that set's output for the parity leg."""
    cfg = dict(synth.WORKLOADS[name])
    dtype = cfg["dtype"]
    B, H, L, d, M = cfg["B"], cfg["H"], cfg["L"], cfg["d"], cfg["M"]
    causal, chunk = cfg["causal"], cfg.get("chunk", 0)
    sets, w0 = [], None
    for i in range(nsets):
        w = synth.make(name, seed=cfg["seed"] + i)
        w0 = w0 or w
        sets.append(dict(Q=fs.to_device(w["Q"], dtype), K=fs.to_device(w["K"], dtype), V=fs.to_device(w["V"], dtype),
                         Omega=torch.from_numpy(w["Omega"]).cuda()))
        del w
    s = w0["qk_scale"]
    for st_ in sets:
        st_["theta"] = fs.fit_params("sderf", st_["Q"], st_["K"], s, groups=H)
    out = dict(cfg=cfg, w0=w0, theta0=sets[0]["theta"])
    if with_fit:
        # fit (timed separately): statistics on the GPU, closed form on the host
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fs.fit_params("sderf", sets[0]["Q"], sets[0]["K"], s, groups=H)
        torch.cuda.synchronize()
        out["fit_ms"] = (time.perf_counter() - t0) * 1e3
        # the same fit with the closed form on the device (asynchronous entry point; the timing includes the final sync)
        fit_ws = torch.empty(fs.fit_device_workspace_bytes(B, H, L, L, d, H), dtype=torch.uint8, device="cuda")
        fs.fit_params_device("sderf", sets[0]["Q"], sets[0]["K"], s, groups=H, workspace=fit_ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        _, fit_status = fs.fit_params_device("sderf", sets[0]["Q"], sets[0]["K"], s, groups=H, workspace=fit_ws)
        torch.cuda.synchronize()
        out["fit_device_ms"] = (time.perf_counter() - t0) * 1e3
        assert int(fit_status.abs().sum().item()) == 0
        del fit_ws

    ws = torch.empty(fs.attention_workspace_bytes(B, H, L, L, d, d, M, causal, H, H), dtype=torch.uint8, device="cuda")
    outs = [torch.empty_like(st_["V"]) for st_ in sets]
    ev = HipEvents()
    pairs = [(ev.create(), ev.create()) for _ in range(steps)]

    # theta and omega are resident: where the library keeps projection constants across calls (the bf16 kernels), they
    # are prepared once per input set, outside the timed region, like the fit
    prepared_ok = fs.prepared_bytes(B, H, d, M, H, H) > 0 and dtype == "bf16"
    if prepared_ok:
        for st_ in sets:
            st_["prepared"] = fs.attention_prepare(st_["theta"], st_["Omega"], B, H, s)

    def step(i, events=None):
        st_ = sets[i % nsets]
        fs.attention(st_["theta"], st_["Q"], st_["K"], st_["V"], s, st_["Omega"], causal=causal, chunk=chunk,
                     out=outs[i % nsets], workspace=ws, events=events)

    def step_prepared(i):
        st_ = sets[i % nsets]
        fs.attention_prepared(st_["prepared"], st_["theta"], st_["Q"], st_["K"], st_["V"], s, st_["Omega"], causal=causal,
                              chunk=chunk, out=outs[i % nsets], workspace=ws)

    if calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    ms_unprepared = timed(step, steps, warmup, torch)
    ms_per_step = timed(step_prepared, steps, warmup, torch) if prepared_ok else ms_unprepared
    # dominant kernel: events attached by the library to its dispatch, in a loop of calls right after the timed ones
    # (not in them: the steps are timed by the wall clock between two synchronisations, without events)
    for i in range(steps):
        step(i, pairs[i])
    torch.cuda.synchronize()
    main_ms = float(np.mean([ev.elapsed_ms(a, b) for a, b in pairs]))
    if prepared_ok:      # the parity leg checks what the timed call produces: the first input set once more, prepared
        step_prepared(0)
        torch.cuda.synchronize()
    for a, b in pairs:
        ev.destroy(a)
        ev.destroy(b)
    assert all(torch.isfinite(o.float()).all().item() for o in outs)

    counts = algorithmic_counts(cfg)
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if dtype == "bf16" else MFMA_F32_PEAK_TFLOPS
    t_hbm = counts["bytes"] / (HBM_PEAK_GBS * 1e9)
    t_mfma = counts["flops"] / (mfma_peak * 1e12)
    traffic = MEASURED_TRAFFIC_BYTES.get(name)
    # the dominant kernel is credited with its own share of the algorithmic work, the call with all of it
    if t_hbm >= t_mfma:
        ach = counts["main_bytes"] / (main_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS}
    else:
        ach = counts["main_flops"] / (main_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": ach, "peak": mfma_peak, "unit": "TFLOP/s", "frac": ach / mfma_peak}
    roofline.update({
        "traffic": traffic[0] if traffic else None, "call_traffic": traffic[1] if traffic else None,
        "traffic_source": traffic[2] if traffic else None,
        "call_frac": max(t_hbm, t_mfma) / (ms_per_step * 1e-3),
        "kernel_hbm_frac": counts["main_bytes"] / (HBM_PEAK_GBS * 1e9) / (main_ms * 1e-3),
        "kernel_mfma_frac": counts["main_flops"] / (mfma_peak * 1e12) / (main_ms * 1e-3),
        "call_hbm_frac": t_hbm / (ms_per_step * 1e-3), "call_mfma_frac": t_mfma / (ms_per_step * 1e-3)})
    out.update(ms_per_step=ms_per_step, ms_per_step_unprepared=ms_unprepared, prepared=bool(prepared_ok),
               main_kernel_ms=main_ms, roofline=roofline, counts=counts,
               Y0=outs[0], sets=sets, tokens_per_s=B * L / (ms_per_step * 1e-3))
    return out


def run_families(r: dict, steps: int, warmup: int, fs, torch) -> dict:
    """ms per call of the same workload (first input set, prepared constants where the library keeps them) with the
    parameters of the other families: GERF (isotropic, B1 = B2 like SDERF), SADERF and ADERF (dense key-side
    quadratic form, B1 != B2: the calls that also run the row-term kernel and reload projection slices)."""
    cfg, st_ = r["cfg"], r["sets"][0]
    B, H, L, d, M = cfg["B"], cfg["H"], cfg["L"], cfg["d"], cfg["M"]
    causal, chunk, s = cfg["causal"], cfg.get("chunk", 0), r["w0"]["qk_scale"]
    ws = torch.empty(fs.attention_workspace_bytes(B, H, L, L, d, d, M, causal, H, H), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(st_["V"])
    res = {}
    for variant in ("gerf", "saderf", "aderf"):
        theta = fs.fit_params(variant, st_["Q"], st_["K"], s, groups=H)
        if r["prepared"]:
            prep = fs.attention_prepare(theta, st_["Omega"], B, H, s)
            step = lambda i: fs.attention_prepared(prep, theta, st_["Q"], st_["K"], st_["V"], s, st_["Omega"], causal=causal,
                                                   chunk=chunk, out=out, workspace=ws)
        else:
            step = lambda i: fs.attention(theta, st_["Q"], st_["K"], st_["V"], s, st_["Omega"], causal=causal, chunk=chunk,
                                          out=out, workspace=ws)
        res[variant] = timed(step, steps, warmup, torch)
        assert torch.isfinite(out.float()).all().item(), variant
    return res


def describe_attention(name: str, cfg: dict) -> str:
    causal = cfg["causal"]
    return (f"{name}: {'causal' if causal else 'non-causal'} attention, {cfg['dtype']} in / f32 accumulate, "
            f"B={cfg['B']} H={cfg['H']} L={cfg['L']} d={cfg['d']} M={cfg['M']}"
            + (f" chunk={cfg.get('chunk', 0)}" if causal else "") + ", SDERF per head, theta and omega resident"
            + (" (projection constants prepared once: favorsharp_attention_prepared)" if cfg["dtype"] == "bf16" else ""))


def summary_of(r: dict) -> dict:
    rf = r["roofline"]
    return {"ms_per_step": r["ms_per_step"], "ms_per_step_unprepared": r["ms_per_step_unprepared"],
            "tokens_per_s": r["tokens_per_s"], "main_kernel_ms": r["main_kernel_ms"],
            "roofline": {"bound": rf["bound"], "frac": rf["frac"], "step_frac": rf["call_frac"], "unit": rf["unit"],
                         "achieved": rf["achieved"], "peak": rf["peak"], "traffic": rf["traffic"]}}


# ---------------------------------------------------------------------------------------------- kernel operator
def run_matvec(steps: int, warmup: int, fs, synth, torch) -> dict:
    """c2, the kernel operator K^(alpha)(X, Y) C of Section 2.1: one step = one favorsharp_kernel_matvec call with
    theta and omega resident; fp32 in and out, so the bound is the fp32 MFMA peak."""
    cfg = dict(synth.WORKLOADS["c2"])
    N, d, M, n, alpha = cfg["N"], cfg["d"], cfg["M"], cfg["n"], cfg["alpha"]
    sets, w0 = [], None
    for i in range(3):
        w = synth.make("c2", seed=cfg["seed"] + i)
        w0 = w0 or w
        X = torch.from_numpy(w["X"].astype(np.float32)).cuda()
        C = torch.from_numpy(w["C"].astype(np.float32)).cuda()
        Om = torch.from_numpy(w["Omega"].astype(np.float32)).cuda()
        theta = fs.fit_params("sderf", X, X, w["qk_scale"], groups=1)
        sets.append((theta, X, C, Om, w["qk_scale"]))
    ws = torch.empty(fs.kernel_matvec_workspace_bytes(N, N, d, M, n), dtype=torch.uint8, device="cuda")
    last = {}

    def step(i):
        theta, X, C, Om, s = sets[i % 3]
        last[i % 3] = fs.kernel_matvec(theta, X, X, s, alpha, Om, C, workspace=ws)

    ms = timed(step, steps, warmup, torch)
    assert torch.isfinite(last[0]).all().item()
    flops = N * (2 * 2 * d * M + 2 * 2 * M * n)          # two projections, state update and state read
    tf = flops / (ms * 1e-3) / 1e12
    return dict(cfg=cfg, w0=w0, theta0=sets[0][0], out0=last[0], ms_per_step=ms, points_per_s=N / (ms * 1e-3),
                roofline={"bound": "mfma", "achieved": tf, "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                          "frac": tf / MFMA_F32_PEAK_TFLOPS, "step_frac": tf / MFMA_F32_PEAK_TFLOPS, "traffic": None})


# ---------------------------------------------------------------------------------------------- backward pass
def run_backward(name: str, steps: int, warmup: int, fs, synth, torch) -> dict:
    """Backward pass of attention on the c3 (non-causal) or c4 (causal) shapes, bf16 inputs and gradients: one step =
    one favorsharp_attention_backward_prepared call with theta, omega and the projection constants derived from
    them resident (`ms_per_step_unprepared`: favorsharp_attention_backward, which rebuilds the constants); bf16 MFMA
    kernels; bound: the bf16 MFMA peak.  Algorithmic flops per head-token: the two projections twice (features are rebuilt, and dE W) 8 d M, six
    M x (dv + 1) contractions (T, P T, G1 T^T, P^T G1, S R, [V 1] R^T) 12 M (dv + 1), and when causal the
    intra-chunk triangles of 64 rows (three times the forward pass's extra term)."""
    cfg = dict(synth.WORKLOADS[name])
    B, H, L, d, M, causal = cfg["B"], cfg["H"], cfg["L"], cfg["d"], cfg["M"], bool(cfg["causal"])
    nsets = 3 if name == "c3" else 2
    sets, w0, dY0 = [], None, None
    for i in range(nsets):
        w = synth.make(name, seed=cfg["seed"] + i)
        rng = np.random.default_rng(900 + i)
        dY = synth.round_to_bf16(rng.standard_normal(w["V"].shape).astype(np.float32))
        if w0 is None:
            w0, dY0 = w, dY
        Q, K, V = (fs.to_device(w[k], "bf16") for k in "QKV")
        theta = fs.fit_params("sderf", Q, K, w["qk_scale"], groups=H)
        Om = torch.from_numpy(w["Omega"]).cuda()
        sets.append((theta, Q, K, V, fs.to_device(dY, "bf16"), Om, w["qk_scale"],
                     fs.attention_prepare(theta, Om, B, H, w["qk_scale"])))
    ws = torch.empty(fs.attention_backward_workspace_bytes(B, H, L, L, d, d, M, causal, H, H), dtype=torch.uint8,
                     device="cuda")
    last = {}

    def step_unprepared(i):
        theta, Q, K, V, dY, Om, s, _ = sets[i % nsets]
        last[i % nsets] = fs.attention_backward(theta, Q, K, V, dY, s, Om, causal=causal, workspace=ws)

    # the step: projection constants prepared once per parameter set, as in the forward workloads
    def step(i):
        theta, Q, K, V, dY, Om, s, prep = sets[i % nsets]
        last[i % nsets] = fs.attention_backward(theta, Q, K, V, dY, s, Om, causal=causal, workspace=ws, prepared=prep)

    ms_unprepared = timed(step_unprepared, steps, warmup, torch)
    ms = timed(step, steps, warmup, torch)
    assert all(torch.isfinite(g.float()).all().item() for g in last[0])
    # the same call with ADERF parameters (dense C2: row-term kernel, dense derivative of the row term), first set
    _, Q, K, V, dY, Om, s, _ = sets[0]
    theta_a = fs.fit_params("aderf", Q, K, s, groups=H)
    prep_a = fs.attention_prepare(theta_a, Om, B, H, s)
    grads_a = {}

    def step_aderf(i):
        grads_a[0] = fs.attention_backward(theta_a, Q, K, V, dY, s, Om, causal=causal, workspace=ws, prepared=prep_a)

    ms_aderf = timed(step_aderf, steps, warmup, torch)
    assert all(torch.isfinite(g.float()).all().item() for g in grads_a[0])
    chunk = cfg.get("chunk", 64)
    per_token = 8 * d * M + 12 * M * (d + 1) + (3 * (chunk + 1) // 2 * (2 * M + 2 * (d + 1)) if causal else 0)
    tf = B * H * L * per_token / (ms * 1e-3) / 1e12
    return dict(cfg=cfg, w0=w0, dY0=dY0, theta0=sets[0][0], grads0=last[0], ms_per_step=ms, ms_per_step_aderf=ms_aderf,
                ms_per_step_unprepared=ms_unprepared,
                tokens_per_s=B * L / (ms * 1e-3),
                roofline={"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                          "frac": tf / MFMA_BF16_PEAK_TFLOPS, "step_frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": None})


def run_many_sequences(steps: int, warmup: int, fs, synth, torch, oracle) -> tuple:
    """Outside the five configurations: the d = 64 / M = 256 kernels on MANY SHORT sequences (512 x 8 sequences of 128
    tokens with the c3 recipe, the shape of an encoder's training batch), where a state is more bytes than a
    sequence's rows: forward and backward, without and with the mask, ms per call, theta and omega resident.  The
    non-causal calls run one workgroup per sequence (k_fast_whole, k_bwd_whole); the causal ones have one slot per
    sequence (no state pass, no scan).  Parity: three whole sequences of every call against the CPU oracle."""
    B, H, L = 512, 8, 128
    w = synth.make("c3", B=B, H=H, L=L)
    d, M, s = w["d"], w["M"], w["qk_scale"]
    rng = np.random.default_rng(977)
    dY = synth.round_to_bf16(rng.standard_normal(w["V"].shape).astype(np.float32))
    Q, K, V, dYd = (fs.to_device(a, "bf16") for a in (w["Q"], w["K"], w["V"], dY))
    Om = torch.from_numpy(w["Omega"]).cuda()
    theta = fs.fit_params("sderf", Q, K, s, groups=H)
    prepared = fs.attention_prepare(theta, Om, B, H, s)
    out = {"workload": f"many short sequences: B={B} H={H} L={L} d={d} M={M}, bf16, SDERF per head, theta and omega "
                       "resident (not one of the five configurations)", "attention_ms": {}, "backward_ms": {}}
    worst = [0.0, 0.0]
    th_host = fs.to_host(theta).astype(np.float32)
    for causal in (False, True):
        key = "causal" if causal else "non_causal"
        ws = torch.empty(fs.attention_backward_workspace_bytes(B, H, L, L, d, d, M, causal, H, H), dtype=torch.uint8,
                         device="cuda")
        wf = torch.empty(fs.attention_workspace_bytes(B, H, L, L, d, d, M, causal, H, H), dtype=torch.uint8, device="cuda")
        Y = torch.empty_like(Q)
        grads = tuple(torch.empty_like(Q) for _ in range(3))
        out["attention_ms"][key] = timed(lambda i: fs.attention_prepared(prepared, theta, Q, K, V, s, Om, causal=causal,
                                                                         chunk=64 if causal else 0, out=Y, workspace=wf),
                                         steps, warmup, torch)
        out["backward_ms"][key] = timed(lambda i: fs.attention_backward(theta, Q, K, V, dYd, s, Om, causal=causal,
                                                                        workspace=ws, grads=grads, prepared=prepared),
                                        steps, warmup, torch)
        if oracle:
            for b, h in ((0, 0), (17, 3), (B - 1, H - 1)):
                th = oracle.theta(th_host[h], d)
                args = (th, w["Omega"][h], w["Q"][b, h], w["K"][b, h], w["V"][b, h])
                fro, row = oracle.errors(fs.to_host(Y[b, h]), oracle.orc.attention(*args, s, causal), w["V"][b, h].astype(np.float64))
                worst = [max(worst[0], fro), max(worst[1], row)]
                for g, rf in zip(grads, oracle.orc.attention_backward(*args, dY[b, h], s, causal)):
                    fro, row = oracle.errors(fs.to_host(g[b, h]), rf, rf)
                    worst = [max(worst[0], fro), max(worst[1], row)]
        del ws, wf, Y, grads
    parity = {"reference": "CPU oracle (fp64), same inputs, omega and float32 parameter block",
              "rows": "every row of Y, dQ, dK, dV of three (b,h) sequences, without and with the mask",
              "worst_frobenius": worst[0], "worst_row": worst[1], "tol_frobenius": 2e-2, "tol_row": 8e-2,
              "ok": bool(worst[0] <= 2e-2 and worst[1] <= 8e-2)} if oracle else None
    torch.cuda.empty_cache()
    return out, parity


# ---------------------------------------------------------------------------------------------- CPU oracle leg
class OracleLeg:
    """Everything that touches the CPU oracle: the timed baseline and the parity figures.  Both sides see the same
    inputs, the same omega and the library's own float32 parameter block (downloaded and handed to the oracle)."""

    def __init__(self, fs):
        from oracle import favorsharp_oracle as orc
        self.orc, self.fs, self.cores = orc, fs, host_cores()

    def theta(self, vec, d):
        u = self.fs.unpack_theta(vec, d)
        f = lambda a: np.asarray(a, dtype=np.float64)
        return self.orc.Theta(A=f(u["A"]), B1=f(u["B1"]), B2=f(u["B2"]), C1=f(u["C1"]), C2=f(u["C2"]), logD=float(u["logD"]))

    @staticmethod
    def errors(got, ref, scale_rows):
        diff = got - ref
        fro = float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-300))
        row = float(np.linalg.norm(diff, axis=1).max() / max(np.linalg.norm(scale_rows, axis=1).max(), 1e-300))
        return fro, row

    def attention_full(self, r: dict, budget_s: float):
        """Whole (b, h) sequences of an attention workload until `budget_s` is spent: the oracle's own fit (timed, as
        part of the baseline) and the oracle's attention at the library's parameter block (timed; it is also the
        parity reference)."""
        orc, w, cfg = self.orc, r["w0"], r["cfg"]
        s, d, H = w["qk_scale"], w["d"], w["H"]
        th_host = self.fs.to_host(r["theta0"]).astype(np.float32)
        Y = r["Y0"]
        pairs = [(b, h) for b in range(w["B"]) for h in range(H)]
        done, worst, dt = 0, [0.0, 0.0], 0.0
        for b, h in pairs:
            t0 = time.perf_counter()
            orc.fit_sderf(s * w["Q"][:, h].reshape(-1, d).astype(np.float64), s * w["K"][:, h].reshape(-1, d).astype(np.float64))
            ref = orc.attention(self.theta(th_host[h], d), w["Omega"][h], w["Q"][b, h], w["K"][b, h], w["V"][b, h], s, cfg["causal"])
            dt += time.perf_counter() - t0               # the comparison below is not part of the baseline's time
            fro, row = self.errors(self.fs.to_host(Y[b, h]), ref, w["V"][b, h].astype(np.float64))
            worst = [max(worst[0], fro), max(worst[1], row)]
            done += 1
            if dt > budget_s:
                break
        tol = TOL[cfg["dtype"]]
        parity = {"reference": "CPU oracle (fp64), same inputs, omega and float32 parameter block",
                  "rows": f"every row of {done} of {len(pairs)} (b,h) sequences", "worst_frobenius": worst[0],
                  "worst_row": worst[1], "tol_frobenius": tol, "tol_row": 4 * tol,
                  "ok": bool(worst[0] <= tol and worst[1] <= 4 * tol)}
        base = dict(value=done * w["L"] / dt / H, unit="tokens/s", cores=self.cores, kind="oracle",
                    sample=f"{done} of {len(pairs)} (b,h) sequences of L={w['L']} (fit + attention, fp64 numpy), "
                           f"{dt:.1f} s; head-tokens/s divided by H={H}")
        return base, parity

    def attention_sampled(self, r: dict, npairs: int, nrows: int):
        """Sampled output rows, evaluated one by one from the definition (rows of K_hat, masked when causal)."""
        import torch
        orc, w, cfg = self.orc, r["w0"], r["cfg"]
        s, d, B, H, L = w["qk_scale"], w["d"], w["B"], w["H"], w["L"]
        th_host = self.fs.to_host(r["theta0"]).astype(np.float32)
        rng = np.random.default_rng(9)
        fixed = [0, 1, 63, 64, 65, L // 2 - 1, L // 2, L - 2, L - 1]
        worst, total = [0.0, 0.0], 0
        for b, h in [(0, 0), (B - 1, H - 1), (B // 2, H // 2)][:npairs]:
            rows = np.unique(np.concatenate([fixed, rng.integers(0, L, nrows)]))
            ref = orc.attention_khat_definition(self.theta(th_host[h], d), w["Omega"][h], w["Q"][b, h], w["K"][b, h],
                                                w["V"][b, h], s, cfg["causal"], rows=rows)
            got = self.fs.to_host(r["Y0"][b, h][torch.from_numpy(rows).cuda()])
            fro, row = self.errors(got, ref, w["V"][b, h].astype(np.float64))
            worst = [max(worst[0], fro), max(worst[1], row)]
            total += len(rows)
        tol = TOL[cfg["dtype"]]
        return {"reference": "CPU oracle (fp64), rows of K_hat from the definition, same inputs, omega and parameter block",
                "rows": f"{total} sampled rows of {npairs} (b,h) sequences", "worst_frobenius": worst[0],
                "worst_row": worst[1], "tol_frobenius": tol, "tol_row": 4 * tol,
                "ok": bool(worst[0] <= tol and worst[1] <= 4 * tol)}

    def matvec(self, r: dict):
        orc, w = self.orc, r["w0"]
        Xs = w["qk_scale"] * w["X"].astype(np.float64)
        th = self.theta(self.fs.to_host(r["theta0"]).astype(np.float32)[0], w["d"])
        t0 = time.perf_counter()
        orc.fit_sderf(Xs, Xs)
        ref = orc.kernel_matvec(th, w["Omega"][0], Xs, Xs, w["C"].astype(np.float64), w["alpha"])
        dt = time.perf_counter() - t0
        got = self.fs.to_host(r["out0"])
        fro = float(np.linalg.norm(got - ref) / np.linalg.norm(ref))
        worst_el = float(np.abs(got - ref).max() / np.abs(ref).max())
        parity = {"reference": "CPU oracle (fp64), the whole operator, same inputs, omega and parameter block",
                  "rows": "all", "worst_frobenius": fro, "worst_element_over_max": worst_el, "tol_frobenius": 1e-4,
                  "ok": bool(fro <= 1e-4)}
        base = dict(value=w["N"] / dt, unit="points/s", cores=self.cores, kind="oracle",
                    sample=f"the whole workload once (fit + operator, fp64 numpy), {dt:.2f} s")
        return base, parity

    def backward(self, r: dict):
        """One whole (b, h) sequence of a backward workload: every gradient row."""
        orc, w, cfg = self.orc, r["w0"], r["cfg"]
        s, d = w["qk_scale"], w["d"]
        th = self.theta(self.fs.to_host(r["theta0"]).astype(np.float32)[0], d)
        ref = orc.attention_backward(th, w["Omega"][0], w["Q"][0, 0], w["K"][0, 0], w["V"][0, 0], r["dY0"][0, 0], s, cfg["causal"])
        worst = [0.0, 0.0]
        for g, rf in zip(r["grads0"], ref):
            fro, row = self.errors(self.fs.to_host(g[0, 0]), rf, rf)
            worst = [max(worst[0], fro), max(worst[1], row)]
        return {"reference": "CPU oracle (fp64) gradients of sum(Y * dY), same inputs, omega and parameter block",
                "rows": "every row of dQ, dK, dV of one (b,h) sequence", "worst_frobenius": worst[0],
                "worst_row": worst[1], "tol_frobenius": 2e-2, "tol_row": 8e-2,
                "ok": bool(worst[0] <= 2e-2 and worst[1] <= 8e-2)}


def free(r: dict, torch):
    for k in ("sets", "Y0", "theta0", "grads0", "out0", "w0", "dY0"):
        r.pop(k, None)
    torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the clocks of the chip settle only after some tens of milliseconds of load (the first calls of a process run
    # the main kernel about 15 % slower than the steady state): the default warm-up covers that
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5", "c3_backward", "c4_backward"],
                    help="the workload of the headline fields (default: the metric workload, c4)")
    ap.add_argument("--only", action="store_true",
                    help="time the headline workload only (no `workloads` object): for profiling runs")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the CPU oracle leg (no baseline, no parity)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device-to-device copy (a kernel of known traffic, for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2302_00787_amd import binding as fs
    from paper_2302_00787_amd import synth

    fs.lib()
    oracle = None if args.no_cpu_baseline else OracleLeg(fs)
    base = {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "data": "synthetic"}
    parity = {}

    # ---- headline workload
    name = args.workload
    if name == "c2":
        r = run_matvec(args.steps, args.warmup, fs, synth, torch)
        result = {"metric": "FAVOR# kernel operator points/s (c2: N=16384 d=32 M=512 n=8, alpha=-1/2)",
                  "value": r["points_per_s"], "unit": "points/s", **base, "ms_per_step": r["ms_per_step"], "dtype": "f32",
                  "config": {"workload": "c2: kernel operator, fp32, X = Y, SDERF, theta and omega resident"},
                  "roofline": r["roofline"]}
        if oracle:
            result["cpu_baseline"], parity["c2"] = oracle.matvec(r)
    elif name.endswith("_backward"):
        short = name.split("_")[0]
        r = run_backward(short, args.steps, args.warmup, fs, synth, torch)
        cfg = r["cfg"]
        result = {"metric": f"FAVOR# attention backward tokens/s ({short} shapes)", "value": r["tokens_per_s"],
                  "unit": "tokens/s", **base, "ms_per_step": r["ms_per_step"], "dtype": "bf16",
                  "config": {"workload": f"{name}: gradients of {'causal' if cfg['causal'] else 'non-causal'} attention "
                                         f"w.r.t. Q, K, V, bf16 in and out, B={cfg['B']} H={cfg['H']} L={cfg['L']} "
                                         f"d={cfg['d']} M={cfg['M']}, SDERF per head, theta and omega resident"},
                  "ms_per_step_unprepared": r["ms_per_step_unprepared"],
                  "families_ms": {"aderf": r["ms_per_step_aderf"]}, "roofline": r["roofline"]}
        if oracle:
            parity[name] = oracle.backward(r)
    else:
        r = run_attention(name, args.steps, args.warmup, fs, synth, torch, nsets=2 if name == "c5" else 3,
                          with_fit=True, calibrate_copy=args.calibrate_copy)
        cfg = r["cfg"]
        result = {
            "metric": "FAVOR# attn tokens/s, causal L=16k d=64 M=256; % of MFMA/HBM roofline" if name == "c4"
                      else f"FAVOR# attn tokens/s ({name})",
            "value": r["tokens_per_s"], "unit": "tokens/s", **base, "ms_per_step": r["ms_per_step"],
            "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32",
            "config": {"workload": describe_attention(name, cfg)},
            "head_tokens_per_s": cfg["B"] * cfg["H"] * cfg["L"] / (r["ms_per_step"] * 1e-3),
            "fit_ms": r["fit_ms"], "fit_device_ms": r["fit_device_ms"], "main_kernel_ms": r["main_kernel_ms"],
            # the same call with the projection constants rebuilt inside it (favorsharp_attention)
            "ms_per_step_unprepared": r["ms_per_step_unprepared"],
            "algorithmic_tflops": r["counts"]["flops"] / (r["ms_per_step"] * 1e-3) / 1e12,
            # dominant kernel (k_fast_causal / k_fast_apply / k_wide_walk / the generic equivalents) in `frac`, the whole
            # call in `call_frac`, both against the tighter of the two bounds on the algorithmic counts
            "roofline": r["roofline"],
        }
        if oracle:
            if name in ("c1", "c4"):
                result["cpu_baseline"], parity[name] = oracle.attention_full(r, 20.0 if name == "c4" else 5.0)
            else:
                parity[name] = oracle.attention_sampled(r, 2, 24)
        if not args.only and name == "c4":
            # (after the oracle leg the chip has been idle for seconds: the full warm-up, for the clocks)
            result["families_ms"] = run_families(r, max(5, min(args.steps, 100)), args.warmup, fs, torch)
    free(r, torch)

    # ---- the other workloads, same run, fewer steps
    if not args.only and name == "c4":
        steps, warmup = max(5, min(args.steps, 50)), max(2, min(args.warmup, 25))
        others = {}
        for other in ("c1", "c3", "c5"):
            r = run_attention(other, steps, warmup, fs, synth, torch, nsets=2 if other == "c5" else 3, with_fit=other == "c5")
            others[other] = summary_of(r)
            others[other]["workload"] = describe_attention(other, r["cfg"])
            if other == "c5":
                others[other]["fit_ms"], others[other]["fit_device_ms"] = r["fit_ms"], r["fit_device_ms"]
            if other != "c1":
                others[other]["families_ms"] = run_families(r, steps, warmup if other == "c5" else args.warmup, fs, torch)
            if oracle:
                # whole sequences, every row (c3: all 64 fit in the budget; c5: as many of its 16 as 10 s of the oracle
                # allow), and for the long workloads also sampled rows straight from the definition of K_hat
                parity[other] = oracle.attention_full(r, {"c1": 5.0, "c3": 10.0, "c5": 10.0}[other])[1]
                if other != "c1":
                    parity[other]["sampled_rows_from_the_definition"] = oracle.attention_sampled(r, 2, 24)
            free(r, torch)
        r = run_matvec(steps, warmup, fs, synth, torch)
        others["c2"] = {"ms_per_step": r["ms_per_step"], "points_per_s": r["points_per_s"], "main_kernel_ms": None,
                        "roofline": r["roofline"],
                        "workload": "c2: kernel operator, fp32, N=16384 d=32 M=512 n=8, alpha=-1/2, X = Y, SDERF"}
        if oracle:
            others["c2"]["cpu_baseline"], parity["c2"] = oracle.matvec(r)
        free(r, torch)
        for short in ("c3", "c4"):
            r = run_backward(short, steps, warmup, fs, synth, torch)
            others[f"{short}_backward"] = {"ms_per_step": r["ms_per_step"],
                                           "ms_per_step_unprepared": r["ms_per_step_unprepared"],
                                           "tokens_per_s": r["tokens_per_s"],
                                           "main_kernel_ms": None, "roofline": r["roofline"],
                                           "families_ms": {"aderf": r["ms_per_step_aderf"]},
                                           "workload": f"{short} shapes: gradients w.r.t. Q, K, V, bf16 in and out"}
            if oracle:
                parity[f"{short}_backward"] = oracle.backward(r)
            free(r, torch)
        others["many_short_sequences"], p = run_many_sequences(steps, warmup, fs, synth, torch, oracle)
        if oracle:
            parity["many_short_sequences"] = p
        result["workloads"] = others
        result["workloads_steps"], result["workloads_warmup"] = steps, warmup
    if oracle:
        result["parity"] = parity
    elif "cpu_baseline" not in result:
        result["cpu_baseline"] = None
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
