#!/usr/bin/env python3
"""Benchmark of the FAVOR# hot path on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4] [--no-cpu-baseline]

One "step" is one call of favorsharp_attention on the metric workload (causal, bf16, B=4 H=8 L=16384 d=64
M=256, chunk 64): projection constants, both feature maps (fused, never stored) and the causal prefix-state
contraction, with Q, K, V, omega and the fitted parameters already resident in HBM.  The closed-form fit
(statistics scan on the GPU + d x d algebra on the host) is timed separately and reported as `fit_ms`, the
device-resident variant of the same fit as `fit_device_ms`.
Inputs rotate over three distinct sets so the 256 MB last-level cache cannot hold a set across steps.

Prints ONE JSON line: throughput in tokens/s (B*L per step), the roofline of the dominant kernel measured
with HIP events recorded by the library around that kernel, and the CPU oracle timed on a bounded sample.
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
# HBM bytes per launch of the dominant kernel, from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of this
# script with --calibrate-copy, each counter scaled by what it reads for the 256 MiB copy (FETCH_SIZE x 2.0,
# WRITE_SIZE x 1.0); figures and commands in profiles/c4_hbm_traffic.md.  The kernel reads Q, K, V and the prefix
# states once and writes Y once, so the figure does not depend on how its instructions are scheduled.
MEASURED_TRAFFIC_BYTES = {"c4": 291.9e6, "c3": 111.6e6, "c5": 3.31e9}     # c3, c5: profiles/c3_c5_hbm_traffic.md


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
    return dict(head_tokens=ht, bytes=ht * 4 * d * esz, flops=ht * flops)


def cpu_baseline(w: dict, budget_s: float = 20.0) -> dict:
    """The CPU oracle, as it stands, on whole (b, h) sequences of the same workload until ~budget_s is spent."""
    from oracle import favorsharp_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    s, d = w["qk_scale"], w["d"]
    done, t0 = 0, time.perf_counter()
    pairs = [(b, h) for b in range(w["B"]) for h in range(w["H"])]
    for b, h in pairs:
        th = orc.fit_sderf(s * w["Q"][:, h].reshape(-1, d).astype(np.float64),
                           s * w["K"][:, h].reshape(-1, d).astype(np.float64))
        orc.attention(th, w["Omega"][h], w["Q"][b, h], w["K"][b, h], w["V"][b, h], s, w["causal"])
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    head_tokens_per_s = done * w["L"] / dt
    return dict(value=head_tokens_per_s / w["H"], unit="tokens/s", cores=int(cores), kind="oracle",
                sample=f"{done} of {len(pairs)} (b,h) sequences of L={w['L']} (fit + attention, fp64 numpy), "
                       f"{dt:.1f} s; head-tokens/s divided by H={w['H']}")


def bench_matvec(args, cfg, fs, synth, util, torch):
    """The kernel-operator workload (K^(alpha)(X, Y) C, Section 2.1): one step = one favorsharp_kernel_matvec call
    with theta and omega resident; fp32 in and out, so the bound is the fp32 MFMA peak."""
    N, d, M, n, alpha = cfg["N"], cfg["d"], cfg["M"], cfg["n"], cfg["alpha"]
    sets = []
    for i in range(3):
        w = synth.make(args.workload, seed=cfg["seed"] + i)
        X = torch.from_numpy(w["X"].astype(np.float32)).cuda()
        C = torch.from_numpy(w["C"].astype(np.float32)).cuda()
        Om = torch.from_numpy(w["Omega"].astype(np.float32)).cuda()
        theta = fs.fit_params("sderf", X, X, w["qk_scale"], groups=1)
        sets.append((theta, X, C, Om, w["qk_scale"]))
    ws = torch.empty(fs.kernel_matvec_workspace_bytes(N, N, d, M, n), dtype=torch.uint8, device="cuda")

    def step(i):
        theta, X, C, Om, s = sets[i % 3]
        return fs.kernel_matvec(theta, X, X, s, alpha, Om, C, workspace=ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        out = step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    assert torch.isfinite(out).all().item()
    flops = N * (2 * 2 * d * M + 2 * 2 * M * n)          # two projections, state update and state read
    tf = flops / (ms * 1e-3) / 1e12
    cpu = None
    if not args.no_cpu_baseline:
        # the oracle on the whole operator (fit + both feature maps + the two products), fp64 numpy
        from oracle import favorsharp_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        w = synth.make(args.workload, seed=cfg["seed"])
        t1 = time.perf_counter()
        Xs = w["qk_scale"] * w["X"].astype(np.float64)
        orc.kernel_matvec(orc.fit_sderf(Xs, Xs), w["Omega"][0], Xs, Xs, w["C"].astype(np.float64), alpha)
        dtc = time.perf_counter() - t1
        cpu = dict(value=N / dtc, unit="points/s", cores=int(cores), kind="oracle",
                   sample=f"the whole workload once (fit + operator, fp64 numpy), {dtc:.2f} s")
    print(json.dumps({
        "metric": "FAVOR# kernel operator points/s (c2: N=16384 d=32 M=512 n=8, alpha=-1/2)", "value": N / (ms * 1e-3),
        "unit": "points/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "c2: kernel operator, fp32, X = Y, SDERF, theta and omega resident"},
        "roofline": {"bound": "mfma", "achieved": tf, "peak": 157.3, "unit": "TFLOP/s", "frac": tf / 157.3,
                     "traffic": None},
        "cpu_baseline": cpu}), flush=True)


def bench_backward(args, fs, synth, util, torch):
    """The backward pass of attention on the c3 (non-causal) or c4 (causal) shapes, bf16 inputs and gradients: one
    step = one favorsharp_attention_backward call with theta and omega resident.  Both run on the bf16 MFMA kernels
    (bound: the bf16 MFMA peak).  Algorithmic flops per
    head-token: the two projections twice (features are rebuilt, and dE W) 8 d M, six M x (dv + 1) contractions
    (T, P T, G1 T^T, P^T G1, S R, [V 1] R^T) 12 M (dv + 1), and when causal the intra-chunk triangles of 64 rows
    (scores and G1 V1^T and their four products: three times the forward pass's extra term)."""
    name = args.workload.split("_")[0]
    cfg = dict(synth.WORKLOADS[name])
    B, H, L, d, M, causal = cfg["B"], cfg["H"], cfg["L"], cfg["d"], cfg["M"], bool(cfg["causal"])
    nsets = 3 if name == "c3" else 2
    sets = []
    for i in range(nsets):
        w = synth.make(name, seed=cfg["seed"] + i)
        rng = np.random.default_rng(900 + i)
        Q, K, V = (util.to_device(w[k], "bf16") for k in "QKV")
        dY = util.to_device(synth.round_to_bf16(rng.standard_normal(w["V"].shape).astype(np.float32)), "bf16")
        theta = fs.fit_params("sderf", Q, K, w["qk_scale"], groups=H)
        sets.append((theta, Q, K, V, dY, torch.from_numpy(w["Omega"]).cuda(), w["qk_scale"]))
    ws = torch.empty(fs.attention_backward_workspace_bytes(B, H, L, L, d, d, M, causal, H, H), dtype=torch.uint8,
                     device="cuda")

    def step(i):
        theta, Q, K, V, dY, Om, s = sets[i % nsets]
        return fs.attention_backward(theta, Q, K, V, dY, s, Om, causal=causal, workspace=ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        grads = step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    assert all(torch.isfinite(g.float()).all().item() for g in grads)
    chunk = cfg.get("chunk", 64)
    per_token = 8 * d * M + 12 * M * (d + 1) + (3 * (chunk + 1) // 2 * (2 * M + 2 * (d + 1)) if causal else 0)
    flops = B * H * L * per_token
    tf = flops / (ms * 1e-3) / 1e12
    peak = MFMA_BF16_PEAK_TFLOPS
    print(json.dumps({
        "metric": f"FAVOR# attention backward tokens/s ({name} shapes: {'causal' if causal else 'non-causal'}, "
                  f"B={B} H={H} L={L} d={d} M={M})",
        "value": B * L / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: gradients of {'causal' if causal else 'non-causal'} attention w.r.t. "
                               "Q, K, V, bf16 in and out, "
                               "bf16 MFMA kernels, fp32 accumulation, SDERF per head, theta and omega resident"},
        "roofline": {"bound": "mfma", "achieved": tf, "peak": peak, "unit": "TFLOP/s", "frac": tf / peak,
                     "traffic": None}}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5", "c3_backward", "c4_backward"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    from tests import util

    fs.lib()
    if args.workload.endswith("_backward"):
        bench_backward(args, fs, synth, util, torch)
        return
    cfg = dict(synth.WORKLOADS[args.workload])
    if cfg.get("kind") == "matvec":
        bench_matvec(args, cfg, fs, synth, util, torch)
        return
    dtype = cfg["dtype"]
    nsets = 3
    sets, w0 = [], None
    for i in range(nsets):
        w = synth.make(args.workload, seed=cfg["seed"] + i)
        w0 = w0 or w
        sets.append(dict(Q=util.to_device(w["Q"], dtype), K=util.to_device(w["K"], dtype),
                         V=util.to_device(w["V"], dtype), Omega=torch.from_numpy(w["Omega"]).cuda()))
    s = w0["qk_scale"]
    B, H, L, d, M = cfg["B"], cfg["H"], cfg["L"], cfg["d"], cfg["M"]
    causal, chunk = cfg["causal"], cfg.get("chunk", 0)

    # fit (timed separately): statistics on the GPU, closed form on the host
    for st_ in sets:
        st_["theta"] = fs.fit_params("sderf", st_["Q"], st_["K"], s, groups=H)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    fs.fit_params("sderf", sets[0]["Q"], sets[0]["K"], s, groups=H)
    torch.cuda.synchronize()
    fit_ms = (time.perf_counter() - t0) * 1e3
    # the same fit with the closed form on the device (asynchronous entry point; the timing includes the final sync)
    fit_ws = torch.empty(fs.fit_device_workspace_bytes(B, H, L, L, d, H), dtype=torch.uint8, device="cuda")
    fs.fit_params_device("sderf", sets[0]["Q"], sets[0]["K"], s, groups=H, workspace=fit_ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    _, fit_status = fs.fit_params_device("sderf", sets[0]["Q"], sets[0]["K"], s, groups=H, workspace=fit_ws)
    torch.cuda.synchronize()
    fit_device_ms = (time.perf_counter() - t0) * 1e3
    assert int(fit_status.abs().sum().item()) == 0

    nbytes = fs.attention_workspace_bytes(B, H, L, L, d, d, M, causal, H, H)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    outs = [torch.empty_like(st_["V"]) for st_ in sets]
    ev = HipEvents()
    pairs = [(ev.create(), ev.create()) for _ in range(args.steps)]

    def step(i, events=None):
        st_ = sets[i % nsets]
        fs.attention(st_["theta"], st_["Q"], st_["K"], st_["V"], s, st_["Omega"], causal=causal, chunk=chunk,
                     out=outs[i % nsets], workspace=ws, events=events)

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, pairs[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    main_ms = float(np.mean([ev.elapsed_ms(a, b) for a, b in pairs]))
    for a, b in pairs:
        ev.destroy(a)
        ev.destroy(b)
    assert all(torch.isfinite(o.float()).all().item() for o in outs)

    ms_per_step = dt / args.steps * 1e3
    counts = algorithmic_counts(cfg)
    achieved = counts["bytes"] / (main_ms * 1e-3) / 1e9
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if dtype == "bf16" else 157.3
    kernel_tflops = counts["flops"] / (main_ms * 1e-3) / 1e12
    extra = {"kernel_hbm_gbs": achieved, "kernel_hbm_frac": achieved / HBM_PEAK_GBS,
             "kernel_mfma_tflops": kernel_tflops, "kernel_mfma_frac": kernel_tflops / mfma_peak,
             "step_hbm_frac": counts["bytes"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
             "step_mfma_frac": counts["flops"] / (ms_per_step * 1e-3) / 1e12 / mfma_peak}
    if counts["bytes"] / (HBM_PEAK_GBS * 1e9) >= counts["flops"] / (mfma_peak * 1e12):
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload), **extra}
    else:
        roofline = {"bound": "mfma", "achieved": kernel_tflops, "peak": mfma_peak, "unit": "TFLOP/s",
                    "frac": kernel_tflops / mfma_peak, "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload), **extra}
    result = {
        "metric": "FAVOR# attn tokens/s, causal L=16k d=64 M=256; % of MFMA/HBM roofline",
        "value": B * L / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {'causal' if causal else 'non-causal'} attention, {dtype} in / f32 "
                               f"accumulate, B={B} H={H} L={L} d={d} M={M}"
                               + (f" chunk={chunk}" if causal else "") + ", SDERF per head, theta and omega resident"},
        "head_tokens_per_s": B * H * L / (ms_per_step * 1e-3),
        "fit_ms": fit_ms,
        "fit_device_ms": fit_device_ms,
        "main_kernel_ms": main_ms,
        "algorithmic_tflops": counts["flops"] / (ms_per_step * 1e-3) / 1e12,
        # dominant kernel (k_fast_causal / k_fast_apply / k_wide_walk / the generic equivalents), against the tighter
        # of the two rooflines on the algorithmic counts (c4: 33.6 us of HBM time against 32.1 us of MFMA time; c5 is on
        # the MFMA side); the other one is reported beside it
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w0)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
