#!/usr/bin/env python3
"""Benchmark of the DoRA module hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input, inputs resident in HBM before
the timed region starts.  What the pass is depends on the workload (--config):

  C1  fp32, 256 x 512, r 16, 64 tokens: forward (factored norm inside).  Launch-latency bound.
  C2  bf16, 4096 x 4096, r 384, 4096 tokens: forward (norm + contractions + compose).
  C3  bf16, 8192 x 8192, r 384, 8192 tokens (the headline, default): forward saving h / inner / w_norm,
      then backward (compose backward with the fused dm reduction, dh, dx, dA, dB).
  C4  bf16 MLP pair, up 5120 -> 27648 and down 27648 -> 5120, r 384, 8192 tokens: forward of both modules
      keeping nothing, then backward of both in reverse order with everything recomputed (norm, h, inner):
      the gradient-checkpointing pattern.  tokens/s = 8192 / (t_up + t_down).
  C5  bf16 decoder-layer sweep, 8B-class shapes: seven adapted modules x 32 layers, all 224 resident,
      forward in order then recompute + backward in reverse order, at r = 64, 384 and 768; 4096 tokens.
      Reports aggregate tokens/s (4096 / time of one sweep) and peak device memory per rank.

Prints ONE JSON line: tokens/s of the step, per-step HIP-event timing (median, p10, p90), a roofline object
for the dominant kernel (durations from HIP events the library records on the launch stream inside the timed
steps), the same figures for every other kernel, and the fp64 CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3    # MI355X fp32 vector ALU (the fp32 configuration runs on the VALU)
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

HBM_BOUND = {"compose_fwd", "compose_bwd", "mag_scale"}
K_BASE, K_DX, K_FUSED = 6, 13, 18
N_KERNEL_IDS = 20
METRIC_FMT = "DoRA {phase} tokens/s at d_in={d_in} r={r} {dtype}; %MFMA and %HBM peak"


def kernel_work(cfg, inner_saved=True):
    """Algorithmic work per launch of each kernel: (flops, bytes), every operand touched once.  The forward
    compose pass reads base and lora and writes y and, when it is kept for the backward, inner (4 tensors);
    without the saved inner, and in the recompute that writes inner alone, it moves 3."""
    T, do, di, r = cfg.tokens, cfg.d_out, cfg.d_in, cfg.r
    e = 2 if cfg.dtype == "bf16" else 4
    return {
        "norm_cross_WAt": (2.0 * do * di * (r + 1), e * (do * di + r * di + do * r)),
        "gram_AAt": (2.0 * r * r * di, e * r * di),
        "gram_reduce": (0.0, 0.0),
        "ba_sq_BGB": (2.0 * do * r * (2 * r + 1), e * (do * r + 2 * r * r)),
        "norm_final": (0.0, 0.0),
        "mag_scale": (0.0, 16.0 * do),
        "gemm_base_xWt": (2.0 * T * do * di, e * (T * di + do * di + T * do)),
        "gemm_h_xAt": (2.0 * T * r * di, e * (T * di + r * di + T * r)),
        "gemm_lora_hBt": (2.0 * T * do * r, e * (T * r + do * r + T * do)),
        "compose_fwd": (6.0 * T * do, e * (4.0 if inner_saved else 3.0) * T * do),
        "compose_bwd": (3.0 * T * do, e * 3.0 * T * do),       # reads dy, inner; writes dz
        "dm_final": (0.0, 0.0),
        "gemm_dh_dzB": (2.0 * T * r * do, e * (T * do + do * r + T * r)),
        "gemm_dx": (2.0 * T * di * (do + r), e * (T * do + do * di + T * r + r * di + T * di)),
        "gemm_dA": (2.0 * r * di * T, e * (T * r + T * di) + 4 * r * di),
        "gemm_dB": (2.0 * do * r * T, e * (T * do + T * r) + 4 * do * r),
        "gemm_fused_fwd": (2.0 * T * do * (di + r), e * (T * di + do * di + T * r + do * r + 2 * T * do)),
        "splitk_reduce": (0.0, 0.0),   # the work of a split product is priced on its GEMM launch
    }


def kernel_sources_sha256():
    """Hash of the kernel sources: counter summaries under profiles/ record the one they were taken at."""
    h = hashlib.sha256()
    for p in sorted(glob.glob(os.path.join(ROOT, "paper_2603_22276_amd", "csrc", "*"))):
        h.update(os.path.basename(p).encode())
        h.update(open(p, "rb").read())
    return h.hexdigest()[:16]


def hbm_traffic(workload, kernel):
    """HBM-side bytes per launch of `kernel` from the FETCH_SIZE / WRITE_SIZE counter passes whose summary
    is kept under profiles/ (rocprofv3 cannot run inside this process).  Returns (bytes or None, info):
    the figure is withheld when the summary was taken at other kernel sources than the ones present."""
    rel = f"profiles/hbm_traffic_{workload}.txt"
    path = os.path.join(ROOT, rel)
    info = {"source": rel, "counters": "FETCH_SIZE x calibrated factor + WRITE_SIZE x calibrated factor, per launch",
            "measured_in_this_run": False}
    if not os.path.exists(path):
        info["note"] = "no counter summary for this workload"
        return None, info
    value, taken_at, commit = None, None, None
    for line in open(path):
        f = line.split()
        if line.startswith("# kernel_sources_sha256:"):
            taken_at = f[-1]
        elif line.startswith("# commit:"):
            commit = f[-1]
        elif len(f) >= 3 and f[0] == kernel:
            value = float(f[1]) + float(f[2])
    info["commit"] = commit
    info["kernel_sources_sha256_at_profile"] = taken_at
    now = kernel_sources_sha256()
    if taken_at != now:
        info["note"] = f"stale: kernel sources now hash to {now}; figure withheld"
        return None, info
    return value, info


# ------------------------------------------------------------------------------------------------
# resident modules

class ResidentModule:
    """One module with its inputs and outputs in HBM and the calls of one phase bound to them."""

    def __init__(self, cfg, tensors, mode, shared, D, torch, fused_forward=False):
        self.cfg, self.mode, self.D = cfg, mode, D
        dev, T, do, di, r = shared["dev"], cfg.tokens, cfg.d_out, cfg.d_in, cfg.r
        td = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.desc = D.make_desc(do, di, r, T, D.DORA_BF16 if cfg.dtype == "bf16" else D.DORA_F32, float(cfg.s), 0.0)
        for k, v in tensors.items():
            setattr(self, k, v)

        def buf(name, shape, dtype):  # activation-sized outputs are shared between modules of one shape
            key = (name, tuple(shape), dtype)
            if key not in shared:
                shared[key] = torch.empty(shape, dtype=dtype, device=dev)
            return shared[key]

        self.y = buf("y", (T, do), td)
        self.c = torch.empty(do, dtype=torch.float32, device=dev)
        self.h = self.inner = None
        if mode == "fwd_bwd_saved":
            self.h = torch.empty((T, r), dtype=td, device=dev)
            self.inner = torch.empty((T, do), dtype=td, device=dev)
        if mode != "fwd":
            self.dx = buf("dx", (T, di), td)
            self.dA = torch.empty((r, di), dtype=torch.float32, device=dev)
            self.dB = torch.empty((do, r), dtype=torch.float32, device=dev)
            self.dm = torch.empty(do, dtype=torch.float32, device=dev)
        self.fwd_fn = D.dora_forward_fused if fused_forward else D.dora_forward
        phases = [D.PHASE_FORWARD] + ([] if mode == "fwd" else
                                      [D.PHASE_BACKWARD if mode == "fwd_bwd_saved" else D.PHASE_BACKWARD_RECOMPUTE])
        self.ws_bytes = max(D.dora_workspace_bytes(self.desc, p) for p in phases)
        self.ws = None  # set by the workload: one workspace shared by all modules
        # recompute mode only: keep the [d_out] row norm of the forward for the backward (4 bytes per output row)
        # instead of rebuilding it there
        self.carry_norm = False

    def forward(self, fwd_fn=None):
        (fwd_fn or self.fwd_fn)(self.desc, self.x, self.W, self.A, self.B, self.m, None, None, self.y, self.h, self.inner,
                                self.c if (self.mode == "fwd_bwd_saved" or self.carry_norm) else None, self.ws)

    def backward(self):
        if self.mode == "fwd_bwd_saved":
            self.D.dora_backward(self.desc, self.dy, self.x, self.W, self.A, self.B, self.m, self.c, self.h, self.inner,
                                 self.dx, self.dA, self.dB, self.dm, self.ws)
        elif self.mode == "fwd_bwd_recompute":
            self.D.dora_backward(self.desc, self.dy, self.x, self.W, self.A, self.B, self.m,
                                 self.c if self.carry_norm else None, None, None,
                                 self.dx, self.dA, self.dB, self.dm, self.ws)


def device_tensors(cfg, torch, dev, gen, with_dy):
    """Synthetic inputs of one module drawn on the device (the sweep holds 224 modules; drawing 20 GB on the
    host would take minutes).  Same recipe as inputs.make_inputs: W, A ~ N(0, var 1/d_in); B ~ N(0, std
    sigma_B); x, dy ~ N(0, 1), each rounded once to the storage dtype; m = ||W||_row (1 + N(0, std sigma_m))."""
    td = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32

    def rn(shape, std):
        return (torch.randn(shape, device=dev, generator=gen, dtype=torch.float32) * std).to(td)

    inv = cfg.d_in ** -0.5
    t = {"W": rn((cfg.d_out, cfg.d_in), inv), "A": rn((cfg.r, cfg.d_in), inv), "B": rn((cfg.d_out, cfg.r), cfg.sigma_B),
         "x": rn((cfg.tokens, cfg.d_in), 1.0)}
    row_norm = torch.linalg.vector_norm(t["W"].to(torch.float32), dim=1)
    t["m"] = row_norm * (1.0 + cfg.sigma_m * torch.randn(cfg.d_out, device=dev, generator=gen, dtype=torch.float32))
    if with_dy:
        t["dy"] = rn((cfg.tokens, cfg.d_out), 1.0)
    return t


def host_tensors(cfg, G, I):
    inp = I.make_inputs(cfg)
    return {k: G.to_dev(inp[k]) for k in ("W", "A", "B", "m", "x", "dy")}, inp


class Workload:
    def __init__(self, name, modules, tokens, phase_text, torch, dev):
        self.name, self.modules, self.tokens, self.phase_text = name, modules, tokens, phase_text
        ws_bytes = max(m.ws_bytes for m in modules)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        for m in modules:
            m.ws = ws
        self.ws_bytes = ws_bytes

    def step(self):
        for m in self.modules:
            m.forward()
        for m in reversed(self.modules):
            m.backward()


# ------------------------------------------------------------------------------------------------
# timing

def pct(sorted_vals, q):
    if not sorted_vals:
        return None
    i = min(len(sorted_vals) - 1, max(0, int(round(q * (len(sorted_vals) - 1)))))
    return sorted_vals[i]


def time_steps(torch, fn, steps):
    """Exactly `steps` calls of fn between two synchronisations: host-clock mean, and each call's own duration
    from a pair of events on the launch stream."""
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e0, e1 in evs:
        e0.record()
        fn()
        e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    return (t1 - t0) * 1e3 / steps, {"median": pct(per, 0.5), "p10": pct(per, 0.1), "p90": pct(per, 0.9),
                                     "mean": sum(per) / len(per), "min": per[0], "max": per[-1], "n": len(per)}


def kernel_table(D, torch, wl, reps, dominant_live):
    """Per-kernel durations and roofline fractions.  Two passes with every launch bracketed by HIP events:
    one module at a time, to learn how many launches of each kernel a module's forward and backward make (each
    launch is priced with the algorithmic work of the module it ran for), then `reps` whole steps back to back,
    whose summed durations per kernel are the ones reported (a kernel timed right after an idle gap runs slower
    than inside the sequence).  Returns the per-kernel list and the summed contraction rate."""
    names = [D.dora_trace_name(k) for k in range(N_KERNEL_IDS)]
    tot = {n: {"ms": 0.0, "launches": 0, "flops": 0.0, "bytes": 0.0} for n in names}

    def traced(fn):
        D.dora_trace_reset()
        D.dora_trace_select(~0)
        D.dora_trace_enable(True)
        fn()
        torch.cuda.synchronize()
        D.dora_trace_enable(False)
        D.dora_trace_collect()
        return {n: D.dora_trace_get(k) for k, n in enumerate(names)}

    def price(got, work):
        w = dict(work)
        # launches that carry two contractions at once are priced with the work of both
        if got["gemm_dA"][1] > 0 and got["gemm_dB"][1] == 0:
            w["gemm_dA"] = (w["gemm_dA"][0] + w["gemm_dB"][0], w["gemm_dA"][1] + w["gemm_dB"][1])
        if got["norm_cross_WAt"][1] > 0 and got["gram_AAt"][1] == 0:   # the Gram tiles ride in the cross term's launch
            w["norm_cross_WAt"] = (w["norm_cross_WAt"][0] + w["gram_AAt"][0], w["norm_cross_WAt"][1] + w["gram_AAt"][1])
        for n, (_, cnt) in got.items():
            if cnt and n in w:
                tot[n]["flops"] += w[n][0] * cnt
                tot[n]["bytes"] += w[n][1] * cnt

    seen = {}
    for m in wl.modules:   # modules of one shape and phase make the same launches: trace one of each kind
        key = (m.cfg.d_out, m.cfg.d_in, m.cfg.r, m.cfg.tokens, m.cfg.dtype, m.mode)
        if key not in seen:
            seen[key] = (traced(m.forward), traced(m.backward) if m.mode != "fwd" else None)
        f, b = seen[key]
        price(f, kernel_work(m.cfg, inner_saved=(m.mode == "fwd_bwd_saved")))
        if b is not None:
            price(b, kernel_work(m.cfg, inner_saved=False))

    def whole():
        for _ in range(reps):
            wl.step()
    for n, (ms, cnt) in traced(whole).items():
        tot[n]["ms"], tot[n]["launches"] = ms, cnt
    fp32 = wl.modules[0].cfg.dtype == "f32"
    kernels = []
    for n in names:
        t = tot[n]
        if t["launches"] == 0:
            continue
        live = dominant_live.get(n)
        ms, cnt = (live if live and live[1] > 0 else (t["ms"], t["launches"]))
        secs = ms * 1e-3 * (t["launches"] / cnt)          # total time of this kernel's launches in `reps` steps
        flops, nbytes = t["flops"] * reps, t["bytes"] * reps
        hbm = n in HBM_BOUND
        if hbm:
            bound, ach, peak, unit = "hbm", nbytes / secs / 1e9, PEAK_HBM_GBS, "GB/s"
        elif fp32:
            bound, ach, peak, unit = "alu", flops / secs / 1e12, PEAK_FP32_TFLOPS, "TFLOP/s"
        else:
            bound, ach, peak, unit = "mfma", flops / secs / 1e12, PEAK_BF16_TFLOPS, "TFLOP/s"
        kernels.append({"kernel": n, "launches_per_step": t["launches"] / reps, "avg_us": secs / t["launches"] * 1e6,
                        "us_per_step": secs / reps * 1e6, "bound": bound, "achieved": ach, "peak": peak, "unit": unit,
                        "frac": ach / peak, "gbytes_per_s_algorithmic": nbytes / secs / 1e9,
                        "timed": "inside the timed steps" if live and live[1] > 0 else "separate pass, every launch bracketed"})
    contr = [k for k in kernels if k["bound"] in ("mfma", "alu") and tot[k["kernel"]]["flops"] > 0]
    flops = sum(tot[k["kernel"]]["flops"] for k in contr)
    secs = sum(k["us_per_step"] for k in contr) * 1e-6
    return kernels, (flops / secs / 1e12 if secs > 0 else None)


# ------------------------------------------------------------------------------------------------
# CPU oracle leg

def oracle_cores():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:  # pragma: no cover
        return os.cpu_count() or 1


def cpu_baseline(samples, backward, note):
    """The fp64 oracle, as it stands, on `samples` = [(cfg, stored host arrays, sample tokens)], repeated until
    about ten seconds of CPU work are on the clock."""
    import numpy as np
    from oracle import dora_oracle as O
    from paper_2603_22276_amd import inputs as I
    cores = oracle_cores()
    prepared = []
    for cfg, inp, n in samples:
        n = min(n, cfg.tokens)
        prepared.append((cfg, n, I.to_f64(inp["W"]), I.to_f64(inp["A"]), I.to_f64(inp["B"]), I.to_f64(inp["x"][:n]),
                         I.to_f64(inp["dy"][:n]) if backward else None, np.asarray(inp["m"], dtype=np.float64),
                         float(inp["s"])))
    reps, dt = 0, 0.0
    while dt < 10.0 and reps < 5000:
        t0 = time.perf_counter()
        for cfg, n, W, A, B, x, dy, m, s in prepared:
            f = O.forward(x, W, A, B, m, s, cfg.eps)
            if backward:
                O.backward(dy, x, W, A, B, m, s, cfg.eps, c=f["c"])
            del f
        dt += time.perf_counter() - t0
        reps += 1
    tokens = min(p[1] for p in prepared)   # every module of the sample sees the same number of tokens
    return {"value": tokens * reps / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"fp64 numpy oracle (dense W+sBA norm, forward{', backward' if backward else ''}), full weights, "
                      f"{note}, first {tokens} tokens, {reps} passes, {dt:.1f} s"}


def to_host_inputs(mod, torch):
    """Stored host arrays (the form the oracle leg widens) of a module whose inputs were drawn on the device."""
    import numpy as np
    out = {}
    for k in ("W", "A", "B", "x", "dy"):
        t = getattr(mod, k)
        out[k] = t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.cpu().numpy()
    out["m"] = mod.m.cpu().numpy()
    out["s"] = mod.cfg.s
    return out


# ------------------------------------------------------------------------------------------------
# the rank sweep of the norm in isolation (Sec. 5.6 / Table 5 on this machine)

NORM_SWEEP_SHAPES = ((4096, 4096), (8192, 8192), (4096, 11008), (8192, 28672))   # shapes of Table 5
NORM_SWEEP_RANKS = (16, 64, 128, 256, 384, 512, 768)


def norm_sweep(reps: int):
    """For every shape and rank: dora_norm, dora_norm_cached (base term read from a [d_out] cache), the library's
    scratch against one dense [d_out, d_in] temporary, and, for context only, the dense route in plain PyTorch
    ops on the same GPU (W + s * (B @ A), then a row norm: the computation the factored form replaces).
    Weights are seeded synthetic bf16 with the stated distributions.  Prints one JSON line."""
    import torch
    from paper_2603_22276_amd import binding as D
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(260322276)
    bf = torch.bfloat16

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps   # microseconds per call

    rows = []
    for d_out, d_in in NORM_SWEEP_SHAPES:
        W = (torch.randn(d_out, d_in, device=dev, generator=gen) * d_in ** -0.5).to(bf)
        base_sq = torch.empty(d_out, dtype=torch.float32, device=dev)
        c = torch.empty(d_out, dtype=torch.float32, device=dev)
        for r in NORM_SWEEP_RANKS:
            s = 32.0 / r ** 0.5
            A = (torch.randn(r, d_in, device=dev, generator=gen) * d_in ** -0.5).to(bf)
            B = (torch.randn(d_out, r, device=dev, generator=gen) * 1e-3).to(bf)
            desc = D.make_desc(d_out, d_in, r, 0, D.DORA_BF16, s)
            ws_bytes = D.dora_workspace_bytes(desc, D.PHASE_NORM)
            ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
            D.dora_base_sq(desc, W, base_sq)
            t_norm = timed(lambda: D.dora_norm(desc, W, A, B, c, ws))
            t_cached = timed(lambda: D.dora_norm_cached(desc, base_sq, W, A, B, c, ws))
            t_dense = timed(lambda: torch.linalg.vector_norm((W + s * (B @ A)).float(), dim=1))
            flops = 2.0 * d_out * d_in * (r + 1) + 2.0 * r * r * d_in + 2.0 * d_out * r * r
            nbytes = 2.0 * (d_out * d_in + r * d_in + d_out * r) + 4.0 * d_out
            rows.append({
                "d_out": d_out, "d_in": d_in, "r": r,
                "norm_us": round(t_norm, 1), "norm_cached_us": round(t_cached, 1), "dense_pytorch_us": round(t_dense, 1),
                "tflops": round(flops / t_norm / 1e6, 1), "gbs": round(nbytes / t_norm / 1e3, 1),
                "frac_mfma": round(flops / t_norm / 1e6 / PEAK_BF16_TFLOPS, 3), "frac_hbm": round(nbytes / t_norm / 1e3 / PEAK_HBM_GBS, 3),
                "scratch_bytes": int(ws_bytes), "dense_temp_bytes": 2 * d_out * d_in,
            })
            del A, B, ws
        del W
    print(json.dumps({"metric": "dora_norm latency over rank, in isolation", "unit": "us", "dtype": "bf16",
                      "data": "synthetic", "reps": reps, "rows": rows}))


# ------------------------------------------------------------------------------------------------

def build_workload(name, args, torch, D, G, I, rank=None):
    """-> (Workload, [(cfg, host inputs, sample tokens)] for the oracle leg, oracle note)"""
    dev = G.DEV
    shared = {"dev": dev}
    if name in ("C1", "C2", "C3"):
        cfg = {"C1": I.C1, "C2": I.C2, "C3": I.C3}[name]
        mode = "fwd_bwd_saved" if name == "C3" else "fwd"
        tensors, inp = host_tensors(cfg, G, I)
        mod = ResidentModule(cfg, tensors, mode, shared, D, torch, fused_forward=args.fused_forward)
        phase = ("forward (saves h, inner, w_norm) + backward (dx, dA, dB, dm)" if name == "C3"
                 else "forward (factored norm, contractions, compose)")
        wl = Workload(cfg.name, [mod], cfg.tokens, phase, torch, dev)
        return wl, [(cfg, inp, args.cpu_sample_tokens or cfg.tokens)], "whole batch"
    if name == "C4":
        mods, samples = [], []
        for cfg in (I.C4_UP, I.C4_DOWN):
            tensors, inp = host_tensors(cfg, G, I)
            mods.append(ResidentModule(cfg, tensors, "fwd_bwd_recompute", shared, D, torch))
            samples.append((cfg, inp, args.cpu_sample_tokens or 1024))
        wl = Workload("C4_bf16_mlp_pair_27648x5120_r384", mods, I.C4_UP.tokens,
                      "forward of up and down keeping nothing, then backward of both with norm, h and inner recomputed",
                      torch, dev)
        return wl, samples, "up and down module"
    if name == "C5":
        gen = torch.Generator(device=dev)
        gen.manual_seed(I.BASE_SEED + 5000 + rank)
        mods = []
        for layer in range(args.c5_layers):
            for mi in range(len(I.C5_MODULE_SHAPES)):
                cfg = I.c5_module(mi, rank, layer=layer)
                mods.append(ResidentModule(cfg, device_tensors(cfg, torch, dev, gen, True), "fwd_bwd_recompute", shared,
                                           D, torch))
        wl = Workload(f"C5_bf16_decoder_sweep_{args.c5_layers}x7_r{rank}", mods, mods[0].cfg.tokens,
                      f"forward over {len(mods)} resident modules in order, then recompute + backward in reverse order",
                      torch, dev)
        samples = [(m.cfg, to_host_inputs(m, torch), args.cpu_sample_tokens or m.cfg.tokens) for m in mods[:7]]
        return wl, samples, "the seven modules of layer 0 (the other layers repeat these shapes)"
    raise ValueError(name)


def measure(wl, args, torch, D, extras):
    for _ in range(args.warmup):
        wl.step()
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    # timed region: exactly `steps` steps.  The library brackets the launches of the candidates for the dominant
    # kernel (the two big contractions and the fused one) with HIP events on the launch stream; every other kernel
    # is timed the same way in a second pass, so that the throughput figure does not carry ~30 event records per step.
    D.dora_trace_reset()
    D.dora_trace_select((1 << K_BASE) | (1 << K_DX) | (1 << K_FUSED))
    D.dora_trace_enable(True)
    ms_per_step, per_step = time_steps(torch, wl.step, args.steps)
    D.dora_trace_enable(False)
    D.dora_trace_collect()
    live = {D.dora_trace_name(k): D.dora_trace_get(k) for k in (K_BASE, K_DX, K_FUSED)}
    peak_mem = int(torch.cuda.max_memory_allocated())
    if len(wl.modules) > 1:
        live = {}   # several shapes share a kernel id: the per-module pass below prices each launch with its own work
    reps = args.steps if len(wl.modules) == 1 else min(args.steps, 3)
    kernels, contr_rate = kernel_table(D, torch, wl, reps, live)
    dom = max(kernels, key=lambda k: k["us_per_step"])
    traffic, tinfo = hbm_traffic(wl.name, dom["kernel"])
    roofline = {"kernel": dom["kernel"], "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"],
                "unit": dom["unit"], "frac": dom["frac"], "traffic": traffic, "traffic_info": tinfo}
    ms_untraced, _ = time_steps(torch, wl.step, args.steps)
    out = {
        "value": wl.tokens / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "step_ms_hip_events": per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "roofline": roofline,
        "mfma_frac_all_contractions": (contr_rate / (PEAK_BF16_TFLOPS if dom["bound"] != "alu" else PEAK_FP32_TFLOPS)
                                       if contr_rate else None),
        "hbm_frac_compose_fwd": next((k["frac"] for k in kernels if k["kernel"] == "compose_fwd"), None),
        "hbm_frac_compose_bwd": next((k["frac"] for k in kernels if k["kernel"] == "compose_bwd"), None),
        "ms_per_step_without_event_pairs": ms_untraced,
        "peak_device_memory_bytes": peak_mem,
        "workspace_bytes_shared": wl.ws_bytes,
        "kernels": kernels,
    }
    out.update(extras(wl, ms_untraced) if extras else {})
    return out


def recompute_extras(args, torch):
    """Beside `value` for the recompute workloads (C4, C5): the same step with each module's [d_out] row norm kept
    from its forward and handed to its backward, which then recomputes h and inner but not the norm."""
    def extras(wl, ms_untraced):
        for m in wl.modules:
            m.carry_norm = True
        for _ in range(2):
            wl.step()
        ms, _ = time_steps(torch, wl.step, args.steps)
        for m in wl.modules:
            m.carry_norm = False
        return {"row_norm_carried_to_backward": {
            "ms_per_step_without_event_pairs": ms, "tokens_per_s": wl.tokens / (ms * 1e-3),
            "against_ms_per_step_without_event_pairs": ms_untraced,
            "note": "the norm is rank and batch independent within a step: a caller that keeps the fp32 [d_out] vector "
                    "w_norm_out of dora_forward and passes it to dora_backward skips the second norm of the step; "
                    "`value` recomputes it, as the workload is defined"}}
    return extras


def c3_extras(args, torch, D, G):
    """Figures reported beside `value` for the single bf16 modules: the step as a HIP graph, the other forward
    path, and what this card sustains on a plain copy and a register-resident MFMA loop."""
    def extras(wl, ms_untraced):
        mod = wl.modules[0]
        desc = mod.desc
        out = {}
        ms_graph = None
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                wl.step()
            for _ in range(2):
                graph.replay()
            ms_graph, _ = time_steps(torch, graph.replay, args.steps)
            del graph
        except Exception as exc:  # pragma: no cover - informational figure only
            print(f"bench.py: graph replay not measured ({exc})", file=sys.stderr)
        out["ms_per_step_graph_replay"] = ms_graph
        other = D.dora_forward if args.fused_forward else D.dora_forward_fused

        def other_step():
            mod.forward(other)
            mod.backward()
        for _ in range(2):
            other_step()
        ms_other, _ = time_steps(torch, other_step, args.steps)
        out["other_forward_path"] = {
            "forward_path": "base, lora, compose pass" if args.fused_forward else "fused epilogue",
            "ms_per_step_without_event_pairs": ms_other, "tokens_per_s": wl.tokens / (ms_other * 1e-3)}
        library = {}
        cfg = mod.cfg
        if cfg.dtype == "bf16":
            # the vendor library's GEMM on this module's own x and W, for context (HIP events on torch's stream)
            yy = torch.empty((cfg.tokens, cfg.d_out), dtype=torch.bfloat16, device=G.DEV)
            for _ in range(3):
                torch.matmul(mod.x, mod.W.t(), out=yy)
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(7)]
            for e0, e1 in evs:
                e0.record()
                torch.matmul(mod.x, mod.W.t(), out=yy)
                e1.record()
            torch.cuda.synchronize()
            lib_us = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in evs)[len(evs) // 2]
            library["library_matmul_x_Wt_us"] = lib_us
            library["library_matmul_x_Wt_TFLOPs"] = 2.0 * cfg.tokens * cfg.d_out * cfg.d_in / lib_us / 1e6
            del yy
        probe_bytes = 512 * 2 ** 20
        src = torch.empty(probe_bytes, dtype=torch.uint8, device=G.DEV).fill_(1)
        dst = torch.empty_like(src)
        sink = torch.zeros(512, dtype=torch.float32, device=G.DEV)
        gen = torch.Generator(device=G.DEV)
        gen.manual_seed(1234)
        operands = {"normal": torch.randn(65536 // 2, device=G.DEV, generator=gen).to(torch.bfloat16),
                    "zeros": torch.zeros(65536 // 2, dtype=torch.bfloat16, device=G.DEV)}
        probe_iters, probe_wgs = 1024, 1024
        probe_flop = probe_wgs * 4 * probe_iters * 64 * 16384.0

        def traced(fn, kernel_id, reps=5):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            D.dora_trace_reset()
            D.dora_trace_select(~0)
            D.dora_trace_enable(True)
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            D.dora_trace_enable(False)
            D.dora_trace_collect()
            ms, n = D.dora_trace_get(kernel_id)
            return ms * 1e-3 / n
        copy_s = traced(lambda: D.dora_probe_copy(src, dst, probe_bytes), 16)
        mfma_s = {k: traced(lambda v=v: D.dora_probe_mfma(v, sink, probe_iters, probe_wgs), 17) for k, v in operands.items()}
        sustained = {
            "copy_GBps": 2.0 * probe_bytes / copy_s / 1e9,
            "mfma_bf16_TFLOPs_normal_operands": probe_flop / mfma_s["normal"] / 1e12,
            "mfma_bf16_TFLOPs_zero_operands": probe_flop / mfma_s["zeros"] / 1e12,
            "note": "plain 16-byte-per-lane copy of 512 MiB (read + write counted); register-resident "
                    "v_mfma_f32_16x16x32_bf16 loop, one wave per SIMD, on N(0,1) and on all-zero operands (the card "
                    "is power limited: the rate depends on the operand values); library_matmul: torch.matmul (the vendor "
                    "library) on this module's own x and W, median of 7 back-to-back launches, for context; all "
                    "measured in this run"}
        sustained.update(library)
        out["sustained_on_this_card"] = sustained
        out["workspace_bytes"] = {"norm": D.dora_workspace_bytes(desc, D.PHASE_NORM),
                                  "forward": D.dora_workspace_bytes(desc, D.PHASE_FORWARD),
                                  "backward": D.dora_workspace_bytes(desc, D.PHASE_BACKWARD),
                                  "dense_BA_temporary_avoided": mod.cfg.d_out * mod.cfg.d_in * 2}
        return out
    return extras


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--c5-ranks", default="64,384,768", help="ranks of the decoder-layer sweep (comma separated)")
    ap.add_argument("--c5-layers", type=int, default=32)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fused-forward", action="store_true",
                    help="forward through dora_forward_fused (compose folded into the GEMM epilogue) instead of the\n"
                         "base / lora / compose sequence (C2, C3)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0,
                    help="tokens of the oracle's sample (default: the whole batch; 1024 per module for C4)")
    ap.add_argument("--norm-sweep", action="store_true",
                    help="instead of the step benchmark: time dora_norm alone over ranks and the weight shapes of Table 5")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the DoRA module on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives are part of the path).", file=sys.stderr)
        sys.exit(2)
    if args.norm_sweep:
        norm_sweep(max(args.steps, 1))
        return

    import torch
    from paper_2603_22276_amd import binding as D
    from paper_2603_22276_amd import device as G
    from paper_2603_22276_amd import inputs as I

    if args.config != "C5":
        wl, samples, note = build_workload(args.config, args, torch, D, G, I)
        cfg = wl.modules[0].cfg
        phase = {"C1": "fwd", "C2": "fwd", "C3": "fwd+bwd", "C4": "fwd+recompute+bwd"}[args.config]
        out = {"metric": METRIC_FMT.format(phase=phase, d_in=cfg.d_in if args.config != "C4" else "5120/27648", r=cfg.r,
                                           dtype="bf16" if cfg.dtype == "bf16" else "fp32")}
        extras = (c3_extras(args, torch, D, G) if args.config in ("C2", "C3")
                  else recompute_extras(args, torch) if args.config == "C4" else None)
        out.update(measure(wl, args, torch, D, extras))
        out.update({"dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
                    "config": {"workload": wl.name, "tokens": wl.tokens, "phase": wl.phase_text,
                               "modules": [{"d_out": m.cfg.d_out, "d_in": m.cfg.d_in, "r": m.cfg.r} for m in wl.modules],
                               "forward_path": "fused epilogue" if args.fused_forward else "base, lora, compose pass"}})
        if len(wl.modules) == 1:
            out["config"].update({"d_out": cfg.d_out, "d_in": cfg.d_in, "r": cfg.r})
        out["cpu_baseline"] = None if args.no_cpu_baseline else cpu_baseline(samples, args.config in ("C3", "C4"), note)
        print(json.dumps(out))
        return

    # C5: one sweep per rank; `value` is the aggregate rate at r = 384 (the headline rank), the others beside it
    ranks = [int(v) for v in args.c5_ranks.split(",")]
    per_rank, cpu = {}, None
    for rank in ranks:
        wl, samples, note = build_workload("C5", args, torch, D, G, I, rank=rank)
        res = measure(wl, args, torch, D, recompute_extras(args, torch))
        res["config"] = {"workload": wl.name, "tokens": wl.tokens, "phase": wl.phase_text, "r": rank,
                         "modules_resident": len(wl.modules)}
        per_rank[rank] = res
        if not args.no_cpu_baseline and (rank == 384 or (384 not in ranks and rank == ranks[-1])):
            cpu = cpu_baseline(samples, True, note)
            per_layer_s = min(s[2] for s in samples) / cpu["value"]
            cpu["sample"] += (f"; one layer takes {per_layer_s:.1f} s, so the {args.c5_layers}-layer sweep is put at "
                              f"{args.c5_layers * per_layer_s:.0f} s by extrapolation: `value` is tokens / that")
            cpu["value"] = cpu["value"] / args.c5_layers
        del wl, samples
        torch.cuda.empty_cache()
    head = per_rank.get(384) or per_rank[ranks[-1]]
    out = {"metric": "DoRA fwd+recompute+bwd aggregate tokens/s over a 32-layer decoder sweep (7 adapted modules per layer) "
                     "at r=384 bf16; %MFMA and %HBM peak"}
    out.update({k: v for k, v in head.items() if k != "config"})
    out.update({"dtype": "bf16", "data": "synthetic", "config": head["config"],
                "ranks": {str(r): {k: v for k, v in res.items() if k != "kernels"} for r, res in per_rank.items()},
                "cpu_baseline": cpu})
    print(json.dumps(out))


if __name__ == "__main__":
    main()
