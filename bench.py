#!/usr/bin/env python3
"""Benchmark of the DoRA module hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input: dora_forward (factored
norm, magnitude scale, the three contractions, compose, saving h / inner / w_norm) followed by
dora_backward (compose backward with the fused dm reduction, dh, dx, dA, dB).  The workload is the
headline configuration: d_out = d_in = 8192, r = 384, tokens = 8192, bf16 storage with fp32
accumulation.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: tokens/s for the step, a roofline object for the dominant kernel (duration
measured with HIP events recorded by the library on the launch stream during the timed steps), the
same figures for every other kernel, and the fp64 CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E


def kernel_work(cfg):
    """Algorithmic work per launch of each kernel: (flops, bytes), every operand touched once."""
    T, do, di, r, e = cfg.tokens, cfg.d_out, cfg.d_in, cfg.r, 2
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
        "compose_fwd": (6.0 * T * do, e * 4.0 * T * do),       # reads base, lora; writes y, inner
        "compose_bwd": (3.0 * T * do, e * 3.0 * T * do),       # reads dy, inner; writes dz
        "dm_final": (0.0, 0.0),
        "gemm_dh_dzB": (2.0 * T * r * do, e * (T * do + do * r + T * r)),
        "gemm_dx": (2.0 * T * di * (do + r), e * (T * do + do * di + T * r + r * di + T * di)),
        "gemm_dA": (2.0 * r * di * T, e * (T * r + T * di) + 4 * r * di),
        "gemm_dB": (2.0 * do * r * T, e * (T * do + T * r) + 4 * do * r),
        "gemm_fused_fwd": (2.0 * T * do * (di + r), e * (T * di + do * di + T * r + do * r + 2 * T * do)),
    }


HBM_BOUND = {"compose_fwd", "compose_bwd", "mag_scale"}


def hbm_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` as measured by the FETCH_SIZE / WRITE_SIZE counter passes whose
    summary is kept under profiles/ (rocprofv3 cannot run inside this process); None if not recorded."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 3 and f[0] == kernel:
            return float(f[1]) + float(f[2])
    return None


def cpu_baseline(cfg, inp, sample_tokens):
    """The fp64 oracle, as it stands, on the first `sample_tokens` tokens with the full weights."""
    import numpy as np
    from oracle import dora_oracle as O
    from paper_2603_22276_amd import inputs as I
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:  # pragma: no cover
        cores = os.cpu_count() or 1
    n = min(sample_tokens, cfg.tokens)
    W, A, B = I.to_f64(inp["W"]), I.to_f64(inp["A"]), I.to_f64(inp["B"])
    x, dy = I.to_f64(inp["x"][:n]), I.to_f64(inp["dy"][:n])
    m, s = inp["m"].astype(np.float64), float(inp["s"])
    # the same sample again and again until about ten seconds of CPU work are on the clock (at most 8 passes)
    reps, dt = 0, 0.0
    while reps < 8 and dt < 10.0:
        t0 = time.perf_counter()
        f = O.forward(x, W, A, B, m, s, cfg.eps)
        O.backward(dy, x, W, A, B, m, s, cfg.eps, c=f["c"])
        dt += time.perf_counter() - t0
        reps += 1
        del f
    return {"value": n * reps / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"fp64 numpy oracle, dense W+sBA norm + forward + backward, full weights, first {n} of "
                      f"{cfg.tokens} tokens, {reps} passes, {dt:.1f} s"}


NORM_SWEEP_SHAPES = ((4096, 4096), (8192, 8192), (4096, 11008), (8192, 28672))   # shapes of Table 5
NORM_SWEEP_RANKS = (16, 64, 128, 256, 384, 512, 768)


def norm_sweep(reps: int):
    """Rank sweep of the factored norm in isolation (the experiment of Sec. 5.6 / Table 5 on this machine).

    For every shape and rank: dora_norm, dora_norm_cached (base term read from a [d_out] cache), the library's
    scratch against one dense [d_out, d_in] temporary, and, for context only, the dense route in plain PyTorch
    ops on the same GPU (W + s * (B @ A), then a row norm: the computation the factored form replaces).
    Weights are seeded synthetic bf16 with the stated distributions.  Prints one JSON line.
    """
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="C3", choices=["C2", "C3"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fused-forward", action="store_true",
                    help="forward through dora_forward_fused (compose folded into the GEMM epilogue) instead of the\n"
                         "base / lora / compose sequence")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192)
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
    from paper_2603_22276_amd import inputs as I
    from paper_2603_22276_amd import device as G

    cfg = {"C2": I.C2, "C3": I.C3}[args.config]
    inp = I.make_inputs(cfg)
    mod = G.Module(cfg, inp)
    desc = mod.desc
    T, do, di, r = cfg.tokens, cfg.d_out, cfg.d_in, cfg.r
    bf = torch.bfloat16
    y = torch.empty((T, do), dtype=bf, device=G.DEV)
    h = torch.empty((T, r), dtype=bf, device=G.DEV)
    inner = torch.empty((T, do), dtype=bf, device=G.DEV)
    c = torch.empty(do, dtype=torch.float32, device=G.DEV)
    dx = torch.empty((T, di), dtype=bf, device=G.DEV)
    dA = torch.empty((r, di), dtype=torch.float32, device=G.DEV)
    dB = torch.empty((do, r), dtype=torch.float32, device=G.DEV)
    dm = torch.empty(do, dtype=torch.float32, device=G.DEV)
    ws_f = G.workspace(desc, D.PHASE_FORWARD)
    ws_b = G.workspace(desc, D.PHASE_BACKWARD)

    fwd = D.dora_forward_fused if args.fused_forward else D.dora_forward

    def step():
        fwd(desc, mod.x, mod.W, mod.A, mod.B, mod.m, None, None, y, h, inner, c, ws_f)
        D.dora_backward(desc, mod.dy, mod.x, mod.W, mod.A, mod.B, mod.m, c, h, inner, dx, dA, dB, dm, ws_b)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly `steps` steps.  The library brackets the launches of the candidates for the
    # dominant kernel (the two big contractions and the fused one) with HIP events on the launch stream;
    # every other kernel is timed the same way in a second pass below, so that the throughput figure
    # does not carry ~30 event records per step.
    K_BASE, K_DX, K_FUSED = 6, 13, 18
    D.dora_trace_reset()
    D.dora_trace_select((1 << K_BASE) | (1 << K_DX) | (1 << K_FUSED))
    D.dora_trace_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    D.dora_trace_enable(False)
    D.dora_trace_collect()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    dominant = {k: D.dora_trace_get(k) for k in (K_BASE, K_DX, K_FUSED)}

    # second pass: every kernel bracketed (durations for the per-kernel table)
    D.dora_trace_reset()
    D.dora_trace_select(~0)
    D.dora_trace_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_all_events = (time.perf_counter() - t0) * 1e3 / args.steps
    D.dora_trace_enable(False)
    D.dora_trace_collect()

    # the same number of steps without the event pairs, to show what they cost
    def timed(fn):
        torch.cuda.synchronize()
        a = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - a) * 1e3 / args.steps

    ms_untraced = timed(step)

    # the same step captured once in a HIP graph and replayed: what is left of the gaps between the sixteen launches
    ms_graph = None
    try:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(2):
            graph.replay()
        ms_graph = timed(graph.replay)
        del graph
    except Exception as exc:  # pragma: no cover - informational figure only
        print(f"bench.py: graph replay not measured ({exc})", file=sys.stderr)

    # the other forward path (compose folded into the GEMM epilogue when the default is timed, and the
    # other way round), same backward, no event pairs: reported beside `value`, not instead of it
    other_fwd = D.dora_forward if args.fused_forward else D.dora_forward_fused

    def other_step():
        other_fwd(desc, mod.x, mod.W, mod.A, mod.B, mod.m, None, None, y, h, inner, c, ws_f)
        D.dora_backward(desc, mod.dy, mod.x, mod.W, mod.A, mod.B, mod.m, c, h, inner, dx, dA, dB, dm, ws_b)

    for _ in range(2):
        other_step()
    ms_other = timed(other_step)

    # what this card sustains with no other work in the way: a plain streaming copy and a
    # register-resident MFMA loop, timed the same way (library events on the launch stream)
    probe_bytes = 512 * 2 ** 20
    src = torch.empty(probe_bytes, dtype=torch.uint8, device=G.DEV).fill_(1)
    dst = torch.empty_like(src)
    sink = torch.zeros(512, dtype=torch.float32, device=G.DEV)
    probe_iters, probe_wgs = 512, 1024
    for _ in range(2):
        D.dora_probe_copy(src, dst, probe_bytes)
        D.dora_probe_mfma(sink, probe_iters, probe_wgs)
    torch.cuda.synchronize()
    D.dora_trace_enable(True)
    for _ in range(5):
        D.dora_probe_copy(src, dst, probe_bytes)
        D.dora_probe_mfma(sink, probe_iters, probe_wgs)
    torch.cuda.synchronize()
    D.dora_trace_enable(False)
    D.dora_trace_collect()
    copy_ms, copy_n = D.dora_trace_get(16)
    mfma_ms, mfma_n = D.dora_trace_get(17)
    sustained = {
        "copy_GBps": 2.0 * probe_bytes / (copy_ms * 1e-3 / copy_n) / 1e9,
        "mfma_bf16_TFLOPs": probe_wgs * 8 * probe_iters * 8 * 32768.0 / (mfma_ms * 1e-3 / mfma_n) / 1e12,
        "note": "plain 16-byte-per-lane copy of 512 MiB (read + write counted) and a register-resident "
                "v_mfma_f32_32x32x16_bf16 loop, measured in this run",
    }
    del src, dst

    work = kernel_work(cfg)
    # launches that carry two contractions at once are priced with the work of both
    for host, guest in (("gemm_base_xWt", "gemm_h_xAt"), ("gemm_dA", "gemm_dB")):
        names = [D.dora_trace_name(k) for k in range(16)]
        if D.dora_trace_get(names.index(guest))[1] == 0:
            work[host] = (work[host][0] + work[guest][0], work[host][1] + work[guest][1])
    kernels = []
    for kid in list(range(16)) + [18]:
        total_ms, n = D.dora_trace_get(kid)
        if kid in dominant and dominant[kid][1] > 0:
            total_ms, n = dominant[kid]  # the duration measured inside the timed region
        if n == 0:
            continue
        name = D.dora_trace_name(kid)
        avg_s = total_ms * 1e-3 / n
        flops, nbytes = work[name]
        hbm = name in HBM_BOUND
        ach = (nbytes / avg_s / 1e9) if hbm else (flops / avg_s / 1e12)
        peak = PEAK_HBM_GBS if hbm else PEAK_BF16_TFLOPS
        kernels.append({"kernel": name, "launches_per_step": n / args.steps, "avg_us": avg_s * 1e6,
                        "bound": "hbm" if hbm else "mfma", "achieved": ach, "peak": peak,
                        "unit": "GB/s" if hbm else "TFLOP/s", "frac": ach / peak,
                        "gbytes_per_s_algorithmic": nbytes / avg_s / 1e9})
    dom = max(kernels, key=lambda k: k["avg_us"] * k["launches_per_step"])
    roofline = {"kernel": dom["kernel"], "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"],
                "unit": dom["unit"], "frac": dom["frac"], "traffic": hbm_traffic(cfg.name, dom["kernel"])}
    mfma = [k for k in kernels if k["bound"] == "mfma" and work[k["kernel"]][0] > 0]
    mfma_flops = sum(work[k["kernel"]][0] * k["launches_per_step"] for k in mfma)
    mfma_time = sum(k["avg_us"] * 1e-6 * k["launches_per_step"] for k in mfma)

    out = {
        "metric": "DoRA fwd+bwd tokens/s at d_in=8192 r=384 bf16; %MFMA and %HBM peak",
        "value": T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "d_out": do, "d_in": di, "r": r, "tokens": T,
                   "phase": "forward (saves h, inner, w_norm) + backward (dx, dA, dB, dm)",
                   "forward_path": "fused epilogue" if args.fused_forward else "base, lora, compose pass"},
        "roofline": roofline,
        "mfma_frac_all_contractions": mfma_flops / mfma_time / 1e12 / PEAK_BF16_TFLOPS,
        "hbm_frac_compose_fwd": next((k["frac"] for k in kernels if k["kernel"] == "compose_fwd"), None),
        "hbm_frac_compose_bwd": next(k["frac"] for k in kernels if k["kernel"] == "compose_bwd"),
        "ms_per_step_without_event_pairs": ms_untraced,
        "ms_per_step_with_every_kernel_bracketed": ms_all_events,
        "ms_per_step_graph_replay": ms_graph,
        "other_forward_path": {"forward_path": "base, lora, compose pass" if args.fused_forward else "fused epilogue",
                               "ms_per_step_without_event_pairs": ms_other, "tokens_per_s": T / (ms_other * 1e-3)},
        "sustained_on_this_card": sustained,
        "workspace_bytes": {"norm": D.dora_workspace_bytes(desc, D.PHASE_NORM),
                            "forward": D.dora_workspace_bytes(desc, D.PHASE_FORWARD),
                            "backward": D.dora_workspace_bytes(desc, D.PHASE_BACKWARD),
                            "dense_BA_temporary_avoided": do * di * 2},
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, inp, args.cpu_sample_tokens)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
