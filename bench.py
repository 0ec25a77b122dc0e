#!/usr/bin/env python3
"""Benchmark of the BD K/V up-projection hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--rotate R] [--no-graph] [--no-extras] [--no-sweep]

A "step" is one bda_kv_project call over one batch of the DeepSeek-V2-Lite-shaped workload
(T = 4096 tokens, d_c = 512, 16 K_nope + 16 V heads of 128, fp16): latent tile load, reduced-K MFMA
GEMM over all heads, identity slice, rounding and store.  Inputs are resident in HBM before the
timed region.  Each step works on its own (c, out) buffer pair out of R rotating pairs, so that the
traffic is not served by the 256 MB last-level cache; the weights C are shared, as within a layer.
The K steps are captured once into a HIP graph (untimed) and the timed region is one replay of that
graph = exactly K launches, bracketed by synchronisation; `--no-graph` times a plain launch loop.

Prints ONE JSON line on stdout (progress goes to stderr).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense fp16/bf16 MFMA
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E

METRIC = "BD K/V proj tokens/s, TFLOP/s & GB/s vs roofline; speedup vs dense projection"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--rotate", type=int, default=16, help="distinct (c, out) buffer pairs")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="leave the token-count sweep out of the extras")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--prewarm-ms", type=float, default=200.0,
                    help="untimed run of the same step before the W warm-up steps, so that the clocks have settled")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run three 256 MiB device copies (reference for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU only (the path shards by tokens or heads with no "
            "exchange step, but no multi-GPU code is part of it); run with --gpus 1")
        return 2

    import torch

    import bda_workloads as wl
    import paper_2510_01718_amd as bda

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 3
    bda.load()                                    # fails loudly if libbda.so is not built
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    sid = int(stream.cuda_stream)

    def dev(stored, dtype):
        a = np.ascontiguousarray(stored)
        if dtype == wl.BF16:
            a = a.view(np.int16)
        return torch.from_numpy(a).cuda()

    tdt = {wl.F16: torch.float16, wl.BF16: torch.int16, wl.F32: torch.float32}

    if args.calib_copy:
        xs = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        ys = torch.empty_like(xs)
        for _ in range(3):
            ys.copy_(xs)
        torch.cuda.synchronize()
        del xs, ys

    # ------------------------------------------------------------------ main workload (config 2)
    w = wl.kv_workload("v2lite")
    T, d_c, d_h, H, N, K = w.T, w.d_c, w.d_h, w.H, w.N, w.d_c - w.d_h
    offs = []
    Cs = []
    col = 0
    t_prep0 = time.perf_counter()
    for Hg in H:                                  # library prepare, first-r basis per group
        Cg, _, off, _ = bda.bda_prepare(w.W[:, col:col + Hg * d_h], d_c, Hg, d_h, mode=bda.BASIS_FIRST)
        Cs.append(Cg)
        offs.append(off)
        col += Hg * d_h
    t_prep_host = time.perf_counter() - t_prep0
    C_stored, C64 = wl.to_storage(np.hstack(Cs), w.dtype)
    log(f"workload v2lite: T={T} N={N} K={K} max|C|={np.abs(C64).max():.1f}")
    R = max(1, args.rotate)
    C_d = dev(C_stored, w.dtype)
    c_bufs, o_bufs = [], []
    for r in range(R):
        cw = wl.kv_workload("v2lite", seed=w.seed + 100 * r) if r else w
        c_bufs.append(dev(cw.c_stored, w.dtype))
        o_bufs.append(torch.empty((T, N), dtype=tdt[w.dtype], device="cuda"))

    def timed_run(step_fn, steps, warmup, use_graph):
        """Returns (wall seconds, GPU seconds by HIP events) for exactly `steps` launches."""
        for i in range(warmup):
            step_fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if use_graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):              # captures on a side stream of its own
                cap_id = int(torch.cuda.current_stream().cuda_stream)
                for i in range(steps):
                    step_fn.with_stream(i, cap_id)
            torch.cuda.synchronize()
            g.replay()                             # one untimed replay (graph upload)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
        else:
            t0 = time.perf_counter()
            e0.record()
            for i in range(steps):
                step_fn(i)
            e1.record()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
        return t1 - t0, e0.elapsed_time(e1) * 1e-3

    class Step:
        """A launch closure that can target the bench stream or a capture stream."""
        def __init__(self, fn):
            self.fn = fn

        def __call__(self, i):
            self.fn(i, sid)

        def with_stream(self, i, s):
            self.fn(i, s)

    main_step = Step(lambda i, s: bda.bda_kv_project(c_bufs[i % R], d_c, T, d_c, d_h, H, offs, C_d, N,
                                                     o_bufs[i % R], N, w.dtype, w.dtype, s))
    use_graph = not args.no_graph
    # The chip needs on the order of 100 ms of work to reach its steady clock / power state: a
    # measurement taken after a cold start reads ~10 % slower than the same launches a moment later
    # (extra.main_repeated_later shows the check).  So the step runs untimed for a while first.
    t_end = time.perf_counter() + args.prewarm_ms * 1e-3
    n_pre = 0
    while time.perf_counter() < t_end:
        for i in range(64):
            main_step(i)
        torch.cuda.synchronize()
        n_pre += 64
    wall, gpu = timed_run(main_step, args.steps, args.warmup, use_graph)
    ms_per_step = wall / args.steps * 1e3
    kernel_s = gpu / args.steps
    flops = 2.0 * T * K * N
    alg_bytes = (T * d_c + K * N + T * N) * 2.0
    tokens_per_s = T / (wall / args.steps)
    log(f"main: {ms_per_step * 1e3:.2f} us/step wall, {kernel_s * 1e6:.2f} us/launch by events, "
        f"{flops / kernel_s / 1e12:.1f} TFLOP/s, {alg_bytes / kernel_s / 1e9:.0f} GB/s")

    traffic = None
    tpath = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("v2lite_kv_T4096_f16", {}).get("bytes_per_launch")
        except Exception:
            traffic = None

    result = {
        "metric": METRIC,
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "v2lite_kv_T4096_f16", "T": T, "d_c": d_c, "d_h": d_h, "heads": H,
                   "basis_offset": offs, "N": N, "K": K, "rotating_buffers": R,
                   "launch": "hip_graph" if use_graph else "loop", "prewarm_ms": args.prewarm_ms},
        "roofline": {"bound": "mfma", "achieved": flops / kernel_s / 1e12, "peak": MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": flops / kernel_s / 1e12 / MFMA_PEAK_TFLOPS,
                     "traffic": traffic,
                     "kernel_us": kernel_s * 1e6, "flops_per_launch": flops,
                     "hbm": {"achieved": alg_bytes / kernel_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": alg_bytes / kernel_s / 1e9 / HBM_PEAK_GBS,
                             "bytes_per_launch": alg_bytes}},
    }

    # ------------------------------------------------------------------ extras: other rows of the path
    extra = {}
    if not args.no_extras:
        def bench_small(fn, steps=200, warmup=20, graph=True):
            wall_, gpu_ = timed_run(Step(fn), steps, warmup, graph and use_graph)
            return gpu_ / steps

        # dense comparator on the same latent (Algorithm "MHA Inference" step 2-3), same rotation
        W_stored, _ = wl.to_storage(w.W, w.dtype)
        W_d = dev(W_stored, w.dtype)
        t_dense = bench_small(lambda i, s: bda.bda_dense_project(c_bufs[i % R], d_c, T, d_c, W_d, N, N,
                                                                 o_bufs[i % R], N, w.dtype, w.dtype, s), args.steps, args.warmup)
        extra["dense_v2lite_T4096"] = {"us": t_dense * 1e6, "tflops": 2.0 * T * d_c * N / t_dense / 1e12}
        extra["speedup_vs_dense"] = {"measured": t_dense / kernel_s, "theoretical": d_c / K}
        log(f"dense: {t_dense * 1e6:.2f} us -> speedup {t_dense / kernel_s:.3f} (theory {d_c / K:.3f})")
        # warm-cache figure (one buffer pair)
        t_warm = bench_small(lambda i, s: bda.bda_kv_project(c_bufs[0], d_c, T, d_c, d_h, H, offs, C_d, N,
                                                             o_bufs[0], N, w.dtype, w.dtype, s), args.steps, args.warmup)
        extra["v2lite_T4096_single_buffer"] = {"us": t_warm * 1e6, "tflops": flops / t_warm / 1e12}
        # basis windows inside the latent (Appendix "Residual-Min with Offset Search": window starts at
        # multiples of 16): the same launch with other window starts (timing only: C is not re-derived)
        win = {}
        for name, o2 in (("last", [K, K]), ("offset_192", [192, 192]), ("offset_208", [208, 208])):
            t_o = bench_small(lambda i, s, o2=o2: bda.bda_kv_project(c_bufs[i % R], d_c, T, d_c, d_h, H, o2, C_d, N,
                                                                     o_bufs[i % R], N, w.dtype, w.dtype, s), args.steps, args.warmup)
            win[name] = {"us": t_o * 1e6, "vs_first": t_o / kernel_s}
        extra["window_position_cost"] = win
        log("window position: " + ", ".join(f"{k} {v['us']:.2f} us ({v['vs_first']:.3f}x)" for k, v in win.items()))
        # gradients of the same projection (Section "BDA Training Evaluation"): upstream gradient of
        # the output's shape, both gradients; rotation over the same buffers (o_bufs hold whatever
        # the forward wrote: timing only)
        gc_b = torch.empty((T, d_c), dtype=tdt[w.dtype], device="cuda")
        gC_b = torch.empty((K, N), dtype=tdt[w.dtype], device="cuda")
        t_gc = bench_small(lambda i, s: bda.bda_kv_project_backward(None, d_c, o_bufs[i % R], N, C_d, N, T, d_c, d_h, H, offs,
                                                                    gc_b, d_c, None, N, w.dtype, w.dtype, s), args.steps, args.warmup)
        t_gC = bench_small(lambda i, s: bda.bda_kv_project_backward(c_bufs[i % R], d_c, o_bufs[i % R], N, None, N, T, d_c, d_h, H, offs,
                                                                    None, d_c, gC_b, N, w.dtype, w.dtype, s), args.steps, args.warmup)
        t_both = bench_small(lambda i, s: bda.bda_kv_project_backward(c_bufs[i % R], d_c, o_bufs[i % R], N, C_d, N, T, d_c, d_h, H, offs,
                                                                      gc_b, d_c, gC_b, N, w.dtype, w.dtype, s), args.steps, args.warmup)
        extra["backward_v2lite_T4096"] = {
            "grad_c_us": t_gc * 1e6, "grad_c_tflops": flops / t_gc / 1e12,
            "grad_C_us": t_gC * 1e6, "grad_C_tflops": flops / t_gC / 1e12,
            "both_one_call_us": t_both * 1e6, "both_tflops": 2 * flops / t_both / 1e12,
            "vs_forward": t_both / kernel_s}
        log(f"backward: grad_c {t_gc * 1e6:.1f} us ({flops / t_gc / 1e12:.0f} TFLOP/s), grad_C {t_gC * 1e6:.1f} us "
            f"({flops / t_gC / 1e12:.0f} TFLOP/s), both in one call {t_both * 1e6:.1f} us ({2 * flops / t_both / 1e12:.0f} TFLOP/s)")
        del gc_b, gC_b
        # the main measurement once more, after the other measurements (clock / power state check)
        t_again = bench_small(lambda i, s: main_step.fn(i, s), args.steps, args.warmup)
        extra["main_repeated_later"] = {"us": t_again * 1e6, "vs_first_measurement": t_again / kernel_s}
        log(f"main again: {t_again * 1e6:.2f} us")
        # decode shapes (config 3): rotate over distinct copies of the weights so that each launch
        # streams its 3 MiB of C from HBM, not from cache
        n_w = 96
        C_rot = C_d.unsqueeze(0).repeat(n_w, 1, 1).contiguous()
        dec = {}
        for Td in (1, 8, 32, 64):
            cd = dev(wl.kv_workload("decode", T=Td).c_stored, w.dtype)
            od = torch.empty((Td, N), dtype=tdt[w.dtype], device="cuda")
            t_d = bench_small(lambda i, s: bda.bda_kv_project(cd, d_c, Td, d_c, d_h, H, offs, C_rot[i % n_w], N,
                                                              od, N, w.dtype, w.dtype, s), max(8, min(480, args.steps * 2)), max(2, min(96, args.warmup * 2)))
            by = (Td * d_c + K * N + Td * N) * 2.0
            dec[f"T{Td}"] = {"us": t_d * 1e6, "gbs": by / t_d / 1e9, "frac_hbm": by / t_d / 1e9 / HBM_PEAK_GBS}
            log(f"decode T={Td}: {t_d * 1e6:.2f} us, {by / t_d / 1e9:.0f} GB/s")
        extra["decode_v2lite"] = dec
        del C_rot
        # V3-shaped (config 4), bf16: timing-only weights of the scale prepare produces
        rng = np.random.default_rng(2)
        T4, N4 = 8192, 256 * 128
        c4 = dev(wl.kv_workload("v3").c_stored, wl.BF16)
        C4 = dev(wl.to_storage(rng.standard_normal((K, N4)) * 2.0, wl.BF16)[0], wl.BF16)
        o4 = [torch.empty((T4, N4), dtype=torch.int16, device="cuda") for _ in range(2)]
        t4 = bench_small(lambda i, s: bda.bda_kv_project(c4, d_c, T4, d_c, d_h, [128, 128], [0, 0], C4, N4,
                                                         o4[i % 2], N4, wl.BF16, wl.BF16, s), max(3, args.steps // 10), max(1, args.warmup // 10))
        f4 = 2.0 * T4 * K * N4
        b4 = (T4 * d_c + K * N4 + T4 * N4) * 2.0
        extra["v3_kv_T8192_bf16"] = {"us": t4 * 1e6, "tflops": f4 / t4 / 1e12, "frac_mfma": f4 / t4 / 1e12 / MFMA_PEAK_TFLOPS,
                                     "gbs": b4 / t4 / 1e9, "frac_hbm": b4 / t4 / 1e9 / HBM_PEAK_GBS,
                                     "tokens_per_s": T4 / t4}
        log(f"v3: {t4 * 1e6:.1f} us, {f4 / t4 / 1e12:.0f} TFLOP/s, {b4 / t4 / 1e9:.0f} GB/s")
        # decode shapes at the V3 width (not a BASELINE config; 24 MiB of C per launch, 12 rotating
        # copies so that each launch streams them from HBM): the one small-T case with enough bytes
        # for the HBM rate to show
        n_w4 = 12
        C4_rot = C4.unsqueeze(0).repeat(n_w4, 1, 1).contiguous()
        dec4 = {}
        for Td in (1, 8, 32, 64):
            cd = c4[:Td].contiguous()
            od = torch.empty((Td, N4), dtype=torch.int16, device="cuda")
            t_d = bench_small(lambda i, s: bda.bda_kv_project(cd, d_c, Td, d_c, d_h, [128, 128], [0, 0], C4_rot[i % n_w4], N4,
                                                              od, N4, wl.BF16, wl.BF16, s), max(8, min(240, args.steps)), max(2, min(48, args.warmup)))
            by = (Td * d_c + K * N4 + Td * N4) * 2.0
            dec4[f"T{Td}"] = {"us": t_d * 1e6, "gbs": by / t_d / 1e9, "frac_hbm": by / t_d / 1e9 / HBM_PEAK_GBS}
            log(f"decode at V3 width T={Td}: {t_d * 1e6:.2f} us, {by / t_d / 1e9:.0f} GB/s")
        extra["decode_v3_width"] = dec4
        del C4_rot
        W4 = dev(wl.to_storage(rng.standard_normal((d_c, N4)) * 0.02, wl.BF16)[0], wl.BF16)
        t4d = bench_small(lambda i, s: bda.bda_dense_project(c4, d_c, T4, d_c, W4, N4, N4, o4[i % 2], N4,
                                                             wl.BF16, wl.BF16, s), max(3, args.steps // 10), max(1, args.warmup // 10))
        extra["v3_dense_T8192_bf16"] = {"us": t4d * 1e6, "tflops": 2.0 * T4 * d_c * N4 / t4d / 1e12}
        extra["v3_speedup_vs_dense"] = {"measured": t4d / t4, "theoretical": d_c / K}
        del c4, C4, o4, W4
        # token-count sweep on the V3 k_proj shape (N = 16384, bf16; same weights every launch, as in
        # the throughput tables of Section "BDA Inference Efficiency"): BD projection, our dense
        # comparator, and the vendor GEMM (torch.matmul) doing the dense product
        Ns = 128 * 128
        sweep_T = () if args.no_sweep else (1, 8, 32, 64, 128, 256, 512, 1024, 2048, 4096, 8192)
        Cs_ = dev(wl.to_storage(rng.standard_normal((K, Ns)) * 2.0, wl.BF16)[0], wl.BF16)
        Ws_ = dev(wl.to_storage(rng.standard_normal((d_c, Ns)) * 0.02, wl.BF16)[0], wl.BF16)
        sweep = {}
        for Ts in sweep_T:
            cs_ = dev(wl.to_storage(rng.standard_normal((Ts, d_c)), wl.BF16)[0], wl.BF16)
            os_ = torch.empty((Ts, Ns), dtype=torch.int16, device="cuda")
            n_s, n_w = (max(4, min(100, args.steps // 2)), 4) if Ts <= 2048 else (max(3, min(20, args.steps // 10)), 4)
            bd_s = lambda i, s: bda.bda_kv_project(cs_, d_c, Ts, d_c, d_h, [128], [0], Cs_, Ns, os_, Ns, wl.BF16, wl.BF16, s)
            bench_small(bd_s, n_s, n_w)                    # untimed: clocks settle on this shape first
            t_b = bench_small(lambda i, s: bda.bda_kv_project(cs_, d_c, Ts, d_c, d_h, [128], [0], Cs_, Ns, os_, Ns,
                                                              wl.BF16, wl.BF16, s), n_s, n_w)
            t_d = bench_small(lambda i, s: bda.bda_dense_project(cs_, d_c, Ts, d_c, Ws_, Ns, Ns, os_, Ns,
                                                                 wl.BF16, wl.BF16, s), n_s, n_w)
            cb_, Wb_, ob_ = cs_.view(torch.bfloat16), Ws_.view(torch.bfloat16), os_.view(torch.bfloat16)
            t_v = bench_small(lambda i, s: torch.matmul(cb_, Wb_, out=ob_), n_s, n_w)
            sweep[f"T{Ts}"] = {"bd_us": t_b * 1e6, "dense_us": t_d * 1e6, "vendor_dense_us": t_v * 1e6,
                               "vendor_dense_over_bd": t_v / t_b}
        if sweep:
            extra["token_sweep_v3_kproj_bf16"] = sweep
            log("sweep (BD / dense / vendor dense, us): " + ", ".join(
                f"T={k[1:]} {v['bd_us']:.1f}/{v['dense_us']:.1f}/{v['vendor_dense_us']:.1f}" for k, v in sweep.items()))
        del Cs_, Ws_
        # BD low-rank linear (config 5), fp16, timing-only weights
        T5, d_in, r5, d_out = 8192, 4096, 1024, 11008
        x5 = torch.randn((T5, d_in), device="cuda").to(torch.float16)
        U5 = (torch.randn((d_in, r5), device="cuda") * 0.01).to(torch.float16)
        C5 = (torch.randn((r5, d_out - r5), device="cuda") * 0.03).to(torch.float16)
        o5 = torch.empty((T5, d_out), dtype=torch.float16, device="cuda")
        t5 = bench_small(lambda i, s: bda.bda_lowrank_linear(x5, d_in, T5, d_in, r5, d_out, 0, U5, C5, o5, d_out,
                                                             wl.F16, s), max(3, args.steps // 20), max(1, args.warmup // 20))
        f5 = 2.0 * T5 * (d_in * r5 + r5 * (d_out - r5))
        extra["lowrank_linear_T8192_f16"] = {"us": t5 * 1e6, "tflops": f5 / t5 / 1e12,
                                             "frac_mfma": f5 / t5 / 1e12 / MFMA_PEAK_TFLOPS, "tokens_per_s": T5 / t5}
        log(f"lowrank: {t5 * 1e6:.1f} us, {f5 / t5 / 1e12:.0f} TFLOP/s")
        # comparator: the plain low-rank pair (x U) V through the dense kernel
        V5 = (torch.randn((r5, d_out), device="cuda") * 0.02).to(torch.float16)
        h5 = torch.empty((T5, r5), dtype=torch.float16, device="cuda")

        def lowrank_plain(i, s):
            bda.bda_dense_project(x5, d_in, T5, d_in, U5, r5, r5, h5, r5, wl.F16, wl.F16, s)
            bda.bda_dense_project(h5, r5, T5, r5, V5, d_out, d_out, o5, d_out, wl.F16, wl.F16, s)
        t5p = bench_small(lowrank_plain, max(3, args.steps // 20), max(1, args.warmup // 20))
        extra["lowrank_plain_T8192_f16"] = {"us": t5p * 1e6}
        extra["lowrank_speedup_vs_plain"] = {"measured": t5p / t5, "theoretical": (d_in + d_out) / (d_in + d_out - r5)}
        del x5, U5, C5, o5, V5, h5
        # preparation itself (off the hot path): host float64 routine vs the GPU routine, first window
        prep = {"host_v2lite_32_heads_s": t_prep_host}
        for name, Hh, cdt in (("v2lite_32_heads", 32, wl.F16), ("v3_256_heads", 256, wl.BF16)):
            Wp = torch.randn((d_c, Hh * d_h), dtype=torch.float32, device="cuda") * 0.02
            Cp = torch.empty((K, Hh * d_h), dtype=torch.int16, device="cuda")
            flag = torch.zeros(1, dtype=torch.int32, device="cuda")
            t_p = bench_small(lambda i, s: bda.bda_prepare_device(Wp, Hh * d_h, wl.F32, d_c, Hh, d_h, 0, Cp, Hh * d_h, cdt, flag, s),
                              steps=5, warmup=1, graph=False)
            prep[f"device_{name}_us"] = t_p * 1e6
            assert int(flag.item()) == 0
        extra["prepare"] = prep
        log("prepare: " + ", ".join(f"{k} {v:.3g}" for k, v in prep.items()))
    result["extra"] = extra

    # ------------------------------------------------------------------ CPU baseline: the oracle
    if not args.no_cpu_baseline:
        import oracle
        probe = 8
        t0 = time.perf_counter()
        oracle.kv_project(w.c[:probe], C64, d_h, H, offs)
        per_tok = (time.perf_counter() - t0) / probe
        n = int(min(T, max(probe, args.cpu_seconds / max(per_tok, 1e-9))))
        t0 = time.perf_counter()
        oracle.kv_project(w.c[:n], C64, d_h, H, offs)
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": n / dt, "unit": "tokens/s", "cores": oracle.num_threads(),
                                  "kind": "oracle",
                                  "sample": f"first {n} of {T} tokens of the same workload, all {N} output columns, "
                                            f"fp64 C loops, {dt:.1f} s"}
        log(f"cpu oracle: {n} tokens in {dt:.1f} s on {oracle.num_threads()} threads")
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
