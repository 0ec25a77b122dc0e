#!/usr/bin/env python3
"""Benchmark of the BD K/V up-projection hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--rotate R] [--no-graph] [--no-extras]
                    [--no-sweep] [--no-cpu-baseline] [--workload v3|v2lite]

A "step" is one bda_kv_project call over one batch of the DeepSeek-V3-shaped workload (T = 8192
tokens, d_c = 512, 128 K_nope + 128 V heads of 128, bf16; weights from the library's own
bda_prepare): latent tile load, reduced-K MFMA GEMM over all heads, identity slice, rounding and
store.  Inputs are resident in HBM before the timed region.  Each step works on its own (c, out)
buffer pair out of R rotating pairs (an output alone is 512 MiB, twice the last-level cache); the
weights C are shared, as within a layer.  The K steps are captured once into a HIP graph (untimed)
and the timed region is one replay of that graph = exactly K launches, bracketed by
synchronisation; `--no-graph` times a plain launch loop.  `--workload v2lite` puts the
V2-Lite-shaped fp16 workload (T = 4096) on the main line instead (for profiling that shape alone).

Prints ONE JSON line on stdout (progress goes to stderr).  Besides the contract's fields the line
carries `roofline` (the step's kernel against the published MFMA peak, with the HBM view of the same
launch inside), `cpu_baseline` (the oracle on a bounded token sample) and `extra`: the other
workloads of the path, each timed for a fixed minimum (>= 50 ms and >= 30 launches after >= 10
warm-up launches, whatever --steps says), BD and dense timed alternately, and yardsticks measured in
the same process (empty-launch floor, register-resident MFMA rate, streaming read / write / copy).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

import numpy as np

MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense fp16/bf16 MFMA
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E

METRIC = "BD K/V proj tokens/s, TFLOP/s & GB/s vs roofline; speedup vs dense projection"
ROOT = os.path.dirname(os.path.abspath(__file__))


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--rotate", type=int, default=2, help="distinct (c, out) buffer pairs of the main workload")
    ap.add_argument("--workload", choices=("v3", "v2lite"), default="v3")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--tile-policy", type=int, default=0,
                    help="tile policy of the main workload's launches (0 = the library's own choice; see include/bda.h)")
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
    use_graph = not args.no_graph

    if args.calib_copy:
        xs = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        ys = torch.empty_like(xs)
        for _ in range(3):
            ys.copy_(xs)
        torch.cuda.synchronize()
        del xs, ys

    # ------------------------------------------------------------------ timing helpers
    class Step:
        """A launch closure that can target the bench stream or a capture stream."""
        def __init__(self, fn):
            self.fn = fn

        def __call__(self, i):
            self.fn(i, sid)

        def with_stream(self, i, s):
            self.fn(i, s)

    def capture(step, n):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):                  # captures on a side stream of its own
            cap_id = int(torch.cuda.current_stream().cuda_stream)
            for i in range(n):
                step.with_stream(i, cap_id)
        torch.cuda.synchronize()
        g.replay()                                 # one untimed replay (graph upload)
        torch.cuda.synchronize()
        return g

    def timed_run(step, steps, warmup, graph):
        """Returns (wall seconds, GPU seconds by HIP events on the launch stream) for exactly `steps` launches."""
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if graph:
            g = capture(step, steps)
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
                step(i)
            e1.record()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
        return t1 - t0, e0.elapsed_time(e1) * 1e-3

    MIN_MS, MIN_LAUNCHES, MIN_WARMUP, GRAPH_NODES = 50.0, 30, 10, 400

    def plan_launches(fn):
        """>= 10 warm-up launches, then an estimate of the launch time from 5 more; returns how many
        launches make up the fixed minimum (>= 50 ms and >= 30 launches)."""
        for i in range(MIN_WARMUP):
            fn(i, sid)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(5):
            fn(i, sid)
        e1.record()
        torch.cuda.synchronize()
        est = max(e0.elapsed_time(e1) * 1e-3 / 5, 1e-7)
        return min(20000, max(MIN_LAUNCHES, int(math.ceil(MIN_MS * 1e-3 / est))))

    def bench_fixed(fn, graph=True):
        """Seconds per launch of fn(i, stream), over the fixed minimum.  Graph mode: a graph of up to
        400 launches, replayed as often as the minimum needs, all inside one pair of events."""
        n = plan_launches(fn)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if graph and use_graph:
            nodes = min(n, GRAPH_NODES)
            reps = (n + nodes - 1) // nodes
            g = capture(Step(fn), nodes)
            e0.record()
            for _ in range(reps):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e-3 / (nodes * reps)
        e0.record()
        for i in range(n):
            fn(i, sid)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / n

    def bench_ab(fn_a, fn_b, rounds=4):
        """Two launches timed alternately (A B A B ...), each turn >= a quarter of the fixed minimum,
        so that both see the same clock / power state.  Returns (seconds per A, seconds per B)."""
        fns = (fn_a, fn_b)
        per = [max(8, (plan_launches(f) + rounds - 1) // rounds) for f in fns]       # launches per turn
        nodes = [min(p, GRAPH_NODES) for p in per]
        reps = [(p + n - 1) // n for p, n in zip(per, nodes)]
        graphs = [capture(Step(f), n) for f, n in zip(fns, nodes)] if use_graph else None
        total = [0.0, 0.0]
        for _ in range(rounds):
            for which in (0, 1):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                if use_graph:
                    for _r in range(reps[which]):
                        graphs[which].replay()
                else:
                    for i in range(nodes[which] * reps[which]):
                        fns[which](i, sid)
                e1.record()
                torch.cuda.synchronize()
                total[which] += e0.elapsed_time(e1) * 1e-3
        return tuple(total[k] / (rounds * nodes[k] * reps[k]) for k in (0, 1))

    # ------------------------------------------------------------------ main workload
    name = args.workload
    w = wl.kv_workload(name)
    T, d_c, d_h, H, N, K = w.T, w.d_c, w.d_h, w.H, w.N, w.d_c - w.d_h
    tag = {"v3": "v3_kv_T8192_bf16", "v2lite": "v2lite_kv_T4096_f16"}[name]
    offs, Cs, col = [], [], 0
    t_prep0 = time.perf_counter()
    for Hg in H:                                  # library prepare (host, float64), first-r basis per group
        Cg, _, off, _ = bda.bda_prepare(w.W[:, col:col + Hg * d_h], d_c, Hg, d_h, mode=bda.BASIS_FIRST)
        Cs.append(Cg)
        offs.append(off)
        col += Hg * d_h
    t_prep_host = time.perf_counter() - t_prep0
    C_stored, C64 = wl.to_storage(np.hstack(Cs), w.dtype)
    log(f"workload {tag}: T={T} N={N} K={K} max|C|={np.abs(C64).max():.1f} (host prepare {t_prep_host:.2f} s)")
    R = max(1, args.rotate)
    C_d = dev(C_stored, w.dtype)
    c_bufs, o_bufs = [], []
    for r in range(R):
        cw = wl.kv_workload(name, seed=w.seed + 100 * r) if r else w
        c_bufs.append(dev(cw.c_stored, w.dtype))
        o_bufs.append(torch.empty((T, N), dtype=tdt[w.dtype], device="cuda"))

    main_fn = lambda i, s: bda.bda_kv_project_ex(c_bufs[i % R], d_c, T, d_c, d_h, H, offs, C_d, N,    # noqa: E731
                                                 o_bufs[i % R], N, w.dtype, w.dtype, s, args.tile_policy)
    main_step = Step(main_fn)
    # The chip needs on the order of 100 ms of work to reach its steady clock / power state: a
    # measurement taken after a cold start reads differently from the same launches a moment later
    # (extra.main_repeated_later shows the check).  So the step runs untimed for a while first.
    t_end = time.perf_counter() + args.prewarm_ms * 1e-3
    while time.perf_counter() < t_end:
        for i in range(16):
            main_step(i)
        torch.cuda.synchronize()
    wall, gpu = timed_run(main_step, args.steps, args.warmup, use_graph)
    ms_per_step = wall / args.steps * 1e3
    kernel_s = gpu / args.steps
    flops = 2.0 * T * K * N
    alg_bytes = (T * d_c + K * N + T * N) * 2.0
    tokens_per_s = T / (wall / args.steps)
    log(f"main: {ms_per_step * 1e3:.2f} us/step wall, {kernel_s * 1e6:.2f} us/launch by events, "
        f"{flops / kernel_s / 1e12:.1f} TFLOP/s, {alg_bytes / kernel_s / 1e9:.0f} GB/s")

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(tag, {}).get("bytes_per_launch")
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
        "dtype": wl.DTYPE_NAMES[w.dtype],
        "data": "synthetic",
        "config": {"workload": tag, "T": T, "d_c": d_c, "d_h": d_h, "heads": H,
                   "basis_offset": offs, "N": N, "K": K, "rotating_buffers": R, "weights": "bda_prepare (host fp64), first-r basis",
                   "launch": "hip_graph" if use_graph else "loop", "prewarm_ms": args.prewarm_ms,
                   "tile_policy": args.tile_policy},
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
        extra["timing_rule"] = (f"every figure below: >= {MIN_MS:.0f} ms and >= {MIN_LAUNCHES} launches after >= {MIN_WARMUP} "
                                f"warm-up launches, HIP events on the launch stream, independent of --steps")

        def rate(t, fl, by):
            return {"us": t * 1e6, "tflops": fl / t / 1e12, "frac_mfma": fl / t / 1e12 / MFMA_PEAK_TFLOPS,
                    "gbs": by / t / 1e9, "frac_hbm": by / t / 1e9 / HBM_PEAK_GBS}

        # ---- yardsticks (library-free kernels, same process, same launch mode)
        ypath = os.path.join(ROOT, "paper_2510_01718_amd", "libbda_yardsticks.so")
        if os.path.exists(ypath):
            yl = ctypes.CDLL(ypath)
            vp, ci, u64, u32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32
            yl.bdy_empty.argtypes = [ci, ci, vp]
            yl.bdy_mfma_loop.argtypes = [ci, ci, ci, ci, vp, vp]
            yl.bdy_read.argtypes = [vp, u64, vp, ci, vp]
            yl.bdy_write.argtypes = [vp, u64, u32, ci, ci, vp]
            yl.bdy_copy.argtypes = [vp, vp, u64, ci, vp]
            yl.bdy_stage_model.argtypes = [vp, u64, ci, ci, vp, vp]
            sink = torch.zeros(64, dtype=torch.int32, device="cuda")
            y = {}

            def ck(rc):
                assert rc == 0, "yardstick launch failed"
            y["empty_launch_1x64_us"] = bench_fixed(lambda i, s: ck(yl.bdy_empty(1, 64, s or None))) * 1e6
            y["empty_launch_256x512_us"] = bench_fixed(lambda i, s: ck(yl.bdy_empty(256, 512, s or None))) * 1e6
            y["empty_launch_1x64_loop_us"] = bench_fixed(lambda i, s: ck(yl.bdy_empty(1, 64, s or None)), graph=False) * 1e6
            it = 2000
            for nm, bf in (("f16", 0), ("bf16", 1)):       # uniform operand values, then random ones (the board's power limit shows)
                for rnd, sfx in ((0, ""), (1, "_random_data")):
                    t_m = bench_fixed(lambda i, s: ck(yl.bdy_mfma_loop(512, it, bf, rnd, sink.data_ptr(), s or None)))
                    y[f"mfma_loop_{nm}{sfx}_tflops"] = 512 * 4 * it * 4 * 32768.0 / t_m / 1e12
            # The stage model: MFMAs + LDS fragment reads (+ DMA loads, load wait and barrier) of a 256 x 256 x 64
            # stage at the large-T kernels' ratios, nothing else; bf16 operands 0.5 <= |v| < 2 with random
            # signs and mantissas (what a launch on real data feeds the matrix cores), then zeros.
            win = 2 << 20
            g = torch.Generator(device="cuda").manual_seed(7)
            bits = torch.randint(0, 1 << 16, (8 * win // 2,), dtype=torch.int32, device="cuda", generator=g)
            model_src = ((bits & 0x80FF) | 0x3F00).to(torch.int16)       # sign, exponent 126 / 127, seven mantissa bits
            n_st = 1000
            for sfx, buf in (("random_data", model_src), ("zeros", torch.zeros_like(model_src))):
                for full, nm in ((0, "mfma_lds"), (1, "full")):
                    t_s = bench_fixed(lambda i, s: ck(yl.bdy_stage_model(buf.data_ptr(), win, n_st, full, sink.data_ptr(), s or None)))
                    y[f"stage_model_{nm}_{sfx}_tflops"] = 256 * 8 * 32 * 32768.0 * n_st / t_s / 1e12
            del bits, model_src
            big = 2 << 30                                      # 2 GiB: eight times the last-level cache
            src = torch.empty(big, dtype=torch.uint8, device="cuda").fill_(3)
            dst = torch.empty(big, dtype=torch.uint8, device="cuda")
            t_r = bench_fixed(lambda i, s: ck(yl.bdy_read(src.data_ptr(), big, sink.data_ptr(), 2048, s or None)))
            t_w = bench_fixed(lambda i, s: ck(yl.bdy_write(dst.data_ptr(), big, 7, 2048, 1, s or None)))
            t_wp = bench_fixed(lambda i, s: ck(yl.bdy_write(dst.data_ptr(), big, 7, 2048, 0, s or None)))
            t_c = bench_fixed(lambda i, s: ck(yl.bdy_copy(src.data_ptr(), dst.data_ptr(), big, 2048, s or None)))
            y["hbm_read_gbs"], y["hbm_write_gbs"], y["hbm_write_plain_stores_gbs"] = big / t_r / 1e9, big / t_w / 1e9, big / t_wp / 1e9
            y["hbm_copy_gbs_read_plus_write"] = 2 * big / t_c / 1e9
            del src, dst
            extra["yardsticks"] = y
            log("yardsticks: " + ", ".join(f"{k} {v:.4g}" for k, v in y.items()))
            result["roofline"]["frac_of_measured_mfma_loop"] = result["roofline"]["achieved"] / y[f"mfma_loop_{wl.DTYPE_NAMES[w.dtype]}_tflops"]
            result["roofline"]["frac_of_measured_mfma_loop_random_data"] = (
                result["roofline"]["achieved"] / y[f"mfma_loop_{wl.DTYPE_NAMES[w.dtype]}_random_data_tflops"])
            result["roofline"]["frac_of_stage_model_random_data"] = result["roofline"]["achieved"] / y["stage_model_full_random_data_tflops"]

        # ---- dense comparator of the main workload, timed alternately with the BD launch
        W_stored, _ = wl.to_storage(w.W, w.dtype)
        W_d = dev(W_stored, w.dtype)
        dense_fn = lambda i, s: bda.bda_dense_project(c_bufs[i % R], d_c, T, d_c, W_d, N, N, o_bufs[i % R], N, w.dtype, w.dtype, s)   # noqa: E731
        t_bd, t_dense = bench_ab(main_fn, dense_fn)
        extra["main_vs_dense_alternating"] = {"bd_us": t_bd * 1e6, "dense_us": t_dense * 1e6,
                                              "dense_tflops": 2.0 * T * d_c * N / t_dense / 1e12,
                                              "speedup": t_dense / t_bd, "theoretical": d_c / K}
        extra["speedup_vs_dense"] = {"measured": t_dense / t_bd, "theoretical": d_c / K}
        log(f"BD {t_bd * 1e6:.1f} us vs dense {t_dense * 1e6:.1f} us (alternating) -> speedup {t_dense / t_bd:.3f} (theory {d_c / K:.3f})")
        del W_d
        # basis windows inside the latent (Appendix "Residual-Min with Offset Search": window starts at
        # multiples of 16): the same launch with other window starts (timing only: C is not re-derived)
        win = {}
        for nm, o2 in (("last", [K, K]), ("offset_192", [192, 192]), ("offset_208", [208, 208])):
            t_f, t_o = bench_ab(main_fn, lambda i, s, o2=o2: bda.bda_kv_project(c_bufs[i % R], d_c, T, d_c, d_h, H, o2, C_d, N,
                                                                                 o_bufs[i % R], N, w.dtype, w.dtype, s))
            win[nm] = {"us": t_o * 1e6, "first_us": t_f * 1e6, "vs_first": t_o / t_f}
        extra["window_position_cost"] = win
        log("window position: " + ", ".join(f"{k} {v['us']:.2f} us ({v['vs_first']:.3f}x)" for k, v in win.items()))
        t_again = bench_fixed(main_fn)
        extra["main_repeated_later"] = {"us": t_again * 1e6, "vs_first_measurement": t_again / kernel_s}
        log(f"main again: {t_again * 1e6:.2f} us")
        # the same launch with float32 results (out_dtype = BDA_F32: twice the output bytes)
        o32 = [torch.empty((T, N), dtype=torch.float32, device="cuda") for _ in range(R)]
        t_32 = bench_fixed(lambda i, s: bda.bda_kv_project(c_bufs[i % R], d_c, T, d_c, d_h, H, offs, C_d, N, o32[i % R], N, w.dtype, wl.F32, s))
        extra["main_f32_out"] = {"us": t_32 * 1e6, "tflops": flops / t_32 / 1e12, "store_gbs": T * N * 4.0 / t_32 / 1e9}
        log(f"main with float32 results: {t_32 * 1e6:.2f} us, {T * N * 4.0 / t_32 / 1e9:.0f} GB/s of stores")
        del o32

        # ---- the other large configuration (the V2-Lite shape when the main line is the V3 shape, and vice versa)
        other = "v2lite" if name == "v3" else "v3"
        wo = wl.kv_workload(other)
        To, No = wo.T, wo.N
        Co, col = [], 0
        for Hg in wo.H:
            Cg, _, _, _ = bda.bda_prepare(wo.W[:, col:col + Hg * d_h], d_c, Hg, d_h, mode=bda.BASIS_FIRST)
            Co.append(Cg)
            col += Hg * d_h
        Co_d = dev(wl.to_storage(np.hstack(Co), wo.dtype)[0], wo.dtype)
        Wo_d = dev(wl.to_storage(wo.W, wo.dtype)[0], wo.dtype)
        Ro = 16 if other == "v2lite" else 2
        co_b = [dev(wl.kv_workload(other, seed=wo.seed + 100 * r).c_stored if r else wo.c_stored, wo.dtype) for r in range(Ro)]
        oo_b = [torch.empty((To, No), dtype=tdt[wo.dtype], device="cuda") for _ in range(Ro)]
        bd_o = lambda i, s: bda.bda_kv_project(co_b[i % Ro], d_c, To, d_c, d_h, wo.H, [0, 0], Co_d, No, oo_b[i % Ro], No, wo.dtype, wo.dtype, s)   # noqa: E731
        de_o = lambda i, s: bda.bda_dense_project(co_b[i % Ro], d_c, To, d_c, Wo_d, No, No, oo_b[i % Ro], No, wo.dtype, wo.dtype, s)                # noqa: E731
        t_b, t_d = bench_ab(bd_o, de_o)
        otag = {"v3": "v3_kv_T8192_bf16", "v2lite": "v2lite_kv_T4096_f16"}[other]
        extra[otag] = dict(rate(t_b, 2.0 * To * K * No, (To * d_c + K * No + To * No) * 2.0), tokens_per_s=To / t_b,
                           dense_us=t_d * 1e6, speedup_vs_dense=t_d / t_b, rotating_buffers=Ro)
        log(f"{otag}: BD {t_b * 1e6:.2f} us ({2.0 * To * K * No / t_b / 1e12:.0f} TFLOP/s), dense {t_d * 1e6:.2f} us, speedup {t_d / t_b:.3f}")

        # ---- gradients (Section "BDA Training Evaluation") on the V2-Lite and the V3 shape
        def backward_rates(label, Tb, Hb, dt, c_list, o_list, Cb_d):
            Nb = sum(Hb) * d_h
            fl = 2.0 * Tb * K * Nb
            gc_b = torch.empty((Tb, d_c), dtype=tdt[dt], device="cuda")
            gC_b = torch.empty((K, Nb), dtype=tdt[dt], device="cuda")
            nb = len(o_list)
            t_gc = bench_fixed(lambda i, s: bda.bda_kv_project_backward(None, d_c, o_list[i % nb], Nb, Cb_d, Nb, Tb, d_c, d_h, Hb, [0, 0],
                                                                        gc_b, d_c, None, Nb, dt, dt, s))
            t_gC = bench_fixed(lambda i, s: bda.bda_kv_project_backward(c_list[i % nb], d_c, o_list[i % nb], Nb, None, Nb, Tb, d_c, d_h, Hb, [0, 0],
                                                                        None, d_c, gC_b, Nb, dt, dt, s))
            t_fw = bench_fixed(lambda i, s: bda.bda_kv_project(c_list[i % nb], d_c, Tb, d_c, d_h, Hb, [0, 0], Cb_d, Nb, o_list[i % nb], Nb, dt, dt, s))
            extra[label] = {"grad_c_us": t_gc * 1e6, "grad_c_tflops": fl / t_gc / 1e12, "grad_C_us": t_gC * 1e6,
                            "grad_C_tflops": fl / t_gC / 1e12, "forward_us": t_fw * 1e6, "both_vs_forward": (t_gc + t_gC) / t_fw}
            log(f"{label}: grad_c {t_gc * 1e6:.1f} us, grad_C {t_gC * 1e6:.1f} us, forward {t_fw * 1e6:.1f} us")
        if name == "v3":
            backward_rates("backward_v2lite_T4096_f16", To, wo.H, wo.dtype, co_b, oo_b, Co_d)
            backward_rates("backward_v3_T8192_bf16", T, H, w.dtype, c_bufs, o_bufs, C_d)
        else:
            backward_rates("backward_v2lite_T4096_f16", T, H, w.dtype, c_bufs, o_bufs, C_d)
            backward_rates("backward_v3_T8192_bf16", To, wo.H, wo.dtype, co_b, oo_b, Co_d)

        # ---- decode shapes (config 3): the V2-Lite weights, rotating over distinct copies so that each
        # launch streams its 3 MiB of C from HBM, not from cache
        wd = wo if other == "v2lite" else w
        Cd_one = Co_d if other == "v2lite" else C_d
        Nd = wd.N
        n_w = 96
        C_rot = Cd_one.unsqueeze(0).repeat(n_w, 1, 1).contiguous()
        # the same copies in the packed layout of bda_pack_weights (32-column slices one after the other)
        P_rot = torch.empty_like(C_rot)
        for j in range(n_w):
            bda.bda_pack_weights(C_rot[j], Nd, d_c, d_h, wd.H, wd.dtype, P_rot[j], sid)
        torch.cuda.synchronize()
        floor = extra.get("yardsticks", {}).get("empty_launch_256x512_us")
        dec = {}
        for Td in (1, 8, 32, 64):
            cd = dev(wl.kv_workload("decode", T=Td).c_stored, wd.dtype)
            od = torch.empty((Td, Nd), dtype=tdt[wd.dtype], device="cuda")
            t_d = bench_fixed(lambda i, s: bda.bda_kv_project(cd, d_c, Td, d_c, d_h, wd.H, [0, 0], C_rot[i % n_w], Nd,
                                                              od, Nd, wd.dtype, wd.dtype, s))
            t_p = bench_fixed(lambda i, s: bda.bda_kv_project_packed(cd, d_c, Td, d_c, d_h, wd.H, [0, 0], P_rot[i % n_w],
                                                                     od, Nd, wd.dtype, wd.dtype, s))
            by = (Td * d_c + K * Nd + Td * Nd) * 2.0
            dec[f"T{Td}"] = {"us": t_d * 1e6, "gbs": by / t_d / 1e9, "frac_hbm": by / t_d / 1e9 / HBM_PEAK_GBS,
                             "vs_empty_launch": (t_d * 1e6 / floor) if floor else None,
                             "packed_us": t_p * 1e6, "packed_gbs": by / t_p / 1e9}
            log(f"decode T={Td}: {t_d * 1e6:.2f} us, {by / t_d / 1e9:.0f} GB/s; packed C {t_p * 1e6:.2f} us")
        extra["decode_v2lite"] = dec
        del C_rot, P_rot
        # decode shapes at the V3 width (not a BASELINE config; 24 MiB of C per launch, 12 rotating
        # copies so that each launch streams them from HBM)
        C4_one = C_d if name == "v3" else Co_d
        c4_src = c_bufs[0] if name == "v3" else co_b[0]
        N4, H4, dt4 = 256 * 128, [128, 128], wl.BF16
        n_w4 = 12
        C4_rot = C4_one.unsqueeze(0).repeat(n_w4, 1, 1).contiguous()
        P4_rot = torch.empty_like(C4_rot)
        for j in range(n_w4):
            bda.bda_pack_weights(C4_rot[j], N4, d_c, d_h, H4, dt4, P4_rot[j], sid)
        torch.cuda.synchronize()
        dec4 = {}
        for Td in (1, 8, 32, 64):
            cd = c4_src[:Td].contiguous()
            od = torch.empty((Td, N4), dtype=torch.int16, device="cuda")
            t_d = bench_fixed(lambda i, s: bda.bda_kv_project(cd, d_c, Td, d_c, d_h, H4, [0, 0], C4_rot[i % n_w4], N4,
                                                              od, N4, dt4, dt4, s))
            t_p = bench_fixed(lambda i, s: bda.bda_kv_project_packed(cd, d_c, Td, d_c, d_h, H4, [0, 0], P4_rot[i % n_w4],
                                                                     od, N4, dt4, dt4, s))
            by = (Td * d_c + K * N4 + Td * N4) * 2.0
            dec4[f"T{Td}"] = {"us": t_d * 1e6, "gbs": by / t_d / 1e9, "frac_hbm": by / t_d / 1e9 / HBM_PEAK_GBS,
                              "packed_us": t_p * 1e6, "packed_gbs": by / t_p / 1e9}
            log(f"decode at V3 width T={Td}: {t_d * 1e6:.2f} us, {by / t_d / 1e9:.0f} GB/s; packed C {t_p * 1e6:.2f} us")
        extra["decode_v3_width"] = dec4
        del C4_rot, P4_rot, co_b, oo_b, Co_d, Wo_d

        # ---- token-count sweep on the V3 k_proj shape (N = 16384, bf16; same weights every launch, as in
        # the throughput tables of Section "BDA Inference Efficiency"): BD projection, our dense
        # comparator, and the vendor GEMM (torch.matmul) doing the dense product
        rng = np.random.default_rng(2)
        Ns = 128 * 128
        sweep_T = () if args.no_sweep else (1, 8, 32, 64, 128, 256, 512, 1024, 2048, 4096, 8192)
        Cs_ = dev(wl.to_storage(rng.standard_normal((K, Ns)) * 2.0, wl.BF16)[0], wl.BF16)
        Ws_ = dev(wl.to_storage(rng.standard_normal((d_c, Ns)) * 0.02, wl.BF16)[0], wl.BF16)
        sweep = {}
        for Ts in sweep_T:
            cs_ = dev(wl.to_storage(rng.standard_normal((Ts, d_c)), wl.BF16)[0], wl.BF16)
            os_ = torch.empty((Ts, Ns), dtype=torch.int16, device="cuda")
            t_b, t_d = bench_ab(lambda i, s: bda.bda_kv_project(cs_, d_c, Ts, d_c, d_h, [128], [0], Cs_, Ns, os_, Ns, wl.BF16, wl.BF16, s),
                                lambda i, s: bda.bda_dense_project(cs_, d_c, Ts, d_c, Ws_, Ns, Ns, os_, Ns, wl.BF16, wl.BF16, s))
            cb_, Wb_, ob_ = cs_.view(torch.bfloat16), Ws_.view(torch.bfloat16), os_.view(torch.bfloat16)
            t_v = bench_fixed(lambda i, s: torch.matmul(cb_, Wb_, out=ob_))
            sweep[f"T{Ts}"] = {"bd_us": t_b * 1e6, "dense_us": t_d * 1e6, "vendor_dense_us": t_v * 1e6,
                               "dense_over_bd": t_d / t_b, "vendor_dense_over_bd": t_v / t_b}
        if sweep:
            extra["token_sweep_v3_kproj_bf16"] = sweep
            log("sweep (BD / dense / vendor dense, us): " + ", ".join(
                f"T={k[1:]} {v['bd_us']:.1f}/{v['dense_us']:.1f}/{v['vendor_dense_us']:.1f}" for k, v in sweep.items()))
        del Cs_, Ws_

        # ---- BD low-rank linear (config 5), fp16, timing-only weights, against the plain low-rank pair
        T5, d_in, r5, d_out = 8192, 4096, 1024, 11008
        x5 = torch.randn((T5, d_in), device="cuda").to(torch.float16)
        U5 = (torch.randn((d_in, r5), device="cuda") * 0.01).to(torch.float16)
        C5 = (torch.randn((r5, d_out - r5), device="cuda") * 0.03).to(torch.float16)
        o5 = torch.empty((T5, d_out), dtype=torch.float16, device="cuda")
        V5 = (torch.randn((r5, d_out), device="cuda") * 0.02).to(torch.float16)
        h5 = torch.empty((T5, r5), dtype=torch.float16, device="cuda")

        def lowrank_plain(i, s):
            bda.bda_dense_project(x5, d_in, T5, d_in, U5, r5, r5, h5, r5, wl.F16, wl.F16, s)
            bda.bda_dense_project(h5, r5, T5, r5, V5, d_out, d_out, o5, d_out, wl.F16, wl.F16, s)
        t5, t5p = bench_ab(lambda i, s: bda.bda_lowrank_linear(x5, d_in, T5, d_in, r5, d_out, 0, U5, C5, o5, d_out, wl.F16, s), lowrank_plain)
        f5 = 2.0 * T5 * (d_in * r5 + r5 * (d_out - r5))
        extra["lowrank_linear_T8192_f16"] = {"us": t5 * 1e6, "tflops": f5 / t5 / 1e12, "frac_mfma": f5 / t5 / 1e12 / MFMA_PEAK_TFLOPS,
                                             "tokens_per_s": T5 / t5, "plain_lowrank_pair_us": t5p * 1e6,
                                             "speedup_vs_plain": t5p / t5, "theoretical": (d_in + d_out) / (d_in + d_out - r5)}
        log(f"lowrank: {t5 * 1e6:.1f} us, {f5 / t5 / 1e12:.0f} TFLOP/s; plain pair {t5p * 1e6:.1f} us")
        del x5, U5, C5, o5, V5, h5

        # ---- preparation itself (off the hot path): host float64 routine vs the GPU routine, first window
        prep = {f"host_{tag}_s": t_prep_host}
        for nm, Hh, cdt in (("v2lite_32_heads", 32, wl.F16), ("v3_256_heads", 256, wl.BF16)):
            Wp = torch.randn((d_c, Hh * d_h), dtype=torch.float32, device="cuda") * 0.02
            Cp = torch.empty((K, Hh * d_h), dtype=torch.int16, device="cuda")
            flag = torch.zeros(1, dtype=torch.int32, device="cuda")
            t_p = bench_fixed(lambda i, s: bda.bda_prepare_device(Wp, Hh * d_h, wl.F32, d_c, Hh, d_h, 0, Cp, Hh * d_h, cdt, flag, s), graph=False)
            prep[f"device_{nm}_us"] = t_p * 1e6
            assert int(flag.item()) == 0
        # One layer of the V2-Lite shape prepared on the GPU as the paper's algorithms do it: keys with the query
        # weight as companion (16 heads, W_q 2048 x 2048), values with the output weight (W_o 2048 x 2048), C and the
        # companion stored in fp16, window by Residual-min and by offset search (25 candidate windows).  A model has
        # 27 such layers (context: the paper's preparation-time table is for whole models on other hardware).
        Hl, d_model = 16, 2048
        Wl = torch.randn((d_c, Hl * d_h), dtype=torch.float32, device="cuda") * 0.02
        Wq_l = torch.randn((d_model, Hl * d_h), dtype=torch.float32, device="cuda") * 0.02
        Wo_l = torch.randn((Hl * d_h, d_model), dtype=torch.float32, device="cuda") * 0.02
        Cl = torch.empty((K, Hl * d_h), dtype=torch.float16, device="cuda")
        Sq = torch.empty_like(Wq_l, dtype=torch.float16)
        So = torch.empty_like(Wo_l, dtype=torch.float16)
        off_l = torch.zeros(1, dtype=torch.int32, device="cuda")
        res_l = torch.zeros(3, dtype=torch.float64, device="cuda")
        for mode, mname in ((bda.BASIS_RESIDUAL_MIN, "residual_min"), (bda.BASIS_OFFSET_SEARCH, "offset_search")):
            nb = bda.bda_prepare_device_workspace_bytes(d_c, Hl, d_h, mode, True)
            ws_l = torch.empty(nb, dtype=torch.uint8, device="cuda")

            def layer(i, s):
                flag.zero_()
                bda.bda_prepare_device_ex(Wl, Hl * d_h, wl.F32, d_c, Hl, d_h, Cl, Hl * d_h, wl.F16, side=Wq_l, ld_side=Hl * d_h,
                                          d_side=d_model, side_kind=bda.SIDE_Q, side_out=Sq, ld_side_out=Hl * d_h, mode=mode,
                                          basis_offset_out=off_l, resid_out=res_l, singular_head=flag, workspace=ws_l,
                                          workspace_bytes=nb, stream=s)
                bda.bda_prepare_device_ex(Wl, Hl * d_h, wl.F32, d_c, Hl, d_h, Cl, Hl * d_h, wl.F16, side=Wo_l, ld_side=d_model,
                                          d_side=d_model, side_kind=bda.SIDE_O, side_out=So, ld_side_out=d_model, mode=mode,
                                          basis_offset_out=off_l, resid_out=res_l, singular_head=flag, workspace=ws_l,
                                          workspace_bytes=nb, stream=s)
            layer(0, sid)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            layer(0, sid)
            torch.cuda.synchronize()
            prep[f"device_v2lite_layer_k_and_v_with_companions_{mname}_ms"] = (time.perf_counter() - t0) * 1e3
            assert int(flag.item()) == 0 and int(off_l.item()) >= 0
        # A whole model's worth: 27 such layers, offset search, layer l on stream l mod 8 with outputs and a workspace
        # per stream (one search keeps 16 of the 256 compute units busy in its inversions; the calls share nothing,
        # so independent projections overlap; a process has four hardware queues here and the runtime deals streams
        # out to them in turn, so eight streams cover all four whatever other streams the process has made).
        mode = bda.BASIS_OFFSET_SEARCH
        nb = bda.bda_prepare_device_workspace_bytes(d_c, Hl, d_h, mode, True)
        lanes = []
        for _ in range(8):
            lanes.append(dict(stream=torch.cuda.Stream(), C=torch.empty_like(Cl), Sq=torch.empty_like(Sq), So=torch.empty_like(So),
                              off=torch.zeros(2, dtype=torch.int32, device="cuda"), res=torch.zeros(6, dtype=torch.float64, device="cuda"),
                              flag=torch.zeros(2, dtype=torch.int32, device="cuda"),
                              ws=[torch.empty(nb, dtype=torch.uint8, device="cuda") for _ in range(2)]))

        def model(n_layers):
            for layer_no in range(n_layers):
                b = lanes[layer_no % 8]
                s = int(b["stream"].cuda_stream)
                bda.bda_prepare_device_ex(Wl, Hl * d_h, wl.F32, d_c, Hl, d_h, b["C"], Hl * d_h, wl.F16, side=Wq_l, ld_side=Hl * d_h,
                                          d_side=d_model, side_kind=bda.SIDE_Q, side_out=b["Sq"], ld_side_out=Hl * d_h, mode=mode,
                                          basis_offset_out=b["off"][:1], resid_out=b["res"][:3], singular_head=b["flag"][:1],
                                          workspace=b["ws"][0], workspace_bytes=nb, stream=s)
                bda.bda_prepare_device_ex(Wl, Hl * d_h, wl.F32, d_c, Hl, d_h, b["C"], Hl * d_h, wl.F16, side=Wo_l, ld_side=d_model,
                                          d_side=d_model, side_kind=bda.SIDE_O, side_out=b["So"], ld_side_out=d_model, mode=mode,
                                          basis_offset_out=b["off"][1:], resid_out=b["res"][3:], singular_head=b["flag"][1:],
                                          workspace=b["ws"][1], workspace_bytes=nb, stream=s)
        model(8)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        model(27)
        torch.cuda.synchronize()
        prep["device_v2lite_model_27_layers_offset_search_8_streams_s"] = time.perf_counter() - t0
        assert all(int(b["flag"].sum().item()) == 0 for b in lanes)
        del lanes
        extra["prepare"] = prep
        log("prepare: " + ", ".join(f"{k} {v:.3g}" for k, v in prep.items()))
    result["extra"] = extra

    # ------------------------------------------------------------------ CPU baseline: the oracle
    if not args.no_cpu_baseline:
        import oracle
        probe = min(T, 128)                    # (a handful of tokens would not keep the oracle's threads busy and overestimate)
        oracle.kv_project(w.c[:8], C64, d_h, H, offs)
        t0 = time.perf_counter()
        oracle.kv_project(w.c[:probe], C64, d_h, H, offs)
        per_tok = (time.perf_counter() - t0) / probe
        n = int(min(T, max(256, args.cpu_seconds / max(per_tok, 1e-9))))
        t0 = time.perf_counter()
        oracle.kv_project(w.c[:n], C64, d_h, H, offs)
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": n / dt, "unit": "tokens/s", "cores": oracle.num_threads(),
                                  "kind": "oracle",
                                  "sample": f"first {n} of {T} tokens of the same workload ({tag}), all {N} output columns, "
                                            f"fp64 C loops, {dt:.1f} s"}
        log(f"cpu oracle: {n} tokens in {dt:.1f} s on {oracle.num_threads()} threads")
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
