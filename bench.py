#!/usr/bin/env python3
"""Benchmark of the fused attention forward path on one MI355X.

A step is one attn_fwd call (the whole hot path: tile streaming, QK^T, mask,
streaming softmax, PV, epilogue) on the configuration the headline metric is
quoted on: B=2, Hq=Hkv=32, N=8192, d=128, bf16, non-causal, synthetic N(0,1)*0.5
inputs already resident in HBM.  Prints ONE JSON line on stdout.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config I] [--variant V]
                  [--no-cpu-baseline] [--all-configs] [--paper-grid] [--copy-calibration] [--zero-operands]

--paper-grid also times the paper's own attention shape grid (appendix A: batch 4, 48 heads,
N = 1024 .. 16384, d = 128, causal and non-causal) and reports it under 'paper_grid'.
--zero-operands also times the same launch on all-zero q, k, v (reported in 'zero_operands'): the
same instruction stream with nothing toggling in the data paths, which the board runs at its full
clock: the gap to the headline figure is what the power limit costs on random data.
--copy-calibration runs nothing but a 1 GiB device-to-device copy (three times): under
`rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` it gives the factor that converts those
counters into bytes (see profiles/).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2516.6, "fp8_e4m3": 5033.2}  # 256 CUs x 2.4 GHz x 4096 (8192) flop/clk/CU, dense
# The default fp8 kernel takes the scores on the fp8 matrix path and P V on the bf16 path (half of the
# flops each): the rate at which the matrix pipe alone could run that mix is 2 / (1/5033.2 + 1/2516.6).
FP8_MIXED_PATH_CEILING_TFLOPS = 2.0 / (1.0 / 5033.2 + 1.0 / 2516.6)
# Figures that come from rocprofv3 runs recorded under profiles/, not from this run: HBM bytes per launch
# (FETCH_SIZE x 2.0 KiB + WRITE_SIZE x 1.0 KiB, factors from a 1 GiB copy) and the shader clock the
# kernel sustains (GRBM_GUI_ACTIVE / 8 / kernel duration).  None where no such run has been made.
PROFILED = {"long_noncausal_8k": {"traffic_bytes": 5.393e8, "shader_clock_ghz": 1.65,
                                  "source": "profiles/attn_fwd_sp_bf16_long_noncausal_8k.md"}}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_config(A, torch, cfg, steps, warmup, variant=None, zero_operands=False):
    import workloads as wl

    inp = wl.make_inputs(cfg)
    dev = wl.to_device(inp)
    if zero_operands:
        for t in dev.values():
            t.zero_()
    B, Hq, Hkv, N, d = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["N"], cfg["d"]
    o = torch.empty((B, Hq, N, d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, Hq, N), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step(on=stream):
        if cfg["dtype"] == "bf16":
            if variant is None:
                A.attn_fwd(dev["q"], dev["k"], dev["v"], o, lse, B, Hq, Hkv, N, d, cfg["causal"], cfg["scale"], A.ATTN_BF16,
                           stream=on)
            else:
                A.attn_fwd_variant(dev["q"], dev["k"], dev["v"], o, lse, B, Hq, Hkv, N, d, cfg["causal"], cfg["scale"],
                                   A.ATTN_BF16, variant, stream=on)
        else:
            ds = inp["descale"]
            A.attn_fwd_fp8(dev["q"], dev["k"], dev["v"], o, lse, B, Hq, Hkv, N, d, cfg["causal"], cfg["scale"], ds[0], ds[1],
                           ds[2], stream=on)

    # per-launch durations from events recorded on the launch stream (created before the warm-up so
    # that nothing but the synchronisation sits between the warm-up and the timed steps)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in evs:
        a.record(stream)
        step()
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [a.elapsed_time(b) for a, b in evs]
    if os.environ.get("BENCH_TRACE"):
        log("[bench] per-step kernel ms: " + " ".join(f"{x:.4f}" for x in kern_ms))
    flops = wl.algorithmic_flops(cfg)
    return dict(inp=inp, dev=dev, o=o, lse=lse, wall_ms=wall * 1e3 / steps, kern_ms_avg=float(np.mean(kern_ms)),
                kern_ms_med=float(np.median(kern_ms)), flops=flops, step=step)


def time_paper_grid(A, torch, cfgs=None):
    """The paper's attention benchmark grid (or the given shapes), bf16.  Inputs are drawn on the
    device (seeded N(0,1), rounded to bf16): only their statistics matter for timing; parity on
    these shapes is covered by the tests."""
    import workloads as wl

    rows = []
    gen = torch.Generator(device="cuda")
    for cfg in (wl.paper_grid() if cfgs is None else cfgs):
        B, H, N, d = cfg["B"], cfg["Hq"], cfg["N"], cfg["d"]
        gen.manual_seed(cfg["seed"])
        q, k, v = (torch.randn((B, H, N, d), device="cuda", generator=gen).to(torch.bfloat16) for _ in range(3))
        o = torch.empty_like(q)
        lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        stream = torch.cuda.current_stream()

        def step(on=stream):
            A.attn_fwd(q, k, v, o, lse, B, H, H, N, d, cfg["causal"], cfg["scale"], A.ATTN_BF16, stream=on)

        flops = wl.algorithmic_flops(cfg)
        est = flops / 1.0e15
        for _ in range(max(3, min(200, int(0.05 / est)))):
            step()
        torch.cuda.synchronize()
        n = max(5, min(50, int(0.05 / est)))
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in evs:
            a.record(stream)
            step()
            b.record(stream)
        torch.cuda.synchronize()
        ms = float(np.median([a.elapsed_time(b) for a, b in evs]))
        tf = flops / (ms * 1e-3) / 1e12
        rows.append({"workload": cfg["name"], "kernel_ms": ms, "TFLOP/s": tf, "pct_of_dense_peak": 100 * tf / PEAK_TFLOPS["bf16"]})
        log(f"[bench] {cfg['name']}: {ms:.4f} ms  {tf:.1f} TFLOP/s = {100 * tf / PEAK_TFLOPS['bf16']:.1f}%")
        if ms < 0.3:  # short launches: also as one of 20 launches in a replayed graph
            gms = graph_ms(torch, step)
            gtf = flops / (gms * 1e-3) / 1e12
            rows[-1].update({"ms_in_graph": gms, "TFLOP/s_in_graph": gtf, "pct_of_dense_peak_in_graph": 100 * gtf / PEAK_TFLOPS["bf16"]})
            log(f"[bench] {cfg['name']} in a graph of 20 launches: {gms:.4f} ms per launch  {gtf:.1f} TFLOP/s = {100 * gtf / PEAK_TFLOPS['bf16']:.1f}%")
        del q, k, v, o, lse
    return rows


def time_persistent(A, torch, cfgs):
    """Static launch (one workgroup per query tile) against the persistent launch with the tile
    queue, same kernel code, interleaved in one process.  Inputs drawn on the device."""
    import workloads as wl

    rows = []
    gen = torch.Generator(device="cuda")
    for cfg in cfgs:
        B, Hq, Hkv, N, d = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["N"], cfg["d"]
        gen.manual_seed(cfg["seed"])
        sig = cfg.get("sigma", 1.0)
        q = (torch.randn((B, Hq, N, d), device="cuda", generator=gen) * sig).to(torch.bfloat16)
        k, v = ((torch.randn((B, Hkv, N, d), device="cuda", generator=gen) * sig).to(torch.bfloat16) for _ in range(2))
        o = torch.empty_like(q)
        lse = torch.empty((B, Hq, N), dtype=torch.float32, device="cuda")
        queue = torch.zeros(A.attn_persistent_queue_bytes(), dtype=torch.uint8, device="cuda")
        stream = torch.cuda.current_stream()
        twin = next(i for i in range(A.attn_num_variants()) if A.attn_variant_name(i) == f"bf16 d{d} pipelined BM256 BN64")

        def static():
            A.attn_fwd_variant(q, k, v, o, lse, B, Hq, Hkv, N, d, cfg["causal"], cfg["scale"], A.ATTN_BF16, twin, stream=stream)

        def persistent():
            A.attn_fwd_persistent(q, k, v, o, lse, B, Hq, Hkv, N, d, cfg["causal"], cfg["scale"], A.ATTN_BF16, queue, stream=stream)

        flops = wl.algorithmic_flops(cfg)
        est = flops / 1.0e15 + 5e-6
        n = max(5, min(50, int(0.05 / est)))
        res = {}
        for _ in range(max(3, n)):
            static()
            persistent()
        torch.cuda.synchronize()
        for rep in range(2):
            for name, fn in (("static", static), ("persistent", persistent)):
                evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
                for a, b in evs:
                    a.record(stream)
                    fn()
                    b.record(stream)
                torch.cuda.synchronize()
                res.setdefault(name, []).extend(a.elapsed_time(b) for a, b in evs)
        ms_s, ms_p = float(np.median(res["static"])), float(np.median(res["persistent"]))
        rows.append({"workload": cfg["name"], "static_ms": ms_s, "persistent_ms": ms_p,
                     "static_TFLOP/s": flops / ms_s / 1e9, "persistent_TFLOP/s": flops / ms_p / 1e9})
        log(f"[bench] {cfg['name']}: static {ms_s:.4f} ms ({flops / ms_s / 1e9:.1f} TFLOP/s)  persistent {ms_p:.4f} ms "
            f"({flops / ms_p / 1e9:.1f} TFLOP/s)")
        del q, k, v, o, lse
    return rows


def time_backward(A, torch, cfgs):
    """Backward pass (bf16, d = 128 or 64) on the given shapes: one step = attn_bwd (two kernels).
    Inputs are drawn on the device (seeded N(0,1), rounded to bf16) and O, lse come from
    attn_fwd on them; parity on these shapes is covered by the tests.  TFLOP/s counts the five
    N x N x d products of the textbook backward (2.5 x the forward figure)."""
    import workloads as wl

    rows = []
    gen = torch.Generator(device="cuda")
    for cfg in cfgs:
        B, Hq, Hkv, N, d = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["N"], cfg["d"]
        gen.manual_seed(cfg["seed"])
        sig = cfg.get("sigma", 1.0)
        q = (torch.randn((B, Hq, N, d), device="cuda", generator=gen) * sig).to(torch.bfloat16)
        k, v = ((torch.randn((B, Hkv, N, d), device="cuda", generator=gen) * sig).to(torch.bfloat16) for _ in range(2))
        do = torch.randn((B, Hq, N, d), device="cuda", generator=gen).to(torch.bfloat16)
        o, dq = torch.empty_like(q), torch.empty_like(q)
        dk, dv = torch.empty_like(k), torch.empty_like(v)
        lse = torch.empty((B, Hq, N), dtype=torch.float32, device="cuda")
        ws = torch.empty(A.attn_bwd_workspace_bytes(B, Hq, N) // 4, dtype=torch.float32, device="cuda")
        stream = torch.cuda.current_stream()
        A.attn_fwd(q, k, v, o, lse, B, Hq, Hkv, N, d, cfg["causal"], cfg["scale"], A.ATTN_BF16, stream=stream)

        def step():
            A.attn_bwd(q, k, v, o, do, lse, dq, dk, dv, ws, B, Hq, Hkv, N, d, cfg["causal"], cfg["scale"], A.ATTN_BF16,
                       stream=stream)

        flops = wl.algorithmic_flops_bwd(cfg)
        est = flops / 0.5e15
        for _ in range(max(3, min(100, int(0.05 / est)))):
            step()
        torch.cuda.synchronize()
        n = max(5, min(30, int(0.05 / est)))
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in evs:
            a.record(stream)
            step()
            b.record(stream)
        torch.cuda.synchronize()
        ms = float(np.median([a.elapsed_time(b) for a, b in evs]))
        tf = flops / (ms * 1e-3) / 1e12
        rows.append({"workload": cfg["name"], "ms": ms, "TFLOP/s": tf, "pct_of_dense_peak": 100 * tf / PEAK_TFLOPS["bf16"],
                     "algorithmic_flop": flops})
        log(f"[bench] backward {cfg['name']}: {ms:.4f} ms  {tf:.1f} TFLOP/s = {100 * tf / PEAK_TFLOPS['bf16']:.1f}%")
        del q, k, v, do, o, dq, dk, dv, lse, ws
    return rows


def graph_ms(torch, step_on, launches=20, replays=20):
    """Milliseconds per launch when `launches` calls of step_on(stream) are captured into one HIP
    graph and the graph is replayed: what a caller pays that does not go through the host for every
    launch.  Per-launch event pairs add about 5 microseconds to a kernel of a few microseconds."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step_on(side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(launches):
            step_on(side)
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    ts = []
    for _ in range(replays):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) / launches)
    return float(np.median(ts))


def time_gemm(A, torch, shapes, variants=(None,)):
    """bf16 GEMM on the paper's shapes.  Inputs drawn on the device (seeded N(0,1) rounded to
    bf16); parity on these shapes is covered by the tests."""
    import workloads as wl

    rows = []
    gen = torch.Generator(device="cuda")
    for g in shapes:
        M, N, K = g["M"], g["N"], g["K"]
        gen.manual_seed(g["seed"])
        a = torch.randn((M, K), device="cuda", generator=gen).to(torch.bfloat16)
        b = torch.randn((N, K), device="cuda", generator=gen).to(torch.bfloat16)
        c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        stream = torch.cuda.current_stream()
        flops = wl.gemm_flops(M, N, K)
        for var in variants:
            def step(on=stream):
                if var is None:
                    A.gemm_bf16_nt(a, b, c, M, N, K, stream=on)
                else:
                    A.gemm_bf16_nt_variant(a, b, c, M, N, K, var, stream=on)

            est = flops / 1.0e15 + 5e-6
            for _ in range(max(3, min(200, int(0.05 / est)))):
                step()
            torch.cuda.synchronize()
            n = max(5, min(50, int(0.05 / est)))
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
            for e0, e1 in evs:
                e0.record(stream)
                step()
                e1.record(stream)
            torch.cuda.synchronize()
            ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in evs]))
            tf = flops / (ms * 1e-3) / 1e12
            rows.append({"workload": g["name"], "variant": "library default" if var is None else A.gemm_variant_name(var),
                         "ms": ms, "TFLOP/s": tf, "pct_of_dense_peak": 100 * tf / PEAK_TFLOPS["bf16"]})
            log(f"[bench] gemm {g['name']} [{rows[-1]['variant']}]: {ms:.4f} ms  {tf:.1f} TFLOP/s = "
                f"{100 * tf / PEAK_TFLOPS['bf16']:.1f}%")
            if ms < 0.1:  # launch-bound: also as one of 20 launches in a replayed graph
                gms = graph_ms(torch, step)
                gtf = flops / (gms * 1e-3) / 1e12
                rows[-1].update({"ms_in_graph": gms, "TFLOP/s_in_graph": gtf, "pct_of_dense_peak_in_graph": 100 * gtf / PEAK_TFLOPS["bf16"]})
                log(f"[bench] gemm {g['name']} [{rows[-1]['variant']}] in a graph of 20 launches: {gms:.4f} ms per launch  "
                    f"{gtf:.1f} TFLOP/s = {100 * gtf / PEAK_TFLOPS['bf16']:.1f}%")
        # split-K with the slice count the library recommends (and a sweep of counts with --gemm-variants)
        plan = A.gemm_splitk_plan(M, N, K)
        counts = [plan] if plan > 1 else []
        if len(variants) > 1 and K % 64 == 0 and K >= 4096:
            counts = sorted(set(counts) | {2, 4, 8, 16})
        for splits in counts:
            ws = torch.empty(A.gemm_splitk_workspace_bytes(M, N, splits) // 4, dtype=torch.float32, device="cuda")

            def step_sk():
                A.gemm_bf16_nt_splitk(a, b, c, M, N, K, splits, ws, stream=stream)

            for _ in range(max(3, min(200, int(0.05 / est)))):
                step_sk()
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
            for e0, e1 in evs:
                e0.record(stream)
                step_sk()
                e1.record(stream)
            torch.cuda.synchronize()
            ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in evs]))
            tf = flops / (ms * 1e-3) / 1e12
            tag = f"split-K, {splits} slices" + (" (recommended)" if splits == plan else "")
            rows.append({"workload": g["name"], "variant": tag, "ms": ms, "TFLOP/s": tf, "pct_of_dense_peak": 100 * tf / PEAK_TFLOPS["bf16"]})
            log(f"[bench] gemm {g['name']} [{tag}]: {ms:.4f} ms  {tf:.1f} TFLOP/s = {100 * tf / PEAK_TFLOPS['bf16']:.1f}%")
            del ws
        if g["name"] in ("mi350_2048", "canonical_k4096", "canonical_k8192") and N % 8 == 0:
            bkn = b.t().contiguous()  # the second operand stored [K, N]

            def step_nn():
                A.gemm_bf16_nn(a, bkn, c, M, N, K, stream=stream)

            for _ in range(max(3, min(200, int(0.05 / est)))):
                step_nn()
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
            for e0, e1 in evs:
                e0.record(stream)
                step_nn()
                e1.record(stream)
            torch.cuda.synchronize()
            ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in evs]))
            tf = flops / (ms * 1e-3) / 1e12
            rows.append({"workload": g["name"], "variant": "gemm_bf16_nn (B stored [K,N]), library default", "ms": ms, "TFLOP/s": tf,
                         "pct_of_dense_peak": 100 * tf / PEAK_TFLOPS["bf16"]})
            log(f"[bench] gemm {g['name']} [nn]: {ms:.4f} ms  {tf:.1f} TFLOP/s = {100 * tf / PEAK_TFLOPS['bf16']:.1f}%")
            del bkn
        del a, b, c
    return rows


def cpu_baseline(cfg, inp, budget_s=20.0):
    """The oracle as it stands, timed on the host cores on a bounded sample: whole
    (b, h) heads of the same workload, one after another, until the time budget is
    used.  Rate = algorithmic FLOP of those heads / wall time."""
    from oracle import attn_ref as orc

    try:
        from threadpoolctl import threadpool_info

        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    N, d, G = cfg["N"], cfg["d"], cfg["Hq"] // cfg["Hkv"]
    per_head = 4.0 * N * N * d / (2 if cfg["causal"] else 1)
    heads = 0
    t0 = time.perf_counter()
    while True:
        b, h = divmod(heads, cfg["Hq"])
        if b >= cfg["B"]:
            break
        if inp["q"].dtype == np.uint16:
            dec = orc.bf16_bits_to_f64
            q, k, v = dec(inp["q"][b, h]), dec(inp["k"][b, h // G]), dec(inp["v"][b, h // G])
        else:
            ds = inp["descale"]
            dec = orc.e4m3_bits_to_f64
            q, k, v = dec(inp["q"][b, h]) * ds[0], dec(inp["k"][b, h // G]) * ds[1], dec(inp["v"][b, h // G]) * ds[2]
        orc.attn_head(q, k, v, cfg["causal"], cfg["scale"])
        heads += 1
        el = time.perf_counter() - t0
        if el > budget_s or el + el / heads > budget_s * 1.5:
            break
    el = time.perf_counter() - t0
    return {"value": per_head * heads / el / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{heads} of {cfg['B'] * cfg['Hq']} (batch, head) slices of the same workload, full N x N each, "
                      f"float64 numpy, {el:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=25)  # ~50 ms: the shader clock needs about that long to settle
    ap.add_argument("--config", type=int, default=2, help="index into workloads.CONFIGS (default: the headline config)")
    ap.add_argument("--variant", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--all-configs", action="store_true", help="also time the other bf16 configs (reported in 'others')")
    ap.add_argument("--paper-grid", action="store_true", help="also time the paper's attention shape grid (reported in 'paper_grid')")
    ap.add_argument("--backward", action="store_true",
                    help="also time attn_bwd on the chosen config (with --all-configs: every bf16 d=128 config; with "
                         "--paper-grid: the paper's grid as well); "
                         "reported in 'backward'")
    ap.add_argument("--extra-shapes", action="store_true",
                    help="also time head dimension 64 and ragged lengths at the headline size (reported in 'extra_shapes')")
    ap.add_argument("--persistent", action="store_true",
                    help="also compare the persistent tile-queue launch with the static one on the bf16 configs (with "
                         "--paper-grid: on the grid too); reported in 'persistent'")
    ap.add_argument("--gemm", action="store_true", help="also time the bf16 GEMM on the paper's shapes (reported in 'gemm')")
    ap.add_argument("--gemm-shape", default=None, help="with --gemm: only this shape (a name in workloads.GEMM_SHAPES)")
    ap.add_argument("--gemm-variants", action="store_true", help="with --gemm: time every kernel variant")
    ap.add_argument("--copy-calibration", action="store_true", help="only run a 1 GiB copy (counter calibration)")
    ap.add_argument("--zero-operands", action="store_true",
                    help="also time the same launch on all-zero inputs (same instructions, full clock; reported in 'zero_operands')")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (every (batch, head) is independent, so the path would "
              "shard over heads with no communication); --gpus N with N > 1 is not supported.", file=sys.stderr)
        sys.exit(2)

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "launches": 3}))
        return

    import paper_2605_10905_amd as A
    import workloads as wl

    cfg = wl.CONFIGS[args.config]
    log(f"[bench] config {args.config + 1}: {cfg['name']}  lib={A.lib_path}")
    r = time_config(A, torch, cfg, args.steps, args.warmup, args.variant)
    tflops = r["flops"] / (r["wall_ms"] * 1e-3) / 1e12
    kern_tflops = r["flops"] / (r["kern_ms_avg"] * 1e-3) / 1e12
    # priced against the dense-MFMA peak of the INPUT dtype
    vidx = args.variant if args.variant is not None else A.attn_default_variant(
        0 if cfg["dtype"] == "bf16" else 1, cfg["B"], cfg["Hq"], cfg["N"], cfg["d"])
    vname = A.attn_variant_name(vidx) or ""
    peak = PEAK_TFLOPS[cfg["dtype"]]
    mixed = cfg["dtype"] != "bf16" and "bf16-PV" in vname
    log(f"[bench] wall {r['wall_ms']:.4f} ms/step  kernel avg {r['kern_ms_avg']:.4f} ms (median {r['kern_ms_med']:.4f})  "
        f"{kern_tflops:.1f} TFLOP/s = {100 * kern_tflops / peak:.1f}% of dense peak")

    prof = PROFILED.get(cfg["name"], {}) if args.variant is None else {}
    out = {
        "metric": "attention fwd TFLOP/s and % of MI355X dense MFMA peak (bf16, N=8192, d=128)",
        "value": tflops,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": r["wall_ms"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg["dtype"] == "bf16" else ("fp8 QK^T + bf16 PV" if mixed else "fp8"),
        "data": "synthetic",
        "config": {"workload": f"{cfg['name']}: B={cfg['B']} Hq={cfg['Hq']} Hkv={cfg['Hkv']} N={cfg['N']} d={cfg['d']} "
                               f"{cfg['dtype']} {'causal' if cfg['causal'] else 'non-causal'}",
                   "variant": vname if args.variant is not None else f"library default ({vname})",
                   "pct_of_dense_peak": 100 * tflops / peak},
        "roofline": {"bound": "mfma", "achieved": kern_tflops, "peak": peak, "unit": "TFLOP/s", "frac": kern_tflops / peak,
                     "traffic": prof.get("traffic_bytes"), "traffic_source": prof.get("source"),
                     "shader_clock_ghz": prof.get("shader_clock_ghz"), "shader_clock_source": prof.get("source"),
                     "kernel_ms_avg": r["kern_ms_avg"], "kernel_ms_median": r["kern_ms_med"],
                     "algorithmic_flop_per_launch": r["flops"]},
    }
    if mixed:
        out["roofline"]["mixed_path_ceiling"] = FP8_MIXED_PATH_CEILING_TFLOPS
        out["roofline"]["frac_of_mixed_path_ceiling"] = kern_tflops / FP8_MIXED_PATH_CEILING_TFLOPS
    if args.zero_operands:
        rz = time_config(A, torch, cfg, args.steps, args.warmup, args.variant, zero_operands=True)
        tfz = rz["flops"] / (rz["kern_ms_avg"] * 1e-3) / 1e12
        out["zero_operands"] = {"kernel_ms_avg": rz["kern_ms_avg"], "kernel_ms_median": rz["kern_ms_med"], "TFLOP/s": tfz,
                                "pct_of_dense_peak": 100 * tfz / peak,
                                "what": "the same launch on all-zero q, k, v: identical instruction stream, no data toggling"}
        log(f"[bench] zero operands: kernel avg {rz['kern_ms_avg']:.4f} ms  {tfz:.1f} TFLOP/s = {100 * tfz / peak:.1f}% of dense peak")
        del rz
    if args.all_configs:
        others = []
        for i, c in enumerate(wl.CONFIGS):
            if i == args.config:
                continue
            rr = time_config(A, torch, c, max(5, args.steps // 2), 3)
            tf = rr["flops"] / (rr["kern_ms_med"] * 1e-3) / 1e12
            others.append({"workload": c["name"], "kernel_ms": rr["kern_ms_med"], "TFLOP/s": tf,
                           "pct_of_dense_peak": 100 * tf / PEAK_TFLOPS[c["dtype"]]})
            log(f"[bench] {c['name']}: {rr['kern_ms_med']:.4f} ms  {tf:.1f} TFLOP/s")
            if rr["kern_ms_med"] < 0.3:  # short launches: also as one of 20 launches in a replayed graph
                gms = graph_ms(torch, rr["step"])
                gtf = rr["flops"] / (gms * 1e-3) / 1e12
                others[-1].update({"ms_in_graph": gms, "TFLOP/s_in_graph": gtf, "pct_of_dense_peak_in_graph": 100 * gtf / PEAK_TFLOPS[c["dtype"]]})
                log(f"[bench] {c['name']} in a graph of 20 launches: {gms:.4f} ms per launch  {gtf:.1f} TFLOP/s")
            del rr
        out["others"] = others
    if args.paper_grid:
        out["paper_grid"] = time_paper_grid(A, torch)
    if args.extra_shapes:
        out["extra_shapes"] = time_paper_grid(A, torch, wl.extra_shapes())
    if args.backward:
        cfgs = [c for c in wl.CONFIGS if c["dtype"] == "bf16" and c["d"] == 128 and (args.all_configs or c is cfg)]
        if args.paper_grid:
            cfgs += wl.paper_grid()
        if args.extra_shapes:
            cfgs += [c for c in wl.extra_shapes() if c["d"] == 64]
        out["backward"] = time_backward(A, torch, cfgs)
    if args.persistent:
        cfgs = [c for c in wl.CONFIGS if c["dtype"] == "bf16"]
        if args.paper_grid:
            cfgs += wl.paper_grid()
        out["persistent"] = time_persistent(A, torch, cfgs)
    if args.gemm:
        variants = [None] + list(range(A.gemm_num_variants())) if args.gemm_variants else [None]
        shapes = [g for g in wl.GEMM_SHAPES if args.gemm_shape in (None, g["name"])]
        out["gemm"] = time_gemm(A, torch, shapes, variants)
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(cfg, r["inp"])
        log(f"[bench] cpu oracle: {out['cpu_baseline']}")
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
