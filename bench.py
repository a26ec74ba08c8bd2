#!/usr/bin/env python3
"""Benchmark of the fused per-token adapter switch on one MI355X.

One step = one lsw_switch over ALL layers of the Llama-2-7B-shaped adapter stack (32 layers x 7
adapted linears, 8 experts of rank 8, top-2): route the token's logits, unmerge the previous top-2,
merge the new top-2, in one launch.  Weights, factors and logits are seeded synthetic data already
resident in HBM when timing starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps 64] [--warmup 3] [--workload 7b] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X datasheet: 8 TB/s HBM3E


def algorithmic_bytes(wl, n_terms: int, factor_bytes: int = 4) -> float:
    """Read + write of every bf16 weight, plus every needed factor element once (fp32 storage: 4 bytes each,
    fp32 B, and A as bf16 high + low parts; bf16 storage: 2 bytes each)."""
    return 4.0 * wl.w_elements() + float(factor_bytes) * n_terms * wl.rank * wl.factor_dims()


def cpu_baseline(wl, steps=3):
    """The oracle as it stands, timed on the host: ONE full layer of the workload (its 7 linears),
    `steps` switches after an untimed first merge, median per switch, scaled by the layer count to a
    whole-stack microseconds-per-token figure.  About 10-30 s of CPU work at the 7B shapes."""
    import numpy as np
    from oracle import lsw_oracle as O
    from paper_2405_17741_amd import inputs as I
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    layer0 = [(o, n) for layer, _, o, n in wl.linear_shapes() if layer == 0]
    rng = np.random.default_rng(wl.seed)
    lin = [I.host_linear(rng, o, n, wl.experts, wl.rank, wl.w_std, wl.a_std, wl.b_std) for o, n in layer0]
    routes = [O.route(l, wl.top_k) for l in I.router_logits(wl, steps + 1)]
    Ws = [O.switch_step(W, A, B, [], [], routes[0][0], routes[0][1]) for W, A, B in lin]
    times = []
    for t in range(steps):
        t0 = time.perf_counter()
        Ws = [O.switch_step(W, A, B, routes[t][0], routes[t][1], routes[t + 1][0], routes[t + 1][1])
              for W, (_, A, B) in zip(Ws, lin)]
        times.append(time.perf_counter() - t0)
    med = sorted(times)[len(times) // 2]
    layer_elems = sum(o * n for o, n in layer0)
    us_per_token = med * 1e6 * wl.w_elements() / layer_elems
    return {
        "value": round(us_per_token, 1), "unit": "us/token", "cores": int(threads), "kind": "oracle",
        "sample": f"NumPy fp64 oracle on one full layer ({len(layer0)} linears, {layer_elems} of {wl.w_elements()} weights), "
                  f"median of {steps} switches ({sum(times):.1f} s of CPU work), scaled by weight count; BLAS threads={threads}, "
                  f"element-wise part single-threaded; host cores visible={len(os.sched_getaffinity(0))}",
    }


MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak


def probe_pitch(torch, L):
    """What an in-place pass sustains on this part as a function of the row pitch of the matrix: the switch kernel's
    access pattern (32 rows x 512 bytes per wave and step) with no factor traffic and no matrix work."""
    stream = torch.cuda.current_stream().cuda_stream
    print("columns  row pitch [B]   GB/s (2 waves/CU)   GB/s (4 waves/CU)")
    for cols in (1024, 2048, 3072, 4096, 5120, 6144, 8192, 11008, 12288, 13824, 16384, 16640, 20480, 24576, 28672, 32768, 49152):
        rows = ((1 << 30) // (2 * cols)) // 128 * 128          # four matrices of 1 GiB (one W must stay below 2 GiB)
        Ws = [torch.zeros(rows, cols, dtype=torch.bfloat16, device="cuda") for _ in range(4)]
        A = torch.zeros(1, 8, cols, dtype=torch.float32, device="cuda")
        B = torch.zeros(1, rows, 8, dtype=torch.float32, device="cuda")
        ctx = L.lsw_create_adapters([(W.data_ptr(), A.data_ptr(), B.data_ptr(), rows, cols, i, 0) for i, W in enumerate(Ws)], 1, 8)
        rates = []
        for wpc in (2, 4):
            L.lsw_probe_inplace(ctx, wpc, stream)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(4):
                L.lsw_probe_inplace(ctx, wpc, stream)
            b.record()
            b.synchronize()
            rates.append(4.0 * 4 * rows * cols / (a.elapsed_time(b) / 4 * 1e-3) / 1e9)
        print(f"{cols:7d}  {2 * cols:13d}   {rates[0]:17.1f}   {rates[1]:17.1f}", flush=True)
        torch.cuda.synchronize()
        L.lsw_destroy(ctx)
        del Ws, A, B


def fast_pitch(n_cols: int) -> int:
    """The next leading dimension (elements) at which rows are 4, 8, 16 or 32 KB apart, or a multiple of 32 KB beyond."""
    for ld in (2048, 4096, 8192, 16384):
        if n_cols <= ld:
            return ld
    return -(-n_cols // 16384) * 16384


def switch_roofline(wl, terms, kernels, launch_bytes, avg_ms, bf16_factors, traffic):
    """HBM roofline of the timed launches, or the matrix-core one where the three-pass product needs longer at the bf16
    matrix peak than the algorithmic bytes need at the HBM peak (fused ranks above 64 with fp32-stored factors)."""
    mean_bytes = sum(launch_bytes) / len(launch_bytes)
    achieved = mean_bytes / (avg_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic}
    mean_terms = sum(terms) / len(terms)
    if max(kernels) == 2 and mean_terms * wl.rank > 64:
        # fused ranks above 64: three bf16 passes (two, or one, with bf16-stored factors) of 2*K flop per weight
        passes = (1.0 if wl.rank % 16 == 0 else 2.0) if bf16_factors else 3.0    # exact bf16 factors of such a rank: one pass
        flops = [passes * 2.0 * n * wl.rank * wl.w_elements() for n, k in zip(terms, kernels) if k != 0]
        mean_flops = sum(flops) / len(flops)
        if mean_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12) > mean_bytes / (HBM_PEAK_GBPS * 1e9):
            tf = mean_flops / (avg_ms * 1e-3) / 1e12
            roofline = {"bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic,
                        "hbm_GBps": round(achieved, 1), "hbm_frac": round(achieved / HBM_PEAK_GBPS, 4)}
    return roofline, achieved


def time_switches(torch, L, I, wl, ctx, steps, warmup, bf16_factors, old=None, stream=0):
    """`warmup` untimed and `steps` timed token steps (route on the host, one lsw_switch over all layers), an event pair
    around every launch.  Returns (stats dict, merged set after the last step, wall seconds of the timed region)."""
    import numpy as np
    logits = I.router_logits(wl, warmup + steps)
    old = (np.zeros(0, np.int32), np.zeros(0, np.float32)) if old is None else old

    def token(t, old):
        new = L.lsw_route(logits[t], wl.top_k)                         # step a1 (host)
        L.lsw_switch(ctx, old[0], old[1], new[0], new[1], stream=stream)   # steps a2-a6 (one launch)
        return new

    for t in range(warmup):
        old = token(t, old)
    torch.cuda.synchronize()
    # accounting pass (host only, outside the timed region): how many terms each timed launch carries
    terms, prev = [], old
    for i in range(steps):
        nxt = L.lsw_route(logits[warmup + i], wl.top_k)
        terms.append(len(L.lsw_build_terms(prev[0], prev[1], nxt[0], nxt[1], wl.experts)[0]))
        prev = nxt
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    kernels, variants = [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        ev[i][0].record()
        old = token(warmup + i, old)
        ev[i][1].record()
        kernels.append(L.lsw_query(ctx, L.LSW_Q_LAST_KERNEL))
        variants.append(L.lsw_query(ctx, L.LSW_Q_LAST_VARIANT))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    fb = 2 if bf16_factors else 4
    launch_ms = [a.elapsed_time(b) for (a, b), k in zip(ev, kernels) if k != 0]
    launch_bytes = [algorithmic_bytes(wl, n, fb) for n, k in zip(terms, kernels) if k != 0]
    avg_ms = sum(launch_ms) / len(launch_ms)
    med_ms = sorted(launch_ms)[len(launch_ms) // 2]
    rates = sorted(b / (ms * 1e-3) / 1e9 for b, ms in zip(launch_bytes, launch_ms))
    mix = {}
    for n, k, v, ms in zip(terms, kernels, variants, [a.elapsed_time(b) for a, b in ev]):
        if k == 0:
            continue
        key = f"{n}_terms"
        m = mix.setdefault(key, {"launches": 0, "us": 0.0, "kernel": VARIANT_NAMES.get(v, str(v))})
        m["launches"] += 1
        m["us"] += ms * 1e3
    for m in mix.values():
        m["us"] = round(m["us"] / m["launches"], 1)
    stats = {"terms": terms, "kernels": kernels, "launch_ms": launch_ms, "launch_bytes": launch_bytes, "avg_ms": avg_ms, "med_ms": med_ms,
             "median_GBps": rates[len(rates) // 2], "mix": mix, "grid": L.lsw_query(ctx, L.LSW_Q_LAST_GRID)}
    return stats, old, wall


VARIANT_NAMES = {0: "vector-ALU", 1: "matrix-core, A streamed per step", 2: "matrix-core, A resident in LDS", 3: "matrix-core, chunked fused rank"}


def other_config(torch, L, I, name, factor_dtype, steps, warmup, traffic_table, pad_pitch=False):
    """One more workload on the same line: stack drawn, switched `steps` times, freed.  Returns its entry."""
    wl = I.WORKLOADS[name]
    bf16_factors = factor_dtype == "bf16"
    w_alloc = sum(o * (fast_pitch(n) if pad_pitch else n) for _, _, o, n in wl.linear_shapes())
    need = 2 * w_alloc + (2 if bf16_factors else 4) * 2 * wl.experts * wl.rank * wl.factor_dims() + (6 << 30)
    free, _ = torch.cuda.mem_get_info()
    if free < need:
        return {"skipped": f"needs {need / 1e9:.0f} GB of free device memory, {free / 1e9:.0f} GB are free"}
    t0 = time.perf_counter()
    stack = I.device_stack(wl, factor_dtype=torch.bfloat16 if bf16_factors else torch.float32, ld_of=fast_pitch if pad_pitch else None)
    ctx = L.create_from_tensors(stack, wl.linear_shapes(), wl.experts, wl.rank)
    stream = torch.cuda.current_stream().cuda_stream
    stats, _, wall = time_switches(torch, L, I, wl, ctx, steps, warmup, bf16_factors, stream=stream)
    torch.cuda.synchronize()
    # the ceiling of the access pattern on these tensors: the matrix-core switch launch with the work taken out
    L.lsw_probe_inplace(ctx, 0, stream)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(3):
        L.lsw_probe_inplace(ctx, 0, stream)
    b.record()
    b.synchronize()
    probe_gbps = 4.0 * wl.w_elements() / (a.elapsed_time(b) / 3 * 1e-3) / 1e9
    L.lsw_destroy(ctx)
    del stack
    torch.cuda.empty_cache()
    key = name + ("_bf16_factors" if bf16_factors else "") + ("_pitch_padded" if pad_pitch else "")
    roofline, achieved = switch_roofline(wl, stats["terms"], stats["kernels"], stats["launch_bytes"], stats["avg_ms"], bf16_factors,
                                         traffic_table.get(key))
    extra = {}
    if roofline["bound"] == "hbm":
        extra["inplace_probe"] = {"switch_pattern_GBps": round(probe_gbps, 1), "switch_over_probe": round(achieved / probe_gbps, 4),
                                  "note": "lsw_probe_inplace(ctx, 0): the streaming matrix-core switch launch (4 terms) on the same weights with "
                                          "operand loads and matrix instructions taken out: 4 bytes per weight, nothing else"}
    if roofline["bound"] == "mfma":
        # what the bare inner loop of this kernel sustains on this part (power-limited clock under matrix load):
        # a wave's 32 x 256 tile needs K / 4 groups of six matrix instructions, the chip runs 1024 waves at once
        ns = L.lsw_probe_matrix_loop(600, 4, 2, False)
        ns0 = L.lsw_probe_matrix_loop(600, 4, 2, True)
        k_max = max(stats["terms"]) * wl.rank
        groups = wl.w_elements() / 8192.0 * (k_max / 4.0) / 1024.0
        extra["matrix_loop"] = {"ns_per_group": round(ns, 1), "ns_per_group_zero_operands": round(ns0, 1),
                                "cycles_per_group": 192, "loop_only_us_at_fused_rank": {str(k_max): round(groups * ns * 1e-3, 1)},
                                "note": "lsw_probe_matrix_loop: the kernel's inner loop alone (4 LDS reads + 6 matrix instructions per group, "
                                        "2 LDS-DMA copies riding along, no weight traffic, no barriers) on all CUs: the time it needs for "
                                        "this launch's matrix work is the practical ceiling under the part's power limit"}
    return {
        **extra,
        "workload": f"{wl.name}: {wl.layers} layers x 7 linears, hidden {wl.hidden}, ffn {wl.ffn}, E={wl.experts}, r={wl.rank}, "
                    f"top-{wl.top_k}, factors stored as {factor_dtype}"
                    + (", every weight stored at a row pitch of 4, 8, 16 or 32 KB (lsw_linear::ld; same algorithmic bytes, "
                       f"{2 * w_alloc / 1e9:.1f} GB allocated for {2 * wl.w_elements() / 1e9:.1f} GB of weights)" if pad_pitch else ""),
        "steps": steps, "warmup": warmup,
        "us": {"mean": round(stats["avg_ms"] * 1e3, 1), "median": round(stats["med_ms"] * 1e3, 1), "min": round(min(stats["launch_ms"]) * 1e3, 1),
               "wall_per_step": round(wall * 1e6 / steps, 1)},
        "algorithmic_bytes_mean": int(sum(stats["launch_bytes"]) / len(stats["launch_bytes"])),
        "terms_per_step_mean": round(sum(stats["terms"]) / len(stats["terms"]), 3),
        "launch_mix": stats["mix"],
        "hbm_GBps": {"from_mean": round(achieved, 1), "median_of_launches": round(stats["median_GBps"], 1)},
        "roofline": roofline,
        "setup_s": round(time.perf_counter() - t0 - wall, 1),
    }


OTHER_CONFIGS = (("7b_r64", "fp32", 32, False), ("7b_r64", "bf16", 32, False), ("13b", "fp32", 32, False), ("70b", "fp32", 16, False),
                 ("7b", "fp32", 32, True), ("13b", "fp32", 32, True))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="7b")
    ap.add_argument("--kernel", type=int, default=0, help="0 auto, 1 vector-ALU, 2 matrix-core")
    ap.add_argument("--cpu-steps", type=int, default=3, help="switches the CPU oracle baseline times")
    ap.add_argument("--grid", type=int, default=0)
    ap.add_argument("--tile-cols", type=int, default=0)
    ap.add_argument("--xcd", type=int, default=-1)
    ap.add_argument("--resident-q", type=int, default=-1, help="0: always stream the A operand per step (tuning knob)")
    ap.add_argument("--panel-group", type=int, default=-1, help="column panels per group in the item order of wide matrices (tuning knob)")
    ap.add_argument("--xcd-pool", type=int, default=-1, help="0: resident-A kernel deals every item statically (tuning knob)")
    ap.add_argument("--factor-dtype", choices=("fp32", "bf16"), default="fp32",
                    help="storage type of the LoRA factors (fp32 is what the workloads prescribe)")
    ap.add_argument("--prefill-tokens", type=int, default=2048, help="prompt length of the adapter-path timing")
    ap.add_argument("--probe-pitch", action="store_true",
                    help="instead of the benchmark: in-place read+write bandwidth (lsw_probe_inplace) of 4 GiB of matrices "
                         "as a function of its row pitch; prints a table")
    ap.add_argument("--switch-only", action="store_true",
                    help="time the switch launches only (profiling runs: every launch of the switch kernel is then a timed one)")
    ap.add_argument("--pad-pitch", action="store_true",
                    help="store every weight whose rows are not 4, 8, 16 or 32 KB apart at the next such leading dimension "
                         "(lsw_linear::ld; the padding columns are never touched): an in-place pass runs fastest at those pitches")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--configs", default="all",
                    help="'all' (default): after the headline workload also time 7b_r64 (fp32- and bf16-stored factors), 13b and 70b "
                         "with fewer steps, one entry each under \"configs\"; 'none': the headline only")
    ap.add_argument("--time-budget", type=float, default=420.0,
                    help="seconds this run may take before the remaining workloads under \"configs\" are written as skipped")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 4 GiB device copy (a known-size reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only: the switch needs no collective (every weight element depends on "
              "its own row of B, its own column of A and the token's ids and gates), so more GPUs would each run this "
              "same launch on their share of the layers. Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    t_start = time.perf_counter()
    import numpy as np
    import torch
    from paper_2405_17741_amd import binding as L
    from paper_2405_17741_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.probe_pitch:
        probe_pitch(torch, L)
        return
    wl = I.WORKLOADS[args.workload]
    bf16_factors = args.factor_dtype == "bf16"
    stack = I.device_stack(wl, factor_dtype=torch.bfloat16 if bf16_factors else torch.float32, ld_of=fast_pitch if args.pad_pitch else None)
    ctx = L.create_from_tensors(stack, wl.linear_shapes(), wl.experts, wl.rank)
    if args.kernel:
        L.lsw_set_option(ctx, L.LSW_OPT_KERNEL, args.kernel)
    if args.grid:
        L.lsw_set_option(ctx, L.LSW_OPT_GRID, args.grid)
    if args.tile_cols:
        L.lsw_set_option(ctx, L.LSW_OPT_TILE_COLS, args.tile_cols)
    if args.xcd >= 0:
        L.lsw_set_option(ctx, L.LSW_OPT_XCD_REMAP, args.xcd)
    if args.resident_q >= 0:
        L.lsw_set_option(ctx, L.LSW_OPT_RESIDENT_Q, args.resident_q)
    if args.xcd_pool >= 0:
        L.lsw_set_option(ctx, L.LSW_OPT_XCD_POOL, args.xcd_pool)
    if args.panel_group >= 0:
        L.lsw_set_option(ctx, L.LSW_OPT_PANEL_GROUP, args.panel_group)
    stream = torch.cuda.current_stream().cuda_stream

    logits = I.router_logits(wl, args.warmup + args.steps)
    stats, old, wall = time_switches(torch, L, I, wl, ctx, args.steps, args.warmup, bf16_factors, stream=stream)
    terms, kernels, launch_ms, launch_bytes, avg_ms = stats["terms"], stats["kernels"], stats["launch_ms"], stats["launch_bytes"], stats["avg_ms"]
    achieved = (sum(launch_bytes) / len(launch_bytes)) / (avg_ms * 1e-3) / 1e9
    ms_per_step = wall * 1e3 / args.steps

    probe, subset, rebase, adapter = {}, None, None, None
    gemv_ms = gemv_gbps = dev_us = float("nan")
    n_dev, dev_flags = 0, 0
    if not args.switch_only:
        # yardstick: the same tensors, the same access pattern, no factor traffic and no matrix work
        for wpc in ((0, 2, 4) if wl.rank % 8 == 0 else (2, 4)):
            L.lsw_probe_inplace(ctx, wpc, stream)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(5):
                L.lsw_probe_inplace(ctx, wpc, stream)
            b.record()
            b.synchronize()
            probe["switch_pattern_GBps" if wpc == 0 else f"{wpc}_waves_per_cu_GBps"] = round(4.0 * wl.w_elements() / (a.elapsed_time(b) / 5 * 1e-3) / 1e9, 1)

        # the decode that follows the switch (timed separately): every merged linear once, batch 1
        nx, ny = L.lsw_query(ctx, L.LSW_Q_GEMV_X_ELEMS), L.lsw_query(ctx, L.LSW_Q_GEMV_Y_ELEMS)
        xg = torch.randn(nx, device="cuda").to(torch.bfloat16)
        yg = torch.empty(ny, device="cuda", dtype=torch.float32)
        L.lsw_merged_gemv_all(ctx, xg.data_ptr(), yg.data_ptr(), stream)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            L.lsw_merged_gemv_all(ctx, xg.data_ptr(), yg.data_ptr(), stream)
        b.record()
        b.synchronize()
        gemv_ms = a.elapsed_time(b) / 5
        gemv_gbps = 2.0 * wl.w_elements() / (gemv_ms * 1e-3) / 1e9
        del xg, yg

        # the same token step with the token's (ids, gates) resident on the device: router, term list and switch are
        # all launched without a value coming back to the host (lsw_route_dev + lsw_switch_dev)
        n_dev = min(args.steps, 32)
        logits_d = torch.from_numpy(logits[:n_dev + 1].copy()).cuda()
        bufs = [(torch.zeros(wl.top_k, dtype=torch.int32, device="cuda"), torch.zeros(wl.top_k, dtype=torch.float32, device="cuda"))
                for _ in range(2)]
        bufs[1][0].copy_(torch.from_numpy(old[0])); bufs[1][1].copy_(torch.from_numpy(old[1]))     # what is merged now

        def dev_token(t):
            new, prv = bufs[t % 2], bufs[(t + 1) % 2]
            L.lsw_route_dev(ctx, logits_d[t].data_ptr(), wl.top_k, new[0].data_ptr(), new[1].data_ptr(), stream)
            L.lsw_switch_dev(ctx, prv[0].data_ptr(), prv[1].data_ptr(), wl.top_k, new[0].data_ptr(), new[1].data_ptr(), wl.top_k, stream=stream)

        dev_token(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(1, n_dev + 1):
            dev_token(t)
        torch.cuda.synchronize()
        dev_us = (time.perf_counter() - t0) * 1e6 / n_dev
        dev_flags = L.lsw_dev_status(ctx)

        # a partial layer set (the `layers` argument): the first half of the layers, there and back
        half = list(range(wl.layers // 2)) or [0]
        other = L.lsw_route(logits[0], wl.top_k)
        sub_bytes = algorithmic_bytes(wl, len(L.lsw_build_terms(old[0], old[1], other[0], other[1], wl.experts)[0]),
                                      2 if bf16_factors else 4) * len(half) / wl.layers
        L.lsw_switch(ctx, old[0], old[1], other[0], other[1], layers=half, stream=stream)
        L.lsw_switch(ctx, other[0], other[1], old[0], old[1], layers=half, stream=stream)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(3):
            L.lsw_switch(ctx, old[0], old[1], other[0], other[1], layers=half, stream=stream)
            L.lsw_switch(ctx, other[0], other[1], old[0], old[1], layers=half, stream=stream)
        b.record()
        b.synchronize()
        sub_us = a.elapsed_time(b) * 1e3 / 6
        subset = {"layers": len(half), "us": round(sub_us, 1), "GBps": round(sub_bytes / (sub_us * 1e-6) / 1e9, 1)}

        # drift control: rebuild every weight from a base copy with the current set merged (reads the copy, writes W)
        rebase = None
        if 2 * 2 * wl.w_elements() < 200e9:
            base = [W.clone() for W, _, _ in stack]
            L.lsw_set_base(ctx, [t.data_ptr() for t in base])
            L.lsw_rebase(ctx, old[0], old[1], stream=stream)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(5):
                L.lsw_rebase(ctx, old[0], old[1], stream=stream)
            b.record()
            b.synchronize()
            rb_us = a.elapsed_time(b) * 1e3 / 5
            rebase = {"us": round(rb_us, 1), "GBps": round(algorithmic_bytes(wl, len(old[0]), 2 if bf16_factors else 4) / (rb_us * 1e-6) / 1e9, 1),
                      "note": "lsw_rebase: W <- rne(W_base + current set), base copy read, W written, one launch"}
            torch.cuda.synchronize()
            del base

        # the un-merged adapter path a prompt takes (Eq. 2): 2048 tokens through the 7 linears of one layer
        adapter = None
        if wl.rank % 8 == 0 and wl.experts * wl.rank <= 256:
            T = args.prefill_tokens
            L.lsw_enable_adapter_path(ctx)
            lg = torch.randn(T, wl.experts, device="cuda")
            idd = torch.zeros(T, wl.top_k, dtype=torch.int32, device="cuda")
            gd = torch.zeros(T, wl.top_k, dtype=torch.float32, device="cuda")
            L.lsw_route_batch_dev(ctx, lg.data_ptr(), T, wl.top_k, idd.data_ptr(), gd.data_ptr(), stream)
            layer0 = [(p, o, n) for p, (layer, _, o, n) in enumerate(wl.linear_shapes()) if layer == 0]
            kinds0 = [kind for layer, kind, _, _ in wl.linear_shapes() if layer == 0]
            # as in a decoder layer: q, k, v read one activation tensor, o another, gate and up a third, down a fourth
            group_of = {0: "attn_in", 1: "attn_in", 2: "attn_in", 3: "o_in", 4: "ffn_in", 5: "ffn_in", 6: "down_in"}

            def activations(tokens):
                made = {}
                return [made.setdefault((group_of[kind], n), torch.randn(tokens, n, device="cuda").to(torch.bfloat16))
                        for kind, (_, _, n) in zip(kinds0, layer0)]
            xs = activations(T)
            ys = [torch.randn(T, o, device="cuda").to(torch.bfloat16) for _, o, _ in layer0]      # one output per linear
            ws = torch.empty(L.lsw_adapter_layer_workspace_bytes(ctx, 0, T) // 4, dtype=torch.float32, device="cuda")
            fb = 2 if bf16_factors else 4

            def prefill_layer():          # all linears of the layer: three launches in all
                L.lsw_adapter_forward_layer(ctx, 0, [x.data_ptr() for x in xs], T, idd.data_ptr(), gd.data_ptr(), wl.top_k,
                                            [y.data_ptr() for y in ys], ws.data_ptr(), stream)

            def prefill_per_linear():     # the same work as seven separate calls (three launches each)
                for i, (p, o, n) in enumerate(layer0):
                    L.lsw_adapter_forward(ctx, p, xs[i].data_ptr(), T, idd.data_ptr(), gd.data_ptr(), wl.top_k, ys[i].data_ptr(),
                                          ws.data_ptr(), stream)

            def timed(fn, reps=10):
                fn()
                torch.cuda.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(reps):
                    fn()
                b.record()
                b.synchronize()
                return a.elapsed_time(b) * 1e3 / reps

            ad_us, ad_us_lin = timed(prefill_layer), timed(prefill_per_linear)
            ad_bytes = sum(T * n * 2 + 2 * T * o * 2 + fb * wl.experts * wl.rank * (n + o) for _, o, n in layer0)
            adapter = {"tokens": T, "linears": len(layer0), "us_per_layer": round(ad_us, 1), "GBps": round(ad_bytes / (ad_us * 1e-6) / 1e9, 1),
                       "frac_of_hbm_peak": round(ad_bytes / (ad_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                       "us_per_layer_one_call_per_linear": round(ad_us_lin, 1), "error_flags": L.lsw_dev_status(ctx),
                       "note": "lsw_adapter_forward_layer over the linears of one layer (three launches in all): per linear X read, Y "
                               "read and written (bf16), every factor once; beside it the same work as one lsw_adapter_forward per linear"}
            if T != 8192 and not args.switch_only:      # the same at a longer prompt
                T8 = 8192
                lg8 = torch.randn(T8, wl.experts, device="cuda")
                id8 = torch.zeros(T8, wl.top_k, dtype=torch.int32, device="cuda")
                g8 = torch.zeros(T8, wl.top_k, dtype=torch.float32, device="cuda")
                L.lsw_route_batch_dev(ctx, lg8.data_ptr(), T8, wl.top_k, id8.data_ptr(), g8.data_ptr(), stream)
                xs8 = activations(T8)
                ys8 = [torch.randn(T8, o, device="cuda").to(torch.bfloat16) for _, o, _ in layer0]
                ws8 = torch.empty(L.lsw_adapter_layer_workspace_bytes(ctx, 0, T8) // 4, dtype=torch.float32, device="cuda")
                us8 = timed(lambda: L.lsw_adapter_forward_layer(ctx, 0, [x.data_ptr() for x in xs8], T8, id8.data_ptr(), g8.data_ptr(),
                                                                wl.top_k, [y.data_ptr() for y in ys8], ws8.data_ptr(), stream), 5)
                b8 = sum(T8 * n * 2 + 2 * T8 * o * 2 + fb * wl.experts * wl.rank * (n + o) for _, o, n in layer0)
                adapter["tokens_8192"] = {"us_per_layer": round(us8, 1), "GBps": round(b8 / (us8 * 1e-6) / 1e9, 1),
                                          "frac_of_hbm_peak": round(b8 / (us8 * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}
                del xs8, ys8, ws8
            del xs, ys, ws

    traffic_table = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic_table = json.load(open(tpath))
        except Exception:
            traffic_table = {}
    roofline, _ = switch_roofline(wl, terms, kernels, launch_bytes, avg_ms, bf16_factors,
                                  traffic_table.get(args.workload + ("_bf16_factors" if bf16_factors else "")))
    roofline["achieved_from_median"] = round(stats["median_GBps"], 1)
    mean_terms = sum(terms) / len(terms)

    out = {
        "metric": "switch latency us/token (all layers) + achieved HBM GB/s, 7B-shaped adapters",
        "value": round(ms_per_step * 1e3, 1), "unit": "us/token",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.layers} layers x 7 linears, hidden {wl.hidden}, ffn {wl.ffn}, "
                               f"E={wl.experts}, r={wl.rank}, top-{wl.top_k}, all layers per launch, factors stored as {args.factor_dtype}"
                               + (", weights stored at 4/8/16/32 KB row pitch" if args.pad_pitch else ""),
                   "w_elements": wl.w_elements(),
                   "kernel": {0: "none", 1: "vector-ALU", 2: "matrix-core"}[max(kernels)],
                   "fused_rank_mean": round(mean_terms * wl.rank, 1),
                   "grid": L.lsw_query(ctx, L.LSW_Q_LAST_GRID),
                   "terms_per_step_mean": round(sum(terms) / len(terms), 3),
                   "launch_us": {"mean": round(avg_ms * 1e3, 1), "min": round(min(launch_ms) * 1e3, 1),
                                 "median": round(sorted(launch_ms)[len(launch_ms) // 2] * 1e3, 1)},
                   "launch_mix": stats["mix"]},
        "achieved_hbm_GBps": round(achieved, 1),
        "roofline": roofline,
    }
    if not args.switch_only:
        out.update({
            "merged_gemv": {"us": round(gemv_ms * 1e3, 1), "GBps": round(gemv_gbps, 1), "frac_of_hbm_peak": round(gemv_gbps / HBM_PEAK_GBPS, 4),
                            "note": "lsw_merged_gemv_all: batch-1 bf16 decode through every merged linear in one launch, "
                                    "2 bytes per weight, timed separately from the switch"},
            "device_routing": {"us_per_token": round(dev_us, 1), "tokens": n_dev, "error_flags": dev_flags,
                               "note": "lsw_route_dev + lsw_switch_dev per token, lists resident on the device, no host round trip; "
                                       "launches sized for k_old + k_new terms"},
            "adapter_prefill": adapter,
            "layer_subset": subset,
            "rebase": rebase,
            "inplace_probe": {**probe, "note": "lsw_probe_inplace on the same weights: in-place bf16 read+write only, no factor traffic, no "
                                               "matrix work; switch_pattern = the switch kernel's own launch (4-wave workgroups, its item "
                                               "order and pool, its per-step schedule) with the work taken out; N_waves_per_cu = single-wave "
                                               "workgroups walking 32-row items",
                              "switch_over_best_probe": round(achieved / max(probe.values()), 4)},
        })
    torch.cuda.synchronize()
    L.lsw_destroy(ctx)
    del stack
    torch.cuda.empty_cache()
    if args.configs == "all" and not args.switch_only and args.workload == "7b" and not bf16_factors:
        # the other workload shapes, fewer steps each; the CPU baseline (about 15 s) still has to fit behind them
        out["configs"] = {}
        for name, fdt, steps, pad in OTHER_CONFIGS:
            key = name + ("_bf16_factors" if fdt == "bf16" else "") + ("_pitch_padded" if pad else "")
            spent = time.perf_counter() - t_start
            if spent > args.time_budget - (150.0 if name == "70b" else 40.0):
                out["configs"][key] = {"skipped": f"time budget: {spent:.0f} s of {args.time_budget:.0f} s spent before this workload"}
                continue
            try:
                out["configs"][key] = other_config(torch, L, I, name, fdt, steps, 2, traffic_table, pad)
            except torch.cuda.OutOfMemoryError as e:
                out["configs"][key] = {"skipped": f"out of device memory: {str(e)[:120]}"}
                torch.cuda.empty_cache()
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                      # reads 4 GiB, writes 4 GiB
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = int(src.numel() * 4)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_steps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
