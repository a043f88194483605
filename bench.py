#!/usr/bin/env python3
"""Benchmark of the STEM FFN hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic tokens, all inputs already
in HBM: stem_ffn_forward (gate GEMM with fused SiLU*gather, down GEMM), stem_ffn_backward
(four GEMMs, fused dU/dG), stem_embed_grad (sort, unique, segmented sum) and
stem_embed_sparse_adamw on the touched rows.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3|C2|C1]

Two more workloads measure the forward-only configurations (not the headline metric):
--workload C4 times a decode step of 256 single tokens through 16 stacked layers, --workload C5
[--ids zipf|uniform] the 65536-token forward with the table in pinned host memory.
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

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--ids", default="zipf", choices=["zipf", "uniform"], help="id distribution for C5")
    ap.add_argument("--cache-slots", type=int, default=0,
                    help="C5: device-resident LFU cache of this many rows (0 = none); ten batches warm it first")
    ap.add_argument("--prefetch-mode", default="kernel", choices=["kernel", "memcpy"],
                    help="C5: how the distinct rows cross the host link (copy kernel reading pinned memory, or packed hipMemcpyAsync)")
    ap.add_argument("--graph", action="store_true", help="C4: capture the 16-layer step in a HIP graph and replay it")
    ap.add_argument("--host-state", action="store_true",
                    help="C2/C3: training step with the table, its fp32 master and the AdamW moments in pinned host "
                         "memory (rows prefetched, optimiser straight on the host-resident state)")
    ap.add_argument("--variant", default="stem", choices=["stem", "dense", "additive"],
                    help="stem: the STEM layer (the headline); dense: SwiGLU FFN with an up projection and no table; "
                         "additive: up projection plus table (C2, C3 only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the short runs of the other configurations (C2, C4, C5) reported under 'secondary'")
    ap.add_argument("--no-overlap-sort", action="store_true",
                    help="run the integer half of the table gradient in line instead of on a second stream under the backward products")
    ap.add_argument("--cpu-sample-tokens", type=int, default=16384)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy (reference point for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch

    from paper_2601_10639_amd import inputs, stemlib as L

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    L.lib()  # fails loudly if libstem.so has not been built
    dev = "cuda:0"
    shape = inputs.SHAPES[args.workload]
    if args.workload == "C4":
        print(json.dumps(bench_decode(args, shape, dev)))
        return 0
    if args.workload == "C5":
        print(json.dumps(bench_host_table(args, shape, dev, [args.ids])[args.ids]))
        return 0
    if args.host_state:
        return bench_host_training(args, shape, dev)
    peaks = measure_peaks(dev)
    out, inp = bench_layer(args, shape, dev, args.steps, args.warmup, peaks, detail=True)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    if args.variant == "stem" and args.workload == "C3" and not args.no_secondary:
        del inp["E"]
        torch.cuda.empty_cache()
        out["secondary"] = secondary_runs(args, dev, peaks)
        inp = None
    if not args.no_cpu_baseline and args.variant == "stem":
        if inp is None:   # same seed: the same batch again
            inp = inputs.layer_inputs(shape, seed=3, device=dev)
        out["cpu_baseline"] = cpu_baseline(shape, inp, args.cpu_sample_tokens, hp)
    print(json.dumps(out))
    return 0


def measure_peaks(dev):
    """What this machine sustains: an MFMA-only loop, a streaming read and a streaming copy of 1 GiB
    (kernels in csrc/calibrate.hip).  The roofline fractions keep the published peaks as denominators;
    `frac_of_measured` next to them uses these."""
    import torch

    from paper_2601_10639_amd import stemlib as L
    a = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    b = torch.empty_like(a)
    g = torch.Generator(device=dev).manual_seed(7)
    normal = torch.randn(1 << 16, device=dev, generator=g).to(torch.bfloat16)   # operands like the layer's own
    sink = torch.zeros(64, device=dev)
    peaks = {
        "mfma_bf16_tflops": round(L.stem_measure_peak(L.STEM_PEAK_MFMA_BF16, a, None, repeats=3), 1),
        "mfma_bf16_unit_normal_data_tflops": round(L.stem_measure_peak(L.STEM_PEAK_MFMA_BF16_DATA, normal, sink, repeats=3), 1),
        "hbm_read_gbs": round(L.stem_measure_peak(L.STEM_PEAK_HBM_READ, a, b, repeats=5), 1),
        "hbm_copy_gbs": round(L.stem_measure_peak(L.STEM_PEAK_HBM_COPY, a, b, repeats=5), 1),
        "how": "stem_measure_peak: loop of independent 32x32x16 bf16 MFMAs on registers with near-constant operands (7 ms), "
               "the same MFMA count on unit-normal operands (the chip is power-limited: the more operand bits toggle, "
               "the lower the clock it sustains); 1 GiB streaming read; 1 GiB streaming copy, bytes read + written; "
               "best of 3 / 3 / 5 / 5 runs between HIP events",
    }
    del a, b, normal, sink
    torch.cuda.empty_cache()
    return peaks


def _dist(ms_list):
    import numpy as np
    ts = np.sort(np.asarray(ms_list, dtype=np.float64))
    return {"median": round(float(np.median(ts)), 4), "p10": round(float(ts[int(0.1 * (len(ts) - 1))]), 4),
            "p90": round(float(ts[int(round(0.9 * (len(ts) - 1)))]), 4), "n": int(len(ts))}


def _event_times(fn, n, warmup):
    """Per-call device time in ms between HIP events recorded on torch's current stream (the stream
    the library launches on) right before and right after each call; calls run back to back."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for e0, e1 in evs:
        e0.record()
        fn()
        e1.record()
    torch.cuda.synchronize()
    return [e0.elapsed_time(e1) for e0, e1 in evs]


def bench_layer(args, shape, dev, steps, warmup, peaks, detail):
    """One layer's training step (forward, backward, table gradient, sparse AdamW) at `shape`.
    Returns (the JSON object, the inputs)."""
    import torch

    from paper_2601_10639_amd import inputs, stemlib as L

    T, d, F, V = shape.tokens, shape.d_model, shape.d_ff, shape.vocab
    bf16 = shape.dtype == "bf16"
    dt = inputs.torch_dtype(shape.dtype)

    inp = inputs.layer_inputs(shape, seed=3, device=dev)
    ctx = L.stem_create(d, F, V, L.STEM_BF16 if bf16 else L.STEM_F32, T, 0,
                        reserve=L.STEM_RESERVE_UP if args.variant != "stem" else 0)
    E = inp["E"]
    master = E.float() if bf16 else None
    m = torch.zeros(V, F, dtype=torch.float32, device=dev)
    v = torch.zeros(V, F, dtype=torch.float32, device=dev)
    y = torch.empty(T, d, dtype=dt, device=dev)
    G = torch.empty(T, F, dtype=dt, device=dev)
    H = torch.empty(T, F, dtype=dt, device=dev)
    dx = torch.empty(T, d, dtype=dt, device=dev)
    dU = torch.empty(T, F, dtype=dt, device=dev)
    dWg = torch.empty(F, d, dtype=torch.float32, device=dev)
    dWd = torch.empty(d, F, dtype=torch.float32, device=dev)
    cap = min(T, V)
    i32 = torch.int32
    sorted_ids = torch.empty(T, dtype=i32, device=dev)
    perm = torch.empty(T, dtype=i32, device=dev)
    uniq_ids = torch.empty(cap, dtype=i32, device=dev)
    seg_offsets = torch.empty(cap + 1, dtype=i32, device=dev)
    n_uniq = torch.zeros(1, dtype=i32, device=dev)
    dE_rows = torch.empty(cap, F, dtype=torch.float32, device=dev)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    step_no = [0]

    variant = args.variant
    if variant != "stem":
        if not bf16:
            raise SystemExit("bench.py: --variant dense/additive needs a bf16 workload (C2, C3)")
        W_up = inputs.normal((F, d), 0.02, 3004, dt, dev)
        Up = torch.empty(T, F, dtype=dt, device=dev)
        dWu = torch.empty(F, d, dtype=torch.float32, device=dev)
    # The integer half of the table gradient (sort, distinct ids, offsets) needs the token ids only:
    # it is enqueued on a second stream after the forward call and joins the main stream before the
    # row sums, so its one workgroup runs in the gaps of the backward products.
    overlap_sort = variant == "stem" and not args.no_overlap_sort
    main_stream = torch.cuda.current_stream()
    side = torch.cuda.Stream() if overlap_sort else None

    def fwd_bwd():
        if variant == "stem":
            L.stem_ffn_forward(ctx, inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], E, y, G, H)
            L.stem_ffn_backward(ctx, inp["dy"], inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], E, G, H, dx, dWg,
                                dWd, dU)
        else:
            tab, tid = (E, inp["ids"]) if variant == "additive" else (None, None)
            L.stem_ffn_up_forward(ctx, inp["x"], tid, inp["W_gate"], W_up, inp["W_down"], tab, y, G, Up, H)
            L.stem_ffn_up_backward(ctx, inp["dy"], inp["x"], tid, inp["W_gate"], W_up, inp["W_down"], tab, G, Up, H,
                                   dx, dWg, dWu, dWd, dU)

    def step():
        step_no[0] += 1
        if overlap_sort:
            L.stem_ffn_forward(ctx, inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], E, y, G, H)
            side.wait_stream(main_stream)      # after the previous step's optimiser, which reads uniq_ids / n_uniq
            L.stem_embed_grad(ctx, inp["ids"], None, sorted_ids, perm, uniq_ids, seg_offsets, n_uniq, None, stream=side)
            L.stem_ffn_backward(ctx, inp["dy"], inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], E, G, H, dx, dWg,
                                dWd, dU)
            main_stream.wait_stream(side)
            L.stem_embed_grad_presorted(ctx, dU, perm, seg_offsets, dE_rows)
            L.stem_embed_sparse_adamw(ctx, uniq_ids, n_uniq, dE_rows, E, master, m, v, step=step_no[0], **hp)
            return
        fwd_bwd()
        if variant != "dense":
            L.stem_embed_grad(ctx, inp["ids"], dU, sorted_ids, perm, uniq_ids, seg_offsets, n_uniq, dE_rows)
            L.stem_embed_sparse_adamw(ctx, uniq_ids, n_uniq, dE_rows, E, master, m, v, step=step_no[0], **hp)

    if args.calibrate_copy and detail:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # the contract's figure: W untimed steps, then exactly K steps between two synchronisations
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    L.stem_sync_status(ctx)
    ms_per_step = elapsed / steps * 1e3
    tokens_per_s = T * steps / elapsed
    U = int(n_uniq.item()) if variant != "dense" else 0

    # the same step, and forward + backward alone, timed call by call between HIP events: at least 50 calls
    n_dist = max(50, steps)
    step_dist = _dist(_event_times(step, n_dist, 3))
    fb_dist = _dist(_event_times(fwd_bwd, n_dist, 3))

    # Per-kernel durations: the same K steps again with HIP events around every launch, on the
    # stream the kernels run on.
    L.stem_profile_enable(ctx, True)
    L.stem_profile_reset(ctx)
    for _ in range(steps):
        step()
    prof = L.stem_profile_read(ctx)
    # the stand-alone SiLU * gather kernel at this shape (what backward runs when H was not saved)
    if variant == "stem":
        for _ in range(2):   # the context's own H buffer is touched for the first time here
            L.stem_ffn_backward(ctx, inp["dy"], inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], E, G, None, dx, dWg,
                                dWd, dU)
        L.stem_profile_read(ctx)
        L.stem_profile_reset(ctx)
        for _ in range(10):
            L.stem_ffn_backward(ctx, inp["dy"], inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], E, G, None, dx, dWg,
                                dWd, dU)
        prof["silu_gather"] = L.stem_profile_read(ctx)["silu_gather"]
    L.stem_profile_enable(ctx, False)
    L.stem_sync_status(ctx)

    gemm_flop = 2.0 * T * d * F
    peak_tf = PEAK_BF16_TFLOPS if bf16 else PEAK_FP32_TFLOPS
    es = 2 if bf16 else 4
    algo_bytes = {
        "sparse_adamw": U * F * (30 if bf16 else 28),
        "silu_gather": 2 * T * F * es + U * F * es,
    }
    kernels = {}
    for name, (ms, n) in prof.items():
        avg = ms / n
        k = {"avg_ms": round(avg, 5), "launches": n}
        if name.startswith("gemm_"):
            fl = gemm_flop * (2 if (name == "gemm_dx" and variant != "stem") else 1)   # dx spans both projections
            k["tflops"] = round(fl / (avg * 1e-3) / 1e12, 2)
            k["frac_mfma_peak"] = round(k["tflops"] / peak_tf, 4)
            if bf16:
                k["frac_of_measured"] = round(k["tflops"] / peaks["mfma_bf16_tflops"], 4)
                k["frac_of_measured_on_data"] = round(k["tflops"] / peaks["mfma_bf16_unit_normal_data_tflops"], 4)
        elif name in algo_bytes:
            k["algorithmic_bytes"] = algo_bytes[name]
            k["gbs"] = round(algo_bytes[name] / (avg * 1e-3) / 1e9, 1)
            k["frac_hbm_peak"] = round(k["gbs"] / PEAK_HBM_GBS, 4)
            k["frac_of_measured_copy"] = round(k["gbs"] / peaks["hbm_copy_gbs"], 4)
        if name == "sort_fused" and overlap_sort:
            k["note"] = "one workgroup on a second stream under the backward GEMMs: wall time while it waits for a compute unit; 39 us when it runs alone"
        kernels[name] = k
    # the segmented sum (G3) is everything it launches: the chunk sums and the sums over border-crossing runs
    if "seg_reduce" in kernels:
        g3_ms = kernels["seg_reduce"]["avg_ms"] + kernels.get("seg_combine", {"avg_ms": 0.0})["avg_ms"]
        g3_bytes = T * F * es + U * F * 4
        kernels["table_grad_G3"] = {
            "avg_ms": round(g3_ms, 5), "is": "seg_reduce + seg_combine", "algorithmic_bytes": g3_bytes,
            "gbs": round(g3_bytes / (g3_ms * 1e-3) / 1e9, 1),
            "frac_hbm_peak": round(g3_bytes / (g3_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "frac_of_measured_copy": round(g3_bytes / (g3_ms * 1e-3) / 1e9 / peaks["hbm_copy_gbs"], 4)}
    # measured HBM-side bytes per launch (rocprofv3 FETCH_SIZE / WRITE_SIZE) and MFMA-busy fraction / sustained
    # shader clock per kernel: read from the summaries committed under profiles/ (another run of this command on a
    # box of the same pool, not this run)
    traffic, counters = {}, {}
    tname = "hbm_traffic_%s.json" % shape.name.replace("-", "_")
    cname = "mfma_util_%s.json" % shape.name.replace("-", "_")
    if os.path.exists(os.path.join(ROOT, "profiles", tname)):
        with open(os.path.join(ROOT, "profiles", tname)) as fh:
            traffic = {k: v for k, v in json.load(fh).items() if not k.startswith("_")}
    if os.path.exists(os.path.join(ROOT, "profiles", cname)) and variant == "stem":
        with open(os.path.join(ROOT, "profiles", cname)) as fh:
            counters = {k: v for k, v in json.load(fh).items() if not k.startswith("_")}
    gemms = {k: v for k, v in kernels.items() if k.startswith("gemm_")}
    dom = max(gemms, key=lambda k: gemms[k]["avg_ms"] * gemms[k]["launches"])
    all_gemm_ms = sum(v["avg_ms"] for v in gemms.values())
    n_gemm_units = 6 if variant == "stem" else 9   # products of 2*T*d*F FLOP each per step
    all_tf = n_gemm_units * gemm_flop / (all_gemm_ms * 1e-3) / 1e12
    roofline = {
        "bound": "mfma" if bf16 else "alu",
        "kernel": dom,
        "achieved": gemms[dom]["tflops"],
        "peak": peak_tf,
        "unit": "TFLOP/s",
        "frac": round(gemms[dom]["tflops"] / peak_tf, 4),
        "frac_of_measured": round(gemms[dom]["tflops"] / peaks["mfma_bf16_tflops"], 4) if bf16 else None,
        "frac_of_measured_on_data": round(gemms[dom]["tflops"] / peaks["mfma_bf16_unit_normal_data_tflops"], 4) if bf16 else None,
        "traffic": traffic.get(dom),
        "counters": counters.get(dom),
        "traffic_and_counters_source": "profiles/%s, profiles/%s (committed rocprofv3 summaries of this command)" % (tname, cname),
        "all_gemms_tflops": round(all_tf, 2),
        "all_gemms_frac": round(all_tf / peak_tf, 4),
        "all_gemms_frac_of_measured": round(all_tf / peaks["mfma_bf16_tflops"], 4) if bf16 else None,
        "all_gemms_frac_of_measured_on_data": round(all_tf / peaks["mfma_bf16_unit_normal_data_tflops"], 4) if bf16 else None,
    }

    out = {
        "metric": "STEM FFN fwd+bwd tokens/s per layer" if variant == "stem" else
                  ("dense SwiGLU FFN" if variant == "dense" else "additive-variant FFN") + " fwd+bwd tokens/s per layer",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": shape.dtype,
        "data": "synthetic",
        "config": {"workload": shape.name, "d_model": d, "d_ff": F, "vocab": V, "tokens": T,
                   "n_uniq": U, "ids": "Zipf(s=1.1)", "variant": variant,
                   "step": "fwd+bwd" if variant == "dense" else "fwd+bwd+embed_grad+sparse_adamw",
                   "sort_on_second_stream": bool(overlap_sort)},
        # `value` is the whole step; the metric's own words (forward + backward) are here, both from HIP events
        "step_ms": step_dist,
        "fwd_bwd_ms": fb_dist,
        "fwd_bwd_tokens_per_s": round(T / (fb_dist["median"] * 1e-3), 1),
        "step_tokens_per_s_median": round(T / (step_dist["median"] * 1e-3), 1),
        "measured_peak": peaks,
        "roofline": roofline,
        "kernels": kernels,
    }
    ctx.close()
    return out, inp


def secondary_runs(args, dev, peaks):
    """Short runs of the other configurations, so that their figures come from the same command."""
    import copy

    import torch

    from paper_2601_10639_amd import inputs
    sec = {}
    a = copy.copy(args)
    a.variant, a.graph, a.cache_slots, a.calibrate_copy = "stem", False, 0, False
    c2, _ = bench_layer(a, inputs.SHAPES["C2"], dev, 20, 5, peaks, detail=False)
    sec["C2"] = {"workload": c2["config"]["workload"], "ms_per_step": c2["ms_per_step"], "tokens_per_s": c2["value"],
                 "step_ms": c2["step_ms"], "fwd_bwd_ms": c2["fwd_bwd_ms"],
                 "all_gemms_frac": c2["roofline"]["all_gemms_frac"],
                 "table_grad_G3_frac_hbm": c2["kernels"].get("table_grad_G3", {}).get("frac_hbm_peak"),
                 "sparse_adamw_frac_hbm": c2["kernels"].get("sparse_adamw", {}).get("frac_hbm_peak")}
    del c2
    torch.cuda.empty_cache()
    a.steps, a.warmup = 50, 10
    c4 = bench_decode(a, inputs.SHAPES["C4"], dev)
    sec["C4"] = {"workload": c4["config"]["workload"], "us_per_step": c4["value"], "latency_ms": c4["latency_ms"],
                 "frac_hbm_peak": c4["roofline"]["frac"], "layers": 16}
    del c4
    torch.cuda.empty_cache()
    a.steps, a.warmup = 10, 3
    c5 = bench_host_table(a, inputs.SHAPES["C5"], dev, ["zipf", "uniform"])
    for kind, r in c5.items():
        sec["C5_" + kind] = {"workload": r["config"]["workload"], "ms_per_step": r["ms_per_step"], "tokens_per_s": r["value"],
                             "n_uniq": r["config"]["n_uniq"], "latency_ms": r["latency_ms"],
                             "host_link_gbs": r["roofline"]["achieved"], "host_link_frac_of_contiguous_copy": r["roofline"]["frac"]}
    torch.cuda.empty_cache()
    return sec


def _median_ms(fn, steps, warmup):
    """Wall-clock per call (device idle before and after each), median / p10 / p90 in ms."""
    import numpy as np
    import torch
    for _ in range(warmup):
        fn()
    ts = []
    for _ in range(steps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        ts.append((time.perf_counter() - t0) * 1e3)
    ts = np.sort(np.asarray(ts))
    return float(np.median(ts)), float(ts[int(0.1 * (len(ts) - 1))]), float(ts[int(round(0.9 * (len(ts) - 1)))])


def bench_decode(args, shape, dev):
    """One decode step: T single tokens through n_layers stacked layers (each with its own weights
    and table), residual stream in bf16.  Each layer is one stem_ffn_forward_residual call, in place
    on the stream.  HBM-bound on the weights: 2*d*F*2 bytes per layer."""
    import torch

    from paper_2601_10639_amd import inputs, stemlib as L

    T, d, F, V = shape.tokens, shape.d_model, shape.d_ff, shape.vocab
    n_layers = 16
    ids_np = inputs.zipf_ids(T, V, seed=31)
    ids = torch.from_numpy(ids_np).to(dev)
    U = len(set(ids_np.tolist()))
    ctx = L.stem_create(d, F, V, L.STEM_BF16, T, 0)
    Wg = [inputs.normal((F, d), 0.02, 100 + 3 * l, torch.bfloat16, dev) for l in range(n_layers)]
    Wd = [inputs.normal((d, F), 0.02, 101 + 3 * l, torch.bfloat16, dev) for l in range(n_layers)]
    E = [inputs.normal((V, F), 0.02, 102 + 3 * l, torch.bfloat16, dev) for l in range(n_layers)]
    x0 = inputs.normal((T, d), 1.0, 32, torch.bfloat16, dev)
    x = x0.clone()
    y = torch.empty_like(x0)

    def step():
        x.copy_(x0)
        for l in range(n_layers):   # x <- x + layer_l(x): the add is part of the down product's epilogue
            L.stem_ffn_forward_residual(ctx, x, ids, Wg[l], Wd[l], E[l], x, x)

    eager_step = step
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            eager_step()
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                eager_step()
        torch.cuda.synchronize()
        step = graph.replay
    steps = max(args.steps, 50)
    med, p10, p90 = _median_ms(step, steps, max(args.warmup, 10))
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    L.stem_sync_status(ctx)
    L.stem_profile_enable(ctx, True)
    L.stem_profile_reset(ctx)
    for _ in range(10):
        eager_step()
    prof = L.stem_profile_read(ctx)
    L.stem_profile_enable(ctx, False)
    kernels = {k: {"avg_ms": round(v[0] / v[1], 5), "launches": v[1]} for k, v in prof.items()}
    kern_ms = sum(v[0] for v in prof.values()) / 10
    weight_bytes = n_layers * 2 * d * F * 2
    row_bytes = n_layers * U * F * 2
    act_bytes = n_layers * (2 * T * d * 2 + 2 * T * F * 2)
    algo = weight_bytes + row_bytes + act_bytes
    out = {
        "metric": "STEM FFN decode step latency, 16 stacked layers", "value": round(ms * 1e3, 1), "unit": "us",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": shape.name, "d_model": d, "d_ff": F, "vocab": V, "tokens": T, "layers": n_layers,
                   "n_uniq": U, "ids": "Zipf(s=1.1)", "step": "16 x forward with the residual add fused (stem_ffn_forward_residual)", "hip_graph": bool(args.graph)},
        "latency_ms": {"median": round(med, 4), "p10": round(p10, 4), "p90": round(p90, 4),
                       "back_to_back": round(ms, 4), "kernels_only": round(kern_ms, 4)},
        "roofline": {"bound": "hbm", "kernel": "decode step (all kernels)",
                     "achieved": round(algo / (kern_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(algo / (kern_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4), "traffic": None,
                     "bytes": {"weights": weight_bytes, "table_rows": row_bytes, "activations": act_bytes}},
        "kernels": kernels,
    }
    ctx.close()
    return out


def bench_host_table(args, shape, dev, id_kinds):
    """Forward of one layer over a long sequence with the table in pinned host memory: de-duplicate
    the ids, copy the distinct rows over the host link on a side stream while the gate GEMM runs,
    then the gather epilogue and the down GEMM.  Also times the same forward with a device-resident
    table (what the copy exposes) and a plain pinned host-to-device copy (the link's rate).
    One result per entry of id_kinds ("zipf", "uniform"), all on the same table and weights."""
    import torch

    from paper_2601_10639_amd import inputs

    T, d, F, V = shape.tokens, shape.d_model, shape.d_ff, shape.vocab
    # drawn on the device and copied out: the host generator needs ten seconds for a billion draws
    E_host = inputs.normal((V, F), 0.02, 53, torch.bfloat16, dev).cpu().pin_memory()
    shared = {
        "E_host": E_host,
        "x": inputs.normal((T, d), 1.0, 54, torch.bfloat16, dev),
        "Wg": inputs.normal((F, d), 0.02, 55, torch.bfloat16, dev),
        "Wd": inputs.normal((d, F), 0.02, 56, torch.bfloat16, dev),
        "E_dev": E_host.to(dev),
    }
    return {kind: _host_table_one(args, shape, dev, kind, shared) for kind in id_kinds}


def _host_table_one(args, shape, dev, ids_kind, shared):
    import torch

    from paper_2601_10639_amd import inputs, stemlib as L

    T, d, F, V = shape.tokens, shape.d_model, shape.d_ff, shape.vocab
    ids_np = inputs.zipf_ids(T, V, seed=51) if ids_kind == "zipf" else inputs.uniform_ids(T, V, seed=52)
    ids_host = torch.from_numpy(ids_np)
    U = len(set(ids_np.tolist()))
    ctx = L.stem_create(d, F, V, L.STEM_BF16, T, 0)
    if getattr(args, "prefetch_mode", "kernel") == "memcpy":
        L.stem_set_prefetch_mode(ctx, L.STEM_PREFETCH_MEMCPY)
    E_host, x, Wg, Wd, E_dev = (shared[k] for k in ("E_host", "x", "Wg", "Wd", "E_dev"))
    y = torch.empty(T, d, dtype=torch.bfloat16, device=dev)
    E_compact = torch.empty(U + 8, F, dtype=torch.bfloat16, device=dev)
    remap = torch.empty(T, dtype=torch.int32, device=dev)
    ids_dev = ids_host.to(dev)
    dedup_ms = []
    NS = args.cache_slots
    miss_rows, uniq_rows = [U], [U]
    if NS > 0:
        # one token stream: batches share the vocabulary (which ids are frequent) and differ in the draws
        stream = [torch.from_numpy(inputs.zipf_ids(T, V, seed=500 + b, perm_seed=77) if ids_kind == "zipf"
                                   else inputs.uniform_ids(T, V, seed=500 + b))
                  for b in range(max(args.warmup, 10) + args.steps + 3)]   # no batch is seen twice
        E_cached = torch.empty(NS + T, F, dtype=torch.bfloat16, device=dev)
        L.stem_cache_init(ctx, NS)
        turn = [0]

    def step():
        t0 = time.perf_counter()
        if NS > 0:
            ids_b = stream[turn[0] % len(stream)]
            turn[0] += 1
            n, nm, ev = L.stem_prefetch_rows_cached(ctx, E_host, ids_b, E_cached, NS, remap)
            miss_rows[0], uniq_rows[0] = nm, n
            dedup_ms.append((time.perf_counter() - t0) * 1e3)
            L.stem_ffn_forward(ctx, x, remap, Wg, Wd, E_cached, y, wait_event=ev)
            return
        n, ev = L.stem_prefetch_rows(ctx, E_host, ids_host, E_compact, remap)
        dedup_ms.append((time.perf_counter() - t0) * 1e3)
        L.stem_ffn_forward(ctx, x, remap, Wg, Wd, E_compact, y, wait_event=ev, E_rows=n)

    def step_resident():
        L.stem_ffn_forward(ctx, x, ids_dev, Wg, Wd, E_dev, y)

    steps, warm = args.steps, args.warmup
    if NS > 0:
        warm = max(warm, 10)   # the cache fills and settles
    med, p10, p90 = _median_ms(step, steps, warm)
    del dedup_ms[:warm]
    res_med, _, _ = _median_ms(step_resident, steps, warm)
    L.stem_sync_status(ctx)
    # the link itself: one contiguous pinned copy of as many bytes as the rows
    if NS > 0:
        U = miss_rows[0]           # rows that crossed the link in the last batch
    nbytes = max(U, 1) * F * 2
    flat = E_host.view(-1)[: max(U, 1) * F]
    dst = torch.empty(max(U, 1) * F, dtype=torch.bfloat16, device=dev)
    link_med, _, _ = _median_ms(lambda: dst.copy_(flat, non_blocking=True), 5, 2)
    L.stem_profile_enable(ctx, True)
    L.stem_profile_reset(ctx)
    for _ in range(3):
        step()
    prof = L.stem_profile_read(ctx)
    L.stem_profile_enable(ctx, False)
    kernels = {k: {"avg_ms": round(v[0] / v[1], 5), "launches": v[1]} for k, v in prof.items()}
    copy_ms = kernels["row_copy"]["avg_ms"] * kernels["row_copy"]["launches"] / 3 if "row_copy" in kernels else None
    out = {
        "metric": "STEM FFN forward tokens/s, host-resident table", "value": round(T / (med * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": round(med, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": shape.name, "d_model": d, "d_ff": F, "vocab": V, "tokens": T, "n_uniq": uniq_rows[0],
                   "ids": "Zipf(s=1.1)" if ids_kind == "zipf" else "uniform",
                   "cache_slots": NS, "rows_over_the_link": U, "prefetch_mode": getattr(args, "prefetch_mode", "kernel"),
                   "step": "dedup + row copy over the host link (side stream) + forward"},
        "latency_ms": {"median": round(med, 4), "p10": round(p10, 4), "p90": round(p90, 4),
                       "device_resident_forward": round(res_med, 4), "exposed_by_host_table": round(med - res_med, 4),
                       "host_dedup_and_enqueue": round(sorted(dedup_ms)[len(dedup_ms) // 2], 4)},
        "roofline": {"bound": "host link", "kernel": "row_copy", "achieved": None if not copy_ms else
                     round(nbytes / (copy_ms * 1e-3) / 1e9, 2), "peak": round(nbytes / (link_med * 1e-3) / 1e9, 2),
                     "unit": "GB/s", "frac": None if not copy_ms else round(link_med / copy_ms, 4), "traffic": None,
                     "bytes": nbytes, "peak_is": "measured contiguous pinned host-to-device copy of the same size"},
        "kernels": kernels,
    }
    ctx.close()
    return out


def bench_host_training(args, shape, dev):
    """One training step of the layer with the table and its optimiser state resident in pinned host
    memory: de-duplicate, prefetch the distinct rows, forward and backward on the compact rows, table
    gradient, sparse AdamW reading and writing the touched rows of master / m / v / table over the link."""
    import torch

    from paper_2601_10639_amd import inputs, stemlib as L

    T, d, F, V = shape.tokens, shape.d_model, shape.d_ff, shape.vocab
    bf = torch.bfloat16
    inp = inputs.layer_inputs(shape, seed=3, device=dev)
    ids_host = inp["ids"].cpu()
    E_host = inp["E"].cpu().pin_memory()
    master = E_host.float().pin_memory()
    m = torch.zeros(V, F).pin_memory()
    v = torch.zeros(V, F).pin_memory()
    del inp["E"]
    ctx = L.stem_create(d, F, V, L.STEM_BF16, T, 0)
    y, dx = (torch.empty(T, d, dtype=bf, device=dev) for _ in range(2))
    G, H, dU = (torch.empty(T, F, dtype=bf, device=dev) for _ in range(3))
    dWg = torch.empty(F, d, dtype=torch.float32, device=dev)
    dWd = torch.empty(d, F, dtype=torch.float32, device=dev)
    E_compact = torch.empty(T, F, dtype=bf, device=dev)
    remap = torch.empty(T, dtype=torch.int32, device=dev)
    uniq_host = torch.empty(T, dtype=torch.int32).pin_memory()
    uniq_dev = torch.empty(T, dtype=torch.int32, device=dev)
    i32 = torch.int32
    sorted_ids, perm = (torch.empty(T, dtype=i32, device=dev) for _ in range(2))
    uq = torch.empty(T, dtype=i32, device=dev)
    seg_offsets = torch.empty(T + 1, dtype=i32, device=dev)
    n_uniq = torch.zeros(1, dtype=i32, device=dev)
    dE_rows = torch.empty(T, F, dtype=torch.float32, device=dev)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    step_no, U = [0], [0]

    def step():
        step_no[0] += 1
        n, ev = L.stem_prefetch_rows(ctx, E_host, ids_host, E_compact, remap, uniq_host)
        U[0] = n
        uniq_dev[:n].copy_(uniq_host[:n], non_blocking=True)
        L.stem_ffn_forward(ctx, inp["x"], remap, inp["W_gate"], inp["W_down"], E_compact, y, G, H, wait_event=ev,
                           E_rows=n)
        L.stem_ffn_backward(ctx, inp["dy"], inp["x"], remap, inp["W_gate"], inp["W_down"], E_compact, G, H, dx, dWg,
                            dWd, dU, E_rows=n)
        L.stem_embed_grad(ctx, remap, dU, sorted_ids, perm, uq, seg_offsets, n_uniq, dE_rows)
        L.stem_embed_sparse_adamw(ctx, uniq_dev, n_uniq, dE_rows, E_host, master, m, v, step=step_no[0], **hp)

    med, p10, p90 = _median_ms(step, args.steps, args.warmup)
    L.stem_sync_status(ctx)
    L.stem_profile_enable(ctx, True)
    L.stem_profile_reset(ctx)
    for _ in range(3):
        step()
    prof = L.stem_profile_read(ctx)
    L.stem_profile_enable(ctx, False)
    kernels = {k: {"avg_ms": round(val[0] / val[1], 5), "launches": val[1]} for k, val in prof.items()}
    n = U[0]
    ad = kernels["sparse_adamw"]["avg_ms"]
    rd, wr = n * F * 12, n * F * 14          # master, m, v read; master, m, v, bf16 row written
    out = {
        "metric": "STEM FFN fwd+bwd tokens/s per layer, table and optimiser state in host memory",
        "value": round(T / (med * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(med, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": shape.name, "d_model": d, "d_ff": F, "vocab": V, "tokens": T, "n_uniq": n,
                   "ids": "Zipf(s=1.1)", "step": "dedup+prefetch+fwd+bwd+embed_grad+sparse_adamw on host-resident state"},
        "latency_ms": {"median": round(med, 4), "p10": round(p10, 4), "p90": round(p90, 4)},
        "roofline": {"bound": "host link", "kernel": "sparse_adamw", "achieved": round(max(rd, wr) / (ad * 1e-3) / 1e9, 2),
                     "peak": None, "unit": "GB/s in the busier direction", "frac": None, "traffic": None,
                     "bytes": {"read_over_link": rd, "written_over_link": wr}},
        "kernels": kernels,
    }
    print(json.dumps(out))
    ctx.close()
    return 0


def cpu_baseline(shape, inp, n_tok, hp):
    """The oracle, as it stands, on the first n_tok tokens of the same batch (full widths;
    the table is cut down to the rows those tokens name, which leaves the layer unchanged)."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle import stem_oracle as O
    from paper_2601_10639_amd import inputs

    n_tok = min(n_tok, shape.tokens)
    ids = inp["ids"][:n_tok].cpu().numpy()
    uniq, remap = np.unique(ids, return_inverse=True)
    E_sub = inputs.to_f64(inp["E"][torch_index(inp["E"], uniq)])
    x = inputs.to_f64(inp["x"][:n_tok])
    dy = inputs.to_f64(inp["dy"][:n_tok])
    Wg = inputs.to_f64(inp["W_gate"])
    Wd = inputs.to_f64(inp["W_down"])
    t0 = time.perf_counter()
    O.ffn_forward(x, remap, Wg, Wd, E_sub)
    bw = O.ffn_backward(dy, x, remap, Wg, Wd, E_sub)
    eg = O.embed_grad(remap, bw["dU"])
    z = np.zeros_like(E_sub)
    O.sparse_adamw(eg["uniq_ids"], eg["dE_rows"], E_sub, z, z, step=1, **hp)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": round(n_tok / dt, 2), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"first {n_tok} of {shape.tokens} tokens, full d_model/d_ff, fp64 numpy, {dt:.1f} s"}


def torch_index(E, uniq):
    import torch
    return torch.from_numpy(uniq.astype("int64")).to(E.device)


if __name__ == "__main__":
    sys.exit(main())
