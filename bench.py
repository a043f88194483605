#!/usr/bin/env python3
"""Benchmark of the STEM FFN hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic tokens, all inputs already
in HBM: stem_ffn_forward (gate GEMM with fused SiLU*gather, down GEMM), stem_ffn_backward
(four GEMMs, fused dU/dG), stem_embed_grad (sort, unique, segmented sum) and
stem_embed_sparse_adamw on the touched rows.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3|C2|C1]
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
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy (reference point for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2601_10639_amd import inputs, stemlib as L

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    L.lib()  # fails loudly if libstem.so has not been built
    dev = "cuda:0"
    shape = inputs.SHAPES[args.workload]
    T, d, F, V = shape.tokens, shape.d_model, shape.d_ff, shape.vocab
    bf16 = shape.dtype == "bf16"
    dt = inputs.torch_dtype(shape.dtype)

    inp = inputs.layer_inputs(shape, seed=3, device=dev)
    ctx = L.stem_create(d, F, V, L.STEM_BF16 if bf16 else L.STEM_F32, T, 0)
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

    def step():
        step_no[0] += 1
        L.stem_ffn_forward(ctx, inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], E, y, G, H)
        L.stem_ffn_backward(ctx, inp["dy"], inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], E, G, H, dx, dWg,
                            dWd, dU)
        L.stem_embed_grad(ctx, inp["ids"], dU, sorted_ids, perm, uniq_ids, seg_offsets, n_uniq, dE_rows)
        L.stem_embed_sparse_adamw(ctx, uniq_ids, n_uniq, dE_rows, E, master, m, v, step=step_no[0], **hp)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    L.stem_sync_status(ctx)
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = T * args.steps / elapsed
    U = int(n_uniq.item())

    # Per-kernel durations: the same K steps again with HIP events around every launch, on the
    # stream the kernels run on.
    L.stem_profile_enable(ctx, True)
    L.stem_profile_reset(ctx)
    for _ in range(args.steps):
        step()
    prof = L.stem_profile_read(ctx)
    L.stem_profile_enable(ctx, False)

    gemm_flop = 2.0 * T * d * F
    peak_tf = PEAK_BF16_TFLOPS if bf16 else PEAK_FP32_TFLOPS
    es = 2 if bf16 else 4
    algo_bytes = {
        "seg_reduce": T * F * es + U * F * 4,
        "sparse_adamw": U * F * (30 if bf16 else 28),
        "silu_gather": 2 * T * F * es + U * F * es,
    }
    kernels = {}
    for name, (ms, n) in prof.items():
        avg = ms / n
        k = {"avg_ms": round(avg, 5), "launches": n}
        if name.startswith("gemm_"):
            k["tflops"] = round(gemm_flop / (avg * 1e-3) / 1e12, 2)
            k["frac_mfma_peak"] = round(k["tflops"] / peak_tf, 4)
        elif name in algo_bytes:
            k["gbs"] = round(algo_bytes[name] / (avg * 1e-3) / 1e9, 1)
            k["frac_hbm_peak"] = round(k["gbs"] / PEAK_HBM_GBS, 4)
        kernels[name] = k
    # measured HBM-side bytes per launch (rocprofv3 FETCH_SIZE / WRITE_SIZE), if a summary for this workload is committed
    traffic = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s.json" % shape.name.replace("-", "_"))
    if os.path.exists(tpath):
        with open(tpath) as fh:
            traffic = {k: v for k, v in json.load(fh).items() if not k.startswith("_")}
    gemms = {k: v for k, v in kernels.items() if k.startswith("gemm_")}
    dom = max(gemms, key=lambda k: gemms[k]["avg_ms"] * gemms[k]["launches"])
    all_gemm_ms = sum(v["avg_ms"] for v in gemms.values())
    roofline = {
        "bound": "mfma" if bf16 else "alu",
        "kernel": dom,
        "achieved": gemms[dom]["tflops"],
        "peak": peak_tf,
        "unit": "TFLOP/s",
        "frac": round(gemms[dom]["tflops"] / peak_tf, 4),
        "traffic": traffic.get(dom),
        "all_gemms_tflops": round(len(gemms) * gemm_flop / (all_gemm_ms * 1e-3) / 1e12, 2),
        "all_gemms_frac": round(len(gemms) * gemm_flop / (all_gemm_ms * 1e-3) / 1e12 / peak_tf, 4),
    }

    out = {
        "metric": "STEM FFN fwd+bwd tokens/s per layer",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": shape.dtype,
        "data": "synthetic",
        "config": {"workload": shape.name, "d_model": d, "d_ff": F, "vocab": V, "tokens": T,
                   "n_uniq": U, "ids": "Zipf(s=1.1)", "step": "fwd+bwd+embed_grad+sparse_adamw"},
        "roofline": roofline,
        "kernels": kernels,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, inp, args.cpu_sample_tokens, hp)
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
