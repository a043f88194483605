"""Shared plumbing of the GPU parity tests: runs the HIP path through the C ABI binding and
the oracle on the same seeded inputs.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from oracle import stem_oracle as O
from paper_2601_10639_amd import inputs, stemlib as L

ADAMW = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)

# Tolerances (max |gpu - ref| / max |ref| per tensor).  fp32 runs accumulate in fp32 over
# at most a few hundred terms: 1e-5.  bf16 runs round G, H, dG, dU, y, dx to bf16 (relative
# 2^-9 each) on top of fp32 accumulation: 2e-2.
TOL = {"f32": 1e-5, "bf16": 2e-2}


def max_rel(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    den = np.abs(ref).max()
    if den == 0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / den)


def make_ctx(shape: inputs.StemShape, max_tokens: int, reserve: int = 0) -> L.StemCtx:
    dt = L.STEM_BF16 if shape.dtype == "bf16" else L.STEM_F32
    return L.stem_create(shape.d_model, shape.d_ff, shape.vocab, dt, max_tokens, 0, reserve=reserve)


def hip_forward_backward(ctx, inp, save_H=True, want_dx=True, after_forward=None):
    """forward + backward through libstem; returns device tensors.  `after_forward()` runs between the two calls."""
    dev = inp["x"].device
    dt = inp["x"].dtype
    T, d = inp["x"].shape
    F = inp["W_gate"].shape[0]
    y = torch.empty(T, d, dtype=dt, device=dev)
    G = torch.empty(T, F, dtype=dt, device=dev)
    H = torch.empty(T, F, dtype=dt, device=dev) if save_H else None
    L.stem_ffn_forward(ctx, inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], inp["E"], y, G, H)
    if after_forward is not None:
        after_forward()
    dx = torch.empty(T, d, dtype=dt, device=dev) if want_dx else None
    dWg = torch.empty(F, d, dtype=torch.float32, device=dev)
    dWd = torch.empty(d, F, dtype=torch.float32, device=dev)
    dU = torch.empty(T, F, dtype=dt, device=dev)
    L.stem_ffn_backward(ctx, inp["dy"], inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], inp["E"], G, H, dx,
                        dWg, dWd, dU)
    return {"y": y, "G": G, "H": H, "dx": dx, "dW_gate": dWg, "dW_down": dWd, "dU": dU}


def hip_embed_grad(ctx, ids, dU, V, with_rows=True, stream=None):
    dev = ids.device
    T = ids.shape[0]
    cap = max(1, min(T, V))
    out = {
        "sorted_ids": torch.empty(max(T, 1), dtype=torch.int32, device=dev),
        "perm": torch.empty(max(T, 1), dtype=torch.int32, device=dev),
        "uniq_ids": torch.empty(cap, dtype=torch.int32, device=dev),
        "seg_offsets": torch.empty(cap + 1, dtype=torch.int32, device=dev),
        "n_uniq": torch.full((1,), -7, dtype=torch.int32, device=dev),
    }
    F = ctx.d_ff
    out["dE_rows"] = torch.empty(cap, F, dtype=torch.float32, device=dev) if with_rows else None
    L.stem_embed_grad(ctx, ids, dU if with_rows else None, out["sorted_ids"], out["perm"], out["uniq_ids"],
                      out["seg_offsets"], out["n_uniq"], out["dE_rows"], T=T, stream=stream)
    return out


def check_integers(eg, ids_np):
    """Bit-exact comparison of the sort / unique outputs with the oracle's."""
    T = len(ids_np)
    s, p = O.sort_ids(ids_np)
    u, offs = O.unique_segments(s)
    U = int(eg["n_uniq"].item())
    assert U == len(u)
    np.testing.assert_array_equal(eg["sorted_ids"][:T].cpu().numpy(), s)
    np.testing.assert_array_equal(eg["perm"][:T].cpu().numpy(), p)
    np.testing.assert_array_equal(eg["uniq_ids"][:U].cpu().numpy(), u)
    np.testing.assert_array_equal(eg["seg_offsets"][:U + 1].cpu().numpy(), offs)
    return U
