"""Seeded synthetic inputs for the STEM FFN layer.

This module is the one piece that both the HIP path's callers (tests, bench)
and the CPU oracle's callers draw from.  It holds no arithmetic of the method
itself: only random draws, the workload shapes, and dtype quantisation of the
drawn values.  Token streams follow a bounded Zipf law because the paper's
system section states that input token ids are Zipfian; the exponent (1.1) and
the shapes are this build's workload definition, standing in for the paper's
pre-training token streams.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class StemShape:
    """One workload: a single STEM layer (Method, STEM definition) and its token batch."""

    name: str
    d_model: int
    d_ff: int
    vocab: int
    n_seqs: int
    seq_len: int
    dtype: str  # "f32" or "bf16": storage type of activations, weights and the table

    @property
    def tokens(self) -> int:
        return self.n_seqs * self.seq_len


SHAPES = {
    # tiny fp32 layer the oracle finishes in well under a second
    "C1": StemShape("C1-tiny-f32", 64, 256, 1000, 2, 64, "f32"),
    # 350M-shaped layer
    "C2": StemShape("C2-350M-bf16", 1024, 4096, 50304, 8, 2048, "bf16"),
    # 1B-shaped layer (Llama-3.2-1B widths; table = 128256 x 8192)
    "C3": StemShape("C3-1B-bf16", 2048, 8192, 128256, 4, 4096, "bf16"),
    # one decode step: 256 single tokens, stacked 1B-shaped layers
    "C4": StemShape("C4-decode-bf16", 2048, 8192, 128256, 256, 1, "bf16"),
    # long-context forward, table resident in host memory
    "C5": StemShape("C5-long-bf16", 2048, 8192, 128256, 1, 65536, "bf16"),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def zipf_ids(n: int, vocab: int, seed: int, s: float = 1.1, permute: bool = True,
             perm_seed: int | None = None) -> np.ndarray:
    """n token ids in [0, vocab) with P(rank k) proportional to k**-s, k = 1..vocab.

    Sampling is inverse-CDF on an fp64 cumulative table.  With `permute` the
    rank -> id map is a seeded permutation, so frequent rows are scattered
    through the table as in a real vocabulary; otherwise rank k maps to id k-1.
    Successive batches of one token stream share `perm_seed` (the vocabulary)
    and differ in `seed` (the draws); by default each seed has its own vocabulary.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = rng.random(n)
    ranks = np.minimum(np.searchsorted(cdf, u, side="right"), vocab - 1)
    if permute:
        pi = np.random.Generator(np.random.PCG64(seed + 7919 if perm_seed is None else perm_seed)).permutation(vocab)
        ranks = pi[ranks]
    return ranks.astype(np.int32)


def uniform_ids(n: int, vocab: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def normal(shape, std: float, seed: int, dtype: torch.dtype, device="cpu") -> torch.Tensor:
    """N(0, std^2) draws, rounded to `dtype` (round-to-nearest-even by torch)."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    t.mul_(std)
    return t.to(dtype)


def layer_inputs(shape: StemShape, seed: int, device="cpu", tokens: int | None = None,
                 ids: np.ndarray | None = None) -> dict:
    """All tensors one forward+backward of a layer needs.

    x ~ N(0,1) for the bf16 shapes and N(0, 0.02^2) for the fp32 tiny shape;
    W_gate [d_ff, d_model], W_down [d_model, d_ff] and the table E [vocab, d_ff]
    ~ N(0, 0.02^2); upstream gradient dy ~ N(0,1).  Everything is rounded to the
    shape's storage dtype, so both sides of a parity test start from the same bits.
    """
    dt = torch_dtype(shape.dtype)
    T = shape.tokens if tokens is None else tokens
    x_std = 0.02 if shape.dtype == "f32" else 1.0
    if ids is None:
        ids = zipf_ids(T, shape.vocab, seed * 1000 + 1)
    out = {
        "ids": torch.from_numpy(np.ascontiguousarray(ids)).to(device),
        "x": normal((T, shape.d_model), x_std, seed * 1000 + 2, dt, device),
        "W_gate": normal((shape.d_ff, shape.d_model), 0.02, seed * 1000 + 3, dt, device),
        "W_down": normal((shape.d_model, shape.d_ff), 0.02, seed * 1000 + 4, dt, device),
        "E": normal((shape.vocab, shape.d_ff), 0.02, seed * 1000 + 5, dt, device),
        "dy": normal((T, shape.d_model), 1.0, seed * 1000 + 6, dt, device),
    }
    return out


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a stored tensor to an fp64 numpy array (for the oracle)."""
    return t.detach().to("cpu").to(torch.float64).numpy()
