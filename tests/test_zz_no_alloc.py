"""The table-gradient entry point that allocates nothing (static device scratch, no context), called
through the C ABI: its results against stem_embed_grad's on the same inputs, twice in a row, the
second call on a smaller input (so whatever the first call left in the shared scratch is there to
be tripped over)."""
import numpy as np
import pytest
import torch

from oracle import stem_oracle as O
from paper_2601_10639_amd import inputs, stemlib as L
from tests import harness as Hn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _noalloc(dtype, V, F, ids, dU):
    T = ids.shape[0]
    cap = max(1, min(T, V))
    i32 = dict(dtype=torch.int32, device=DEV)
    out = {"sorted_ids": torch.full((max(T, 1),), -5, **i32), "perm": torch.full((max(T, 1),), -5, **i32),
           "uniq_ids": torch.full((cap,), -5, **i32), "seg_offsets": torch.full((cap + 1,), -5, **i32),
           "n_uniq": torch.full((1,), -7, **i32), "dE_rows": torch.full((cap, F), 3.0, dtype=torch.float32, device=DEV)}
    flag = torch.zeros(1, **i32)
    L.stem_embed_grad_noalloc(dtype, V, F, ids, dU, out["sorted_ids"], out["perm"], out["uniq_ids"],
                              out["seg_offsets"], out["n_uniq"], out["dE_rows"], id_flag=flag)
    return out, flag


@pytest.mark.parametrize("dtype,V,F,sizes", [
    ("bf16", 128256, 8192, (16384, 5000)),      # the 1B-shaped layer's batch (one-workgroup sort), then a smaller one
    ("bf16", 50304, 1024, (40000, 16384)),      # multi-kernel sort, then the one-workgroup sort
    ("f32", 1000, 256, (3000, 128)),
])
def test_no_alloc_entry_point_matches_the_context_one_on_two_calls_in_a_row(dtype, V, F, sizes):
    shape = inputs.StemShape("noalloc", 64, F, V, 1, max(sizes), dtype)
    dt = inputs.torch_dtype(dtype)
    code = L.STEM_BF16 if dtype == "bf16" else L.STEM_F32
    ctx = Hn.make_ctx(shape, max(sizes))
    for k, T in enumerate(sizes):
        ids_np = inputs.zipf_ids(T, V, seed=900 + k)
        ids = torch.from_numpy(ids_np).to(DEV)
        dU = inputs.normal((T, F), 1.0, 910 + k, dt, DEV)
        got, flag = _noalloc(code, V, F, ids, dU)
        want = Hn.hip_embed_grad(ctx, ids, dU, V)
        torch.cuda.synchronize()
        L.stem_sync_status(ctx)
        U = Hn.check_integers(got, ids_np)                  # bit-exact against the oracle's sort / unique / offsets
        assert U == int(want["n_uniq"].item())
        for name in ("sorted_ids", "perm"):
            assert torch.equal(got[name][:T], want[name][:T]), name
        assert torch.equal(got["uniq_ids"][:U], want["uniq_ids"][:U])
        assert torch.equal(got["seg_offsets"][:U + 1], want["seg_offsets"][:U + 1])
        # same kernels, same fixed summation order: the row sums are bit-identical
        assert torch.equal(got["dE_rows"][:U], want["dE_rows"][:U])
        assert bool((got["dE_rows"][U:] == 3.0).all())      # rows beyond n_uniq are not written
        assert int(flag.item()) == 0
        oeg = O.embed_grad(ids_np, inputs.to_f64(dU))
        assert Hn.max_rel(got["dE_rows"][:U].cpu(), oeg["dE_rows"]) <= 1e-5
    ctx.close()


def test_no_alloc_entry_point_limits_and_flag():
    V, F = 300, 64
    ids = torch.from_numpy(inputs.zipf_ids(200, V, seed=930)).to(DEV)
    bad = ids.clone()
    bad[17] = V
    dU = inputs.normal((200, F), 1.0, 931, torch.bfloat16, DEV)
    out, flag = _noalloc(L.STEM_BF16, V, F, bad, dU)
    torch.cuda.synchronize()
    assert int(flag.item()) == 1                            # reported, and clamped to the last row
    Hn.check_integers(out, np.clip(bad.cpu().numpy(), 0, V - 1))
    # integer part only
    i32 = dict(dtype=torch.int32, device=DEV)
    s, p, u, o, n = (torch.empty(200, **i32), torch.empty(200, **i32), torch.empty(200, **i32),
                     torch.empty(201, **i32), torch.zeros(1, **i32))
    L.stem_embed_grad_noalloc(L.STEM_BF16, V, F, ids, None, s, p, u, o, n, None)
    torch.cuda.synchronize()
    Hn.check_integers({"sorted_ids": s, "perm": p, "uniq_ids": u, "seg_offsets": o, "n_uniq": n}, ids.cpu().numpy())
    # beyond the static scratch: refused on the host with the limit named, nothing launched
    big = torch.zeros(65537, **i32)
    with pytest.raises(L.StemError) as e:
        L.stem_embed_grad_noalloc(L.STEM_BF16, V, F, big, None, big, big, big, big, n, None)
    assert e.value.status == L.STEM_ERR_SHAPE and "65536" in str(e.value)
    ids2 = torch.zeros(32768, **i32)
    dU2 = torch.zeros(1, 8, dtype=torch.bfloat16, device=DEV)   # never read: the call is refused first
    with pytest.raises(L.StemError) as e:
        L.stem_embed_grad_noalloc(L.STEM_BF16, V, 8192, ids2, dU2, ids2, ids2, ids2, ids2, n, torch.zeros(1, 8, device=DEV), T=32768)
    assert e.value.status == L.STEM_ERR_SHAPE and "partial sums" in str(e.value)
    with pytest.raises(L.StemError) as e:
        L.stem_embed_grad_noalloc(7, V, F, ids, None, s, p, u, o, n, None)
    assert e.value.status == L.STEM_ERR_INVALID_ARG
