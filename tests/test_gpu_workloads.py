"""GPU parity at the full workload sizes (every element of C2 and C3 against a whole-batch oracle run;
sampled tokens for the 65536-token host-resident case; sampled tokens and sampled columns at the largest
token count a context accepts), the stacked decode chain, and the host-resident-table mode.  All through
the C ABI."""
import os

import numpy as np
import pytest
import torch

from oracle import stem_oracle as O
from paper_2601_10639_amd import inputs, stemlib as L
from tests import harness as Hn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rows(t, idx):
    """Rows idx of a device tensor as fp64 numpy."""
    return inputs.to_f64(t[torch.as_tensor(np.asarray(idx, dtype=np.int64), device=t.device)])


def _full_size_case(name, seed):
    """Whole hot path in the launch configuration bench.py times, against one run of the oracle over
    the whole batch: every element of y, G, H, dx, dU, dW_gate, dW_down and of the table-gradient
    rows is compared.  (The oracle works on the table cut down to the rows the batch names, which
    leaves the layer unchanged.)"""
    shape = inputs.SHAPES[name]
    T, d, F, V = shape.tokens, shape.d_model, shape.d_ff, shape.vocab
    tol = Hn.TOL[shape.dtype]
    inp = inputs.layer_inputs(shape, seed, device=DEV)
    ctx = Hn.make_ctx(shape, T)
    out = Hn.hip_forward_backward(ctx, inp)
    eg = Hn.hip_embed_grad(ctx, inp["ids"], out["dU"], V)
    L.stem_sync_status(ctx)
    ids = inp["ids"].cpu().numpy()
    U = Hn.check_integers(eg, ids)

    uniq_all, remap_all = np.unique(ids, return_inverse=True)
    E_u = _rows(inp["E"], uniq_all)
    Wg, Wd = inputs.to_f64(inp["W_gate"]), inputs.to_f64(inp["W_down"])
    x_all, dy_all = inputs.to_f64(inp["x"]), inputs.to_f64(inp["dy"])
    y, fw = O.ffn_forward(x_all, remap_all, Wg, Wd, E_u)
    errs = {"y": Hn.max_rel(inputs.to_f64(out["y"]), y), "G": Hn.max_rel(inputs.to_f64(out["G"]), fw["g"]),
            "H": Hn.max_rel(inputs.to_f64(out["H"]), fw["h"])}
    del y, fw
    bw = O.ffn_backward(dy_all, x_all, remap_all, Wg, Wd, E_u)
    errs["dx"] = Hn.max_rel(inputs.to_f64(out["dx"]), bw["dx"])
    errs["dU"] = Hn.max_rel(inputs.to_f64(out["dU"]), bw["dU"])
    errs["dW_gate"] = Hn.max_rel(inputs.to_f64(out["dW_gate"]), bw["dW_gate"])
    errs["dW_down"] = Hn.max_rel(inputs.to_f64(out["dW_down"]), bw["dW_down"])
    oeg = O.embed_grad(ids, bw["dU"])
    del bw
    np.testing.assert_array_equal(oeg["uniq_ids"], uniq_all)
    errs["dE_rows"] = Hn.max_rel(inputs.to_f64(eg["dE_rows"][:U]), oeg["dE_rows"])
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"{name}: over tolerance {tol}: {bad} (all: {errs})"
    print(name, "max-relative errors over all elements", {k: float("%.3g" % v) for k, v in errs.items()}, "n_uniq", U)

    # the optimiser state is compared on a sample of features (all touched rows)
    rng = np.random.default_rng(seed)
    fs = np.unique(np.concatenate([[0, 1, 255, 256, F - 1], rng.integers(0, F, 27)]))
    fs_t = torch.as_tensor(fs, device=DEV)
    oeg = {"dE_rows": oeg["dE_rows"][:, fs]}
    # sparse AdamW on the touched rows (own gradients on each side; see the small-size test for why
    # parameters are compared where the gradient's sign is certain)
    E = inp["E"]
    E0_rows = _rows(E, uniq_all)[:, fs]
    master = E.float()
    m = torch.zeros(V, F, dtype=torch.float32, device=DEV)
    v = torch.zeros(V, F, dtype=torch.float32, device=DEV)
    L.stem_embed_sparse_adamw(ctx, eg["uniq_ids"], eg["n_uniq"], eg["dE_rows"], E, master, m, v, step=1, **Hn.ADAMW)
    L.stem_sync_status(ctx)
    ui = torch.as_tensor(uniq_all.astype(np.int64), device=DEV)
    z = np.zeros_like(E0_rows)
    p_ref, m_ref, v_ref = O.sparse_adamw_rows(oeg["dE_rows"], E0_rows, z, z, step=1, **Hn.ADAMW)
    assert Hn.max_rel(inputs.to_f64(m[ui][:, fs_t]), m_ref) <= tol
    assert Hn.max_rel(inputs.to_f64(v[ui][:, fs_t]), v_ref) <= 2 * tol
    sure = np.abs(oeg["dE_rows"]) > 2 * tol * np.abs(oeg["dE_rows"]).max()
    p_gpu = inputs.to_f64(master[ui][:, fs_t])
    assert np.abs(p_gpu - p_ref)[sure].max() / np.abs(p_ref).max() <= 1e-5
    np.testing.assert_array_equal(inputs.to_f64(E[ui][:, fs_t]), O.bf16_round(p_gpu))
    # an untouched row keeps its bits
    untouched = int(np.setdiff1d(np.arange(min(V, 4 * T)), uniq_all)[0])
    assert not m[untouched].any() and not v[untouched].any()
    ctx.close()


def test_c2_350m_shaped_layer_full_size():
    _full_size_case("C2", seed=21)


def test_c3_1b_shaped_layer_full_size():
    _full_size_case("C3", seed=22)


def test_largest_token_count_a_bf16_context_accepts():
    """T = 131071 tokens at d_ff = 8192: the [T, d_ff] activations end 16 KiB below 2^31 bytes, the largest
    the 32-bit buffer offsets of the products allow (stem_create refuses one token more).  T is odd, so every
    product has a ragged last tile and the weight-gradient products a ragged last K tile.  The oracle
    runs (a) the whole layer on a sample of tokens that includes the first and last rows and both sides
    of tile borders (y, G, H, dx, dU rows) and (b) the layer cut down to a sample of d_ff columns, first
    and last included, on ALL tokens, which yields those columns of G, H, dU and dW_down, those rows of
    dW_gate and those columns of the table-gradient rows exactly.  Sort outputs are compared bit for bit."""
    d, F, V = 1024, 8192, 4096
    T = (2 ** 31 - 1) // (2 * F)
    assert T == 131071
    shape = inputs.StemShape("bf16-max-tokens", d, F, V, 1, T, "bf16")
    with pytest.raises(L.StemError):
        Hn.make_ctx(shape, T + 1)
    tol = Hn.TOL["bf16"]
    inp = inputs.layer_inputs(shape, seed=31, device=DEV, tokens=T)
    ctx = Hn.make_ctx(shape, T)
    out = Hn.hip_forward_backward(ctx, inp)
    eg = Hn.hip_embed_grad(ctx, inp["ids"], out["dU"], V)
    L.stem_sync_status(ctx)
    ids = inp["ids"].cpu().numpy()
    U = Hn.check_integers(eg, ids)
    uniq_all, remap_all = np.unique(ids, return_inverse=True)
    Wg, Wd = inputs.to_f64(inp["W_gate"]), inputs.to_f64(inp["W_down"])
    E_u = _rows(inp["E"], uniq_all)
    rng = np.random.default_rng(31)

    # (a) whole layer, sampled tokens
    ts = np.unique(np.concatenate([[0, 1, 255, 256, 257, 65535, 65536, T - 258, T - 257, T - 256, T - 255, T - 2, T - 1],
                                   rng.integers(0, T, 51)]))
    x_s, dy_s = _rows(inp["x"], ts), _rows(inp["dy"], ts)
    y, fw = O.ffn_forward(x_s, remap_all[ts], Wg, Wd, E_u)
    bw = O.ffn_backward(dy_s, x_s, remap_all[ts], Wg, Wd, E_u)
    errs = {"y": Hn.max_rel(_rows(out["y"], ts), y), "G": Hn.max_rel(_rows(out["G"], ts), fw["g"]),
            "H": Hn.max_rel(_rows(out["H"], ts), fw["h"]), "dx": Hn.max_rel(_rows(out["dx"], ts), bw["dx"]),
            "dU": Hn.max_rel(_rows(out["dU"], ts), bw["dU"])}
    del y, fw, bw

    # (b) sampled d_ff columns, all tokens
    fs = np.unique(np.concatenate([[0, 1, 7, 8, 255, 256, F - 9, F - 8, F - 1], rng.integers(0, F, 15)]))
    fs_t = torch.as_tensor(fs, device=DEV)
    x_all, dy_all = inputs.to_f64(inp["x"]), inputs.to_f64(inp["dy"])
    _, fw = O.ffn_forward(x_all, remap_all, Wg[fs], Wd[:, fs], E_u[:, fs])
    errs["G cols"] = Hn.max_rel(inputs.to_f64(out["G"][:, fs_t]), fw["g"])
    errs["H cols"] = Hn.max_rel(inputs.to_f64(out["H"][:, fs_t]), fw["h"])
    del fw
    bw = O.ffn_backward(dy_all, x_all, remap_all, Wg[fs], Wd[:, fs], E_u[:, fs])
    errs["dU cols"] = Hn.max_rel(inputs.to_f64(out["dU"][:, fs_t]), bw["dU"])
    errs["dW_down cols"] = Hn.max_rel(inputs.to_f64(out["dW_down"][:, fs_t]), bw["dW_down"])
    errs["dW_gate rows"] = Hn.max_rel(inputs.to_f64(out["dW_gate"][fs_t]), bw["dW_gate"])
    oeg = O.embed_grad(ids, bw["dU"])
    np.testing.assert_array_equal(oeg["uniq_ids"], uniq_all)
    errs["dE_rows cols"] = Hn.max_rel(inputs.to_f64(eg["dE_rows"][:U][:, fs_t]), oeg["dE_rows"])
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, (bad, errs)
    print("T = 131071:", {k: float("%.3g" % v) for k, v in errs.items()}, "n_uniq", U)
    ctx.close()


def test_widest_layer_a_bf16_context_accepts():
    """d_model = 8192, d_ff = 65472: the fp32 weight gradients end 2 MiB below 2^31 bytes (stem_create
    refuses d_ff = 65536).  600 tokens, so the 256x256-tile kernels run every product, with ragged row
    tiles, 1023 K tiles in dx and 8192 output tiles in each weight gradient.  Checked as in the test
    above: the whole layer on sampled tokens, and the layer cut down to sampled d_ff columns (first and
    last included) on all tokens."""
    d, F, V, T = 8192, 65472, 64, 600
    with pytest.raises(L.StemError):
        Hn.make_ctx(inputs.StemShape("bf16-too-wide", d, F + 64, V, 1, T, "bf16"), T)
    shape = inputs.StemShape("bf16-widest", d, F, V, 1, T, "bf16")
    tol = Hn.TOL["bf16"]
    inp = inputs.layer_inputs(shape, seed=32, device=DEV, tokens=T)
    ctx = Hn.make_ctx(shape, T)
    out = Hn.hip_forward_backward(ctx, inp)
    L.stem_sync_status(ctx)
    ids = inp["ids"].cpu().numpy()
    E = inputs.to_f64(inp["E"])
    rng = np.random.default_rng(32)
    x_all, dy_all = inputs.to_f64(inp["x"]), inputs.to_f64(inp["dy"])

    # (b) sampled d_ff columns, all tokens (before the full weights are widened: less host memory at once)
    fs = np.unique(np.concatenate([[0, 1, 255, 256, F - 65, F - 64, F - 2, F - 1], rng.integers(0, F, 16)]))
    fs_t = torch.as_tensor(fs, device=DEV)
    Wg_s, Wd_s = inputs.to_f64(inp["W_gate"][fs_t]), inputs.to_f64(inp["W_down"][:, fs_t])
    _, fw = O.ffn_forward(x_all, ids, Wg_s, Wd_s, E[:, fs])
    errs = {"G cols": Hn.max_rel(inputs.to_f64(out["G"][:, fs_t]), fw["g"]),
            "H cols": Hn.max_rel(inputs.to_f64(out["H"][:, fs_t]), fw["h"])}
    bw = O.ffn_backward(dy_all, x_all, ids, Wg_s, Wd_s, E[:, fs])
    errs["dU cols"] = Hn.max_rel(inputs.to_f64(out["dU"][:, fs_t]), bw["dU"])
    errs["dW_down cols"] = Hn.max_rel(inputs.to_f64(out["dW_down"][:, fs_t]), bw["dW_down"])
    errs["dW_gate rows"] = Hn.max_rel(inputs.to_f64(out["dW_gate"][fs_t]), bw["dW_gate"])
    del fw, bw

    # (a) whole layer, sampled tokens
    ts = np.unique(np.concatenate([[0, 1, 255, 256, 511, 512, T - 2, T - 1], rng.integers(0, T, 16)]))
    Wg, Wd = inputs.to_f64(inp["W_gate"]), inputs.to_f64(inp["W_down"])
    y, fw = O.ffn_forward(x_all[ts], ids[ts], Wg, Wd, E)
    bw = O.ffn_backward(dy_all[ts], x_all[ts], ids[ts], Wg, Wd, E)
    errs.update({"y": Hn.max_rel(_rows(out["y"], ts), y), "G": Hn.max_rel(_rows(out["G"], ts), fw["g"]),
                 "H": Hn.max_rel(_rows(out["H"], ts), fw["h"]), "dx": Hn.max_rel(_rows(out["dx"], ts), bw["dx"]),
                 "dU": Hn.max_rel(_rows(out["dU"], ts), bw["dU"])})
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, (bad, errs)
    print("d_model 8192, d_ff 65472:", {k: float("%.3g" % v) for k, v in errs.items()})
    ctx.close()


@pytest.mark.parametrize("with_table", [False, True])
def test_c2_shaped_dense_and_additive_layers_full_size(with_table):
    """The dense SwiGLU layer and the additive variant at the 350M shape, every element of every output
    against one run of the oracle over the whole batch.  At this size the backward products read the
    weights and both operands of the weight gradients rows-contiguous over many K tiles, dx runs over
    the concatenated K range of two operand pairs, and the weight gradients are cut along K."""
    shape = inputs.SHAPES["C2"]
    T, d, F, V = shape.tokens, shape.d_model, shape.d_ff, shape.vocab
    tol = Hn.TOL["bf16"]
    inp = inputs.layer_inputs(shape, seed=23, device=DEV)
    Wu = inputs.normal((F, d), 0.02, 24, torch.bfloat16, DEV)
    E = inp["E"] if with_table else None
    ids = inp["ids"] if with_table else None
    ctx = Hn.make_ctx(shape, T, reserve=L.STEM_RESERVE_UP)
    bf = torch.bfloat16
    y = torch.empty(T, d, dtype=bf, device=DEV)
    G, Up, H, dV = (torch.empty(T, F, dtype=bf, device=DEV) for _ in range(4))
    dx = torch.empty(T, d, dtype=bf, device=DEV)
    dWg, dWu = (torch.empty(F, d, dtype=torch.float32, device=DEV) for _ in range(2))
    dWd = torch.empty(d, F, dtype=torch.float32, device=DEV)
    L.stem_ffn_up_forward(ctx, inp["x"], ids, inp["W_gate"], Wu, inp["W_down"], E, y, G, Up, H)
    L.stem_ffn_up_backward(ctx, inp["dy"], inp["x"], ids, inp["W_gate"], Wu, inp["W_down"], E, G, Up, H, dx, dWg, dWu,
                           dWd, dV)
    L.stem_sync_status(ctx)
    ids_np = inp["ids"].cpu().numpy()
    uniq_all, remap_all = np.unique(ids_np, return_inverse=True)
    E_u = _rows(inp["E"], uniq_all) if with_table else None   # the table cut down to the rows the batch names
    Wg, Wd, Wu64 = inputs.to_f64(inp["W_gate"]), inputs.to_f64(inp["W_down"]), inputs.to_f64(Wu)
    x_all, dy_all = inputs.to_f64(inp["x"]), inputs.to_f64(inp["dy"])
    ref, fw = O.up_forward(x_all, remap_all, Wg, Wu64, Wd, E_u)
    errs = {"y": Hn.max_rel(inputs.to_f64(y), ref), "G": Hn.max_rel(inputs.to_f64(G), fw["g"]),
            "Up": Hn.max_rel(inputs.to_f64(Up), fw["up"]), "H": Hn.max_rel(inputs.to_f64(H), fw["h"])}
    del ref, fw
    bw = O.up_backward(dy_all, x_all, remap_all, Wg, Wu64, Wd, E_u)
    errs.update({"dx": Hn.max_rel(inputs.to_f64(dx), bw["dx"]), "dV": Hn.max_rel(inputs.to_f64(dV), bw["dV"]),
                 "dW_gate": Hn.max_rel(inputs.to_f64(dWg), bw["dW_gate"]), "dW_up": Hn.max_rel(inputs.to_f64(dWu), bw["dW_up"]),
                 "dW_down": Hn.max_rel(inputs.to_f64(dWd), bw["dW_down"])})
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, (bad, errs)
    print("C2 dense" if not with_table else "C2 additive", {k: float("%.3g" % v) for k, v in errs.items()})
    ctx.close()


@pytest.mark.parametrize("fused", [False, True])
def test_c4_decode_chain_sixteen_layers(fused):
    """256 single tokens through 16 stacked 1B-shaped layers, residual stream rounded to bf16 between
    layers on both sides; every layer has its own weights and table, the ids are the same."""
    shape = inputs.SHAPES["C4"]
    T, d, F, V = shape.tokens, shape.d_model, shape.d_ff, shape.vocab
    n_layers = 16
    ids_np = inputs.zipf_ids(T, V, seed=31)
    ids = torch.from_numpy(ids_np).to(DEV)
    uniq, remap = np.unique(ids_np, return_inverse=True)
    ui = torch.as_tensor(uniq.astype(np.int64), device=DEV)
    ctx = Hn.make_ctx(shape, T)
    x0 = inputs.normal((T, d), 1.0, 32, torch.bfloat16, DEV)
    x = x0.clone()
    y = torch.empty_like(x)
    layers_ref, outs = [], []
    for l in range(n_layers):
        Wg = inputs.normal((F, d), 0.02, 100 + 3 * l, torch.bfloat16, DEV)
        Wd = inputs.normal((d, F), 0.02, 101 + 3 * l, torch.bfloat16, DEV)
        E = inputs.normal((V, F), 0.02, 102 + 3 * l, torch.bfloat16, DEV)
        if fused:   # the residual add in the down product's epilogue, in place on the stream
            L.stem_ffn_forward_residual(ctx, x, ids, Wg, Wd, E, x, x)
        else:
            L.stem_ffn_forward(ctx, x, ids, Wg, Wd, E, y)
            x = (x.float() + y.float()).to(torch.bfloat16)
        outs.append(x.float().cpu().numpy().astype(np.float64))
        layers_ref.append((inputs.to_f64(Wg), inputs.to_f64(Wd), inputs.to_f64(E[ui])))
        del E
    L.stem_sync_status(ctx)
    ref = O.decode_chain(inputs.to_f64(x0), remap, layers_ref)
    worst = max(Hn.max_rel(outs[l], ref[l]) for l in range(n_layers))
    assert worst <= Hn.TOL["bf16"], worst
    print("decode chain: worst layer error", worst)
    ctx.close()


def test_decode_forward_can_be_captured_in_a_hip_graph():
    """A four-layer decode chain captured once and replayed five times, with eager work and
    synchronisations between the replays; every replay must equal the eager result bit for bit."""
    shape = inputs.StemShape("decode-graph", 512, 1024, 2000, 64, 1, "bf16")
    T, d, F, V = shape.tokens, shape.d_model, shape.d_ff, shape.vocab
    ids = torch.from_numpy(inputs.zipf_ids(T, V, seed=33)).to(DEV)
    ctx = Hn.make_ctx(shape, T)
    layers = [(inputs.normal((F, d), 0.02, 300 + 3 * l, torch.bfloat16, DEV),
               inputs.normal((d, F), 0.02, 301 + 3 * l, torch.bfloat16, DEV),
               inputs.normal((V, F), 0.02, 302 + 3 * l, torch.bfloat16, DEV)) for l in range(4)]
    x0 = inputs.normal((T, d), 1.0, 34, torch.bfloat16, DEV)
    x = x0.clone()
    y = torch.empty_like(x)

    def chain():
        x.copy_(x0)
        for Wg, Wd, E in layers:
            L.stem_ffn_forward(ctx, x, ids, Wg, Wd, E, y)
            x.add_(y)

    chain()
    torch.cuda.synchronize()
    want = x.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        chain()                       # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            chain()
    torch.cuda.synchronize()
    for r in range(5):
        x.zero_()
        y.fill_(3.0)                  # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(x, want), r
        chain()                       # and an eager run in between
        torch.cuda.synchronize()
        assert torch.equal(x, want)
    L.stem_sync_status(ctx)
    ctx.close()


def _prefetch_case(shape, T, ids_np, seed, mode=None):
    d, F, V = shape.d_model, shape.d_ff, shape.vocab
    dt = inputs.torch_dtype(shape.dtype)
    ctx = Hn.make_ctx(shape, T)
    E_host = inputs.normal((V, F), 0.02, seed, dt, "cpu").pin_memory()
    ids_host = torch.from_numpy(ids_np)
    o_uniq, o_remap = O.dedup_remap(ids_np)
    cap = len(o_uniq) + 3
    E_compact = torch.full((cap, F), 7.0, dtype=dt, device=DEV)
    remap = torch.empty(T, dtype=torch.int32, device=DEV)
    uniq_host = torch.empty(cap, dtype=torch.int32)
    if mode == "memcpy":
        L.stem_set_prefetch_mode(ctx, L.STEM_PREFETCH_MEMCPY)
    n, ev = L.stem_prefetch_rows(ctx, E_host, ids_host, E_compact, remap, uniq_host)
    assert n == len(o_uniq) and ev
    x = inputs.normal((T, d), 1.0, seed + 1, dt, DEV)
    Wg = inputs.normal((F, d), 0.02, seed + 2, dt, DEV)
    Wd = inputs.normal((d, F), 0.02, seed + 3, dt, DEV)
    y = torch.empty(T, d, dtype=dt, device=DEV)
    L.stem_ffn_forward(ctx, x, remap, Wg, Wd, E_compact, y, wait_event=ev, E_rows=n)
    L.stem_sync_status(ctx)
    # integers and copied rows: bit-exact
    np.testing.assert_array_equal(uniq_host[:n].numpy(), o_uniq)
    np.testing.assert_array_equal(remap.cpu().numpy(), o_remap)
    want_rows = E_host[torch.from_numpy(o_uniq.astype(np.int64))]
    assert torch.equal(E_compact[:n].cpu().view(torch.int16 if dt == torch.bfloat16 else torch.int32),
                       want_rows.view(torch.int16 if dt == torch.bfloat16 else torch.int32))
    assert bool((E_compact[n:] == 7.0).all())
    # same kernels on the device-resident table with the original ids: bit-identical output
    E_dev = E_host.to(DEV)
    y2 = torch.empty_like(y)
    L.stem_ffn_forward(ctx, x, ids_host.to(DEV), Wg, Wd, E_dev, y2, wait_event=ev)
    L.stem_sync_status(ctx)
    assert torch.equal(y, y2)
    ctx.close()
    return x, Wg, Wd, E_host, y, n


def test_training_step_can_be_captured_in_a_hip_graph():
    """Forward, backward, table gradient and sparse AdamW of one layer captured once and replayed three
    times (the optimiser state moves on with every replay), with eager work and synchronisations
    between the replays; every replay must equal the same sequence run eagerly, bit for bit."""
    shape = inputs.StemShape("train-graph", 256, 1024, 3000, 1, 1100, "bf16")
    T, d, F, V = shape.tokens, shape.d_model, shape.d_ff, shape.vocab
    inp = inputs.layer_inputs(shape, seed=41, device=DEV)
    ctx = Hn.make_ctx(shape, T)
    bf = torch.bfloat16
    y = torch.empty(T, d, dtype=bf, device=DEV)
    G = torch.empty(T, F, dtype=bf, device=DEV)
    H = torch.empty_like(G)
    dU = torch.empty_like(G)
    dx = torch.empty_like(y)
    dWg = torch.empty(F, d, device=DEV)
    dWd = torch.empty(d, F, device=DEV)
    cap = min(T, V)
    i32 = dict(dtype=torch.int32, device=DEV)
    sorted_ids, perm = torch.empty(T, **i32), torch.empty(T, **i32)
    uniq, offs, n_uniq = torch.empty(cap, **i32), torch.empty(cap + 1, **i32), torch.zeros(1, **i32)
    rows = torch.empty(cap, F, device=DEV)
    E = inp["E"].clone()
    master, m, v = E.float(), torch.zeros(V, F, device=DEV), torch.zeros(V, F, device=DEV)

    def reset():
        E.copy_(inp["E"])
        master.copy_(inp["E"].float())
        m.zero_()
        v.zero_()

    def step():
        L.stem_ffn_forward(ctx, inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], E, y, G, H)
        L.stem_ffn_backward(ctx, inp["dy"], inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], E, G, H, dx, dWg, dWd, dU)
        L.stem_embed_grad(ctx, inp["ids"], dU, sorted_ids, perm, uniq, offs, n_uniq, rows)
        L.stem_embed_sparse_adamw(ctx, uniq, n_uniq, rows, E, master, m, v, step=1, **Hn.ADAMW)

    watched = (y, dx, dWg, dWd, E, master, m, v)
    reset()
    want = []
    for r in range(3):
        step()
        torch.cuda.synchronize()
        want.append([t.clone() for t in watched])
    assert not torch.equal(want[0][4], want[2][4])      # the table does move from step to step

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                        # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    reset()
    for r in range(3):
        y.fill_(3.0)                  # eager work between replays
        dWg.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, exp in zip(watched, want[r]):
            assert torch.equal(got, exp), r
    L.stem_sync_status(ctx)
    ctx.close()


@pytest.mark.parametrize("dtype,mode", [("bf16", None), ("bf16", "memcpy"), ("f32", None)])
def test_prefetch_rows_small(dtype, mode):
    shape = inputs.StemShape("host-small", 128, 256, 5000, 1, 3000, dtype)
    ids_np = inputs.zipf_ids(3000, 5000, seed=41)
    x, Wg, Wd, E_host, y, n = _prefetch_case(shape, 3000, ids_np, seed=42, mode=mode)
    ref, _ = O.ffn_forward(inputs.to_f64(x), ids_np, inputs.to_f64(Wg), inputs.to_f64(Wd), inputs.to_f64(E_host))
    assert Hn.max_rel(y.float().cpu(), ref) <= Hn.TOL[dtype]


def test_prefetch_rows_chunked_with_ragged_last_chunk():
    """d_model 2048 gives chunks of 8192 tokens: 20000 tokens are two full chunks and one of 3616,
    each waiting only for the rows its tokens use first.  Every token is checked."""
    T = 20000
    shape = inputs.StemShape("host-chunked", 2048, 128, 5000, 1, T, "bf16")
    ids_np = inputs.uniform_ids(T, 5000, seed=43)
    x, Wg, Wd, E_host, y, n = _prefetch_case(shape, T, ids_np, seed=44)
    ref, _ = O.ffn_forward(inputs.to_f64(x), ids_np, inputs.to_f64(Wg), inputs.to_f64(Wd), inputs.to_f64(E_host))
    assert Hn.max_rel(y.float().cpu(), ref) <= Hn.TOL["bf16"]


@pytest.mark.parametrize("T,d", [(3000, 128), (20000, 2048)])   # 20000 tokens at d_model 2048: three chunks
def test_lfu_row_cache_stream_matches_the_oracle_policy(T, d):
    """Ten batches of one Zipf stream through the cached prefetch: remap, miss count and the content
    of every cache slot equal the oracle's policy bit for bit; every token finds its own row in the
    device buffer; the layer computed from it matches the oracle."""
    V, F, n_slots = 5000, 128, 600
    shape = inputs.StemShape("host-cached", d, F, V, 1, T, "bf16")
    ctx = Hn.make_ctx(shape, T)
    E_host = inputs.normal((V, F), 0.02, 61, torch.bfloat16, "cpu").pin_memory()
    E_dev = torch.zeros(n_slots + T, F, dtype=torch.bfloat16, device=DEV)
    remap = torch.empty(T, dtype=torch.int32, device=DEV)
    x = inputs.normal((T, d), 1.0, 62, torch.bfloat16, DEV)
    Wg = inputs.normal((F, d), 0.02, 63, torch.bfloat16, DEV)
    Wd = inputs.normal((d, F), 0.02, 64, torch.bfloat16, DEV)
    y = torch.empty(T, d, dtype=torch.bfloat16, device=DEV)
    L.stem_cache_init(ctx, n_slots)
    ref_cache = O.LfuRowCache(V, n_slots)
    hits = []
    for b in range(10):
        ids_np = inputs.zipf_ids(T, V, seed=200 + b, perm_seed=9)
        o_remap, o_misses, _ = ref_cache.step(ids_np)
        n_uniq, n_miss, ev = L.stem_prefetch_rows_cached(ctx, E_host, torch.from_numpy(ids_np), E_dev, n_slots, remap)
        L.stem_ffn_forward(ctx, x, remap, Wg, Wd, E_dev, y, wait_event=ev)
        torch.cuda.synchronize()
        L.stem_sync_status(ctx)
        assert n_uniq == len(np.unique(ids_np)) and n_miss == len(o_misses)
        np.testing.assert_array_equal(remap.cpu().numpy(), o_remap)
        np.testing.assert_array_equal(L.stem_cache_state(ctx, n_slots).numpy(), np.asarray(ref_cache.id_in_slot))
        rows = E_dev[remap.long()].cpu().view(torch.int16)
        assert torch.equal(rows, E_host[torch.from_numpy(ids_np.astype(np.int64))].view(torch.int16))
        state = L.stem_cache_state(ctx, n_slots).long()
        used = state >= 0
        assert torch.equal(E_dev[:n_slots][used.to(DEV)].cpu().view(torch.int16), E_host[state[used]].view(torch.int16))
        hits.append(1.0 - n_miss / n_uniq)
    tok = np.arange(0, T, max(1, T // 64))
    uniq_t, remap_t = np.unique(ids_np[tok], return_inverse=True)
    ref, _ = O.ffn_forward(_rows(x, tok), remap_t, inputs.to_f64(Wg), inputs.to_f64(Wd),
                           inputs.to_f64(E_host[torch.from_numpy(uniq_t.astype(np.int64))]))
    assert Hn.max_rel(_rows(y, tok), ref) <= Hn.TOL["bf16"]
    assert hits[0] == 0.0 and hits[-1] > 0.15, hits   # rows (not tokens) served from the cache
    print("row hit rate per batch", [round(h, 2) for h in hits])
    ctx.close()


def test_training_steps_with_host_resident_table_and_optimiser_state():
    """Three training steps with the table, its fp32 master and the AdamW moments in pinned host
    memory: rows prefetched, forward and backward on the compact rows, table gradient, sparse AdamW
    straight on the host-resident state.  The oracle runs the same three steps on its own arrays."""
    T, d, F, V = 1500, 128, 256, 3000
    shape = inputs.StemShape("host-train", d, F, V, 1, T, "bf16")
    bf = torch.bfloat16
    ctx = Hn.make_ctx(shape, T)
    E_host = inputs.normal((V, F), 0.02, 71, bf, "cpu").pin_memory()
    master = E_host.float().pin_memory()
    m = torch.zeros(V, F).pin_memory()
    v = torch.zeros(V, F).pin_memory()
    Wg = inputs.normal((F, d), 0.02, 72, bf, DEV)
    Wd = inputs.normal((d, F), 0.02, 73, bf, DEV)
    o_master, o_m, o_v = inputs.to_f64(E_host), np.zeros((V, F)), np.zeros((V, F))
    o_E = o_master.copy()
    E0 = E_host.float().numpy().copy()
    touched = np.zeros(0, dtype=np.int64)
    E_compact = torch.empty(T, F, dtype=bf, device=DEV)
    remap = torch.empty(T, dtype=torch.int32, device=DEV)
    uniq_host = torch.empty(T, dtype=torch.int32)
    y, dx = (torch.empty(T, d, dtype=bf, device=DEV) for _ in range(2))
    G, H, dU = (torch.empty(T, F, dtype=bf, device=DEV) for _ in range(3))
    dWg = torch.empty(F, d, dtype=torch.float32, device=DEV)
    dWd = torch.empty(d, F, dtype=torch.float32, device=DEV)
    for step in range(1, 4):
        ids_np = inputs.zipf_ids(T, V, seed=80 + step, perm_seed=3)
        x = inputs.normal((T, d), 1.0, 90 + step, bf, DEV)
        dy = inputs.normal((T, d), 1.0, 95 + step, bf, DEV)
        n, ev = L.stem_prefetch_rows(ctx, E_host, torch.from_numpy(ids_np), E_compact, remap, uniq_host)
        L.stem_ffn_forward(ctx, x, remap, Wg, Wd, E_compact, y, G, H, wait_event=ev, E_rows=n)
        L.stem_ffn_backward(ctx, dy, x, remap, Wg, Wd, E_compact, G, H, dx, dWg, dWd, dU, E_rows=n)
        # the compact slots are the distinct ids in ascending order, so the gradient rows of the slots
        # are the gradient rows of the table rows uniq_host[:n]
        eg = Hn.hip_embed_grad(ctx, remap, dU, n)
        assert int(eg["n_uniq"].item()) == n
        L.stem_embed_sparse_adamw(ctx, uniq_host[:n].to(DEV), eg["n_uniq"], eg["dE_rows"], E_host, master, m, v,
                                  step=step, **Hn.ADAMW)
        torch.cuda.synchronize()
        L.stem_sync_status(ctx)
        # oracle: same step on the bf16 table it holds, its own gradients, its own state
        bw = O.ffn_backward(inputs.to_f64(dy), inputs.to_f64(x), ids_np, inputs.to_f64(Wg), inputs.to_f64(Wd), o_E)
        oeg = O.embed_grad(ids_np, bw["dU"])
        np.testing.assert_array_equal(uniq_host[:n].numpy(), oeg["uniq_ids"])
        assert Hn.max_rel(eg["dE_rows"][:n].cpu(), oeg["dE_rows"]) <= Hn.TOL["bf16"]
        o_master, o_m, o_v = O.sparse_adamw(oeg["uniq_ids"], oeg["dE_rows"], o_master, o_m, o_v, step=step, **Hn.ADAMW)
        o_E = O.bf16_round(o_master)
        assert Hn.max_rel(m.numpy(), o_m) <= Hn.TOL["bf16"]
        assert Hn.max_rel(v.numpy(), o_v) <= 2 * Hn.TOL["bf16"]
        # rows no batch has named so far: bit-identical to the initial table on both sides; the bf16
        # table is the rounded master everywhere
        touched = np.union1d(touched, oeg["uniq_ids"])
        untouched = np.setdiff1d(np.arange(V), touched)
        np.testing.assert_array_equal(master.numpy()[untouched], E0[untouched])
        np.testing.assert_array_equal(o_master[untouched].astype(np.float32), E0[untouched])
        assert torch.equal(E_host.view(torch.int16), master.to(bf).view(torch.int16))
        if step == 1:   # the first update is lr * sign(g): compare where the sign of g is beyond its error bound
            sure = np.abs(oeg["dE_rows"]) > 2 * Hn.TOL["bf16"] * np.abs(oeg["dE_rows"]).max()
            diff = np.abs(master.numpy()[oeg["uniq_ids"]] - o_master[oeg["uniq_ids"]])[sure].max()
            assert sure.any() and diff / np.abs(o_master).max() <= 1e-5, diff
    ctx.close()


def test_prefetch_rows_errors():
    shape = inputs.StemShape("host-err", 64, 64, 100, 1, 50, "bf16")
    ctx = Hn.make_ctx(shape, 50)
    E_host = inputs.normal((100, 64), 0.02, 1, torch.bfloat16, "cpu").pin_memory()
    ids = torch.arange(50, dtype=torch.int32)
    E_compact = torch.empty(10, 64, dtype=torch.bfloat16, device=DEV)
    remap = torch.empty(50, dtype=torch.int32, device=DEV)
    with pytest.raises(L.StemError) as e:
        L.stem_prefetch_rows(ctx, E_host, ids, E_compact, remap)
    assert e.value.status == L.STEM_ERR_WORKSPACE
    bad = ids.clone(); bad[7] = 100
    E_big = torch.empty(50, 64, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(L.StemError) as e:
        L.stem_prefetch_rows(ctx, E_host, bad, E_big, remap)
    assert e.value.status == L.STEM_ERR_ID_RANGE
    n, ev = L.stem_prefetch_rows(ctx, E_host, ids, E_big, remap)   # the context is still usable
    assert n == 50
    torch.cuda.synchronize()
    ctx.close()


@pytest.mark.parametrize("dist", ["zipf", "uniform"])
def test_c5_long_context_host_resident_table(dist):
    """One 1B-shaped layer, 65536 tokens, table in pinned host memory; the oracle checks sampled tokens."""
    shape = inputs.SHAPES["C5"]
    T, V = shape.tokens, shape.vocab
    ids_np = inputs.zipf_ids(T, V, seed=51) if dist == "zipf" else inputs.uniform_ids(T, V, seed=52)
    x, Wg, Wd, E_host, y, n = _prefetch_case(shape, T, ids_np, seed=53)
    rng = np.random.default_rng(5)
    tok = np.unique(np.concatenate([[0, 255, 256, T - 1], rng.integers(0, T, 28)]))
    uniq_t, remap_t = np.unique(ids_np[tok], return_inverse=True)
    E_t = inputs.to_f64(E_host[torch.from_numpy(uniq_t.astype(np.int64))])
    ref, _ = O.ffn_forward(_rows(x, tok), remap_t, inputs.to_f64(Wg), inputs.to_f64(Wd), E_t)
    err = Hn.max_rel(_rows(y, tok), ref)
    assert err <= Hn.TOL["bf16"], err
    print(f"C5 {dist}: n_uniq {n} ({n * shape.d_ff * 2 / 1e6:.0f} MB of rows), sampled error {err:.3g}")
