"""GPU parity: libstem (through the C ABI) against the CPU oracle on the same seeded inputs.
Integer outputs are compared bit for bit; floating outputs by max |gpu-ref| / max |ref|."""
import numpy as np
import pytest
import torch

from oracle import stem_oracle as O
from paper_2601_10639_amd import inputs, stemlib as L
from tests import harness as Hn

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _oracle_all(inp):
    f64 = {k: inputs.to_f64(v) for k, v in inp.items() if k != "ids"}
    ids = inp["ids"].cpu().numpy()
    y, fw = O.ffn_forward(f64["x"], ids, f64["W_gate"], f64["W_down"], f64["E"])
    bw = O.ffn_backward(f64["dy"], f64["x"], ids, f64["W_gate"], f64["W_down"], f64["E"])
    eg = O.embed_grad(ids, bw["dU"])
    return y, fw, bw, eg


def _pipeline_case(shape, T, seed, save_H=True, ids=None):
    inp = inputs.layer_inputs(shape, seed, device=DEV, tokens=T, ids=ids)
    ctx = Hn.make_ctx(shape, max(T, 1))
    tol = Hn.TOL[shape.dtype]
    out = Hn.hip_forward_backward(ctx, inp, save_H=save_H)
    eg = Hn.hip_embed_grad(ctx, inp["ids"], out["dU"], shape.vocab)
    L.stem_sync_status(ctx)
    y, fw, bw, oeg = _oracle_all(inp)
    errs = {
        "y": Hn.max_rel(out["y"].float().cpu(), y),
        "G": Hn.max_rel(out["G"].float().cpu(), fw["g"]),
        "dx": Hn.max_rel(out["dx"].float().cpu(), bw["dx"]),
        "dW_gate": Hn.max_rel(out["dW_gate"].cpu(), bw["dW_gate"]),
        "dW_down": Hn.max_rel(out["dW_down"].cpu(), bw["dW_down"]),
        "dU": Hn.max_rel(out["dU"].float().cpu(), bw["dU"]),
    }
    if save_H:
        errs["H"] = Hn.max_rel(out["H"].float().cpu(), fw["h"])
    U = Hn.check_integers(eg, inp["ids"].cpu().numpy())
    errs["dE_rows"] = Hn.max_rel(eg["dE_rows"][:U].cpu(), oeg["dE_rows"])
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"{shape.name} T={T}: over tolerance {tol}: {bad} (all: {errs})"

    # one sparse AdamW step at the end of each side's own chain (GPU: its gradient rows;
    # oracle: its own).  The moments are smooth in the gradient and carry its tolerance; the
    # step-1 parameter update is lr*sign(g), so parameters are compared where the sign of g is
    # beyond doubt, i.e. |g_ref| above the gradient's own error bound.
    V, F = shape.vocab, shape.d_ff
    dt = inp["E"].dtype
    master = inp["E"].float().clone()
    E = inp["E"].clone()
    m = torch.zeros(V, F, dtype=torch.float32, device=DEV)
    v = torch.zeros(V, F, dtype=torch.float32, device=DEV)
    L.stem_embed_sparse_adamw(ctx, eg["uniq_ids"], eg["n_uniq"], eg["dE_rows"], E,
                              master if dt == torch.bfloat16 else None, m, v, step=1, **Hn.ADAMW)
    L.stem_sync_status(ctx)
    p_ref, m_ref, v_ref = O.sparse_adamw(oeg["uniq_ids"], oeg["dE_rows"], inputs.to_f64(inp["E"]),
                                         np.zeros((V, F)), np.zeros((V, F)), step=1, **Hn.ADAMW)
    p_gpu = (master if dt == torch.bfloat16 else E).cpu().numpy()
    assert Hn.max_rel(m.cpu().numpy(), m_ref) <= tol
    assert Hn.max_rel(v.cpu().numpy(), v_ref) <= 2 * tol
    uniq = oeg["uniq_ids"]
    sure = np.abs(oeg["dE_rows"]) > 2 * tol * np.abs(oeg["dE_rows"]).max()
    assert sure.any()
    diff = np.abs(p_gpu[uniq] - p_ref[uniq])[sure].max() / np.abs(p_ref).max()
    assert diff <= 1e-5, diff
    untouched = np.setdiff1d(np.arange(V), uniq)
    np.testing.assert_array_equal(p_gpu[untouched], inp["E"].float().cpu().numpy()[untouched])
    ut = torch.from_numpy(untouched).to(DEV)
    assert not m[ut].any() and not v[ut].any()
    if dt == torch.bfloat16:
        np.testing.assert_array_equal(E[ut].cpu().view(torch.int16).numpy(), inp["E"][ut].cpu().view(torch.int16).numpy())
    ctx.close()
    return errs


def test_c1_tiny_fp32_full_pipeline():
    s = inputs.SHAPES["C1"]
    errs = _pipeline_case(s, s.tokens, seed=1)
    print("C1 errors", errs)


@pytest.mark.parametrize("T", [1, 63, 200])
def test_fp32_ragged_token_counts(T):
    s = inputs.StemShape("f32-ragged", 72, 132, 301, 1, T, "f32")
    _pipeline_case(s, T, seed=2)


@pytest.mark.parametrize("T,d,F", [(600, 192, 576), (257, 64, 64), (1, 128, 320), (1100, 512, 256), (2100, 128, 320),
                                   (600, 1088, 1152)])
def test_bf16_several_tiles_and_ragged_tails(T, d, F):
    # 256-wide tiles: these sizes give full tiles plus a ragged last tile in every dimension; the
    # weight-gradient products of the 4th and 5th are cut along K (2 slices; 4 slices of 9, 9, 9, 6 K tiles);
    # the last has 17 and 18 K tiles in its forward and activation-gradient products, enough for the
    # workgroups to start their K loops at different K tiles (rotation per XCD) and wrap around
    s = inputs.StemShape("bf16-ragged", d, F, 1000, 1, T, "bf16")
    _pipeline_case(s, T, seed=3)


def test_bf16_backward_recomputes_h_when_not_saved():
    s = inputs.StemShape("bf16-noH", 128, 384, 500, 1, 300, "bf16")
    _pipeline_case(s, 300, seed=4, save_H=False)


def test_bf16_all_tokens_same_id_and_all_distinct():
    s = inputs.StemShape("bf16-ids", 64, 128, 700, 1, 520, "bf16")
    _pipeline_case(s, 520, seed=5, ids=np.full(520, 699, np.int32))
    _pipeline_case(s, 520, seed=6, ids=np.random.default_rng(0).permutation(700)[:520].astype(np.int32))


@pytest.mark.parametrize("T,d,F", [(1, 64, 64), (37, 192, 320), (128, 256, 576), (129, 128, 1024), (256, 192, 4096),
                                   (300, 64, 2112), (512, 128, 640), (513, 128, 640)])
def test_bf16_few_row_forward(T, d, F):
    """Decode-sized calls take the 128x64-tile kernel (the down product split along K when d_ff is
    long: 2 slices at F=1024, 8 at 4096, 4 uneven ones at 2112); T=513 is the first size on the
    256x256-tile kernel again.  Forward only, with and without the saved G and H."""
    s = inputs.StemShape("bf16-few-rows", d, F, 500, 1, T, "bf16")
    inp = inputs.layer_inputs(s, seed=7, device=DEV, tokens=T)
    ctx = Hn.make_ctx(s, T)
    dt = inp["x"].dtype
    y = torch.empty(T, d, dtype=dt, device=DEV)
    y2 = torch.empty(T, d, dtype=dt, device=DEV)
    G = torch.empty(T, F, dtype=dt, device=DEV)
    H = torch.empty(T, F, dtype=dt, device=DEV)
    L.stem_ffn_forward(ctx, inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], inp["E"], y, G, H)
    L.stem_ffn_forward(ctx, inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], inp["E"], y2)
    L.stem_sync_status(ctx)
    f64 = {k: inputs.to_f64(v) for k, v in inp.items() if k != "ids"}
    ref, fw = O.ffn_forward(f64["x"], inp["ids"].cpu().numpy(), f64["W_gate"], f64["W_down"], f64["E"])
    errs = {"y": Hn.max_rel(y.float().cpu(), ref), "G": Hn.max_rel(G.float().cpu(), fw["g"]),
            "H": Hn.max_rel(H.float().cpu(), fw["h"])}
    assert all(v <= Hn.TOL["bf16"] for v in errs.values()), errs
    assert torch.equal(y, y2)
    ctx.close()


@pytest.mark.parametrize("with_table", [False, True])
@pytest.mark.parametrize("T,d,F", [(700, 192, 576), (1100, 128, 320), (300, 256, 256)])
def test_bf16_dense_swiglu_and_additive_variant(T, d, F, with_table):
    """The layers the STEM layer is compared with, through the same GEMM kernels: up projection,
    epilogues that multiply SiLU(G) by Up or Up + E[ids], dx over the concatenated K range."""
    V = 300
    s = inputs.StemShape("up-variants", d, F, V, 1, T, "bf16")
    inp = inputs.layer_inputs(s, seed=17, device=DEV, tokens=T)
    Wu = inputs.normal((F, d), 0.02, 18, torch.bfloat16, DEV)
    E = inp["E"] if with_table else None
    ids = inp["ids"] if with_table else None
    ctx = Hn.make_ctx(s, T, reserve=L.STEM_RESERVE_UP)
    bf = torch.bfloat16
    y = torch.empty(T, d, dtype=bf, device=DEV)
    G, Up, H, dV = (torch.empty(T, F, dtype=bf, device=DEV) for _ in range(4))
    dx = torch.empty(T, d, dtype=bf, device=DEV)
    dWg, dWu = (torch.empty(F, d, dtype=torch.float32, device=DEV) for _ in range(2))
    dWd = torch.empty(d, F, dtype=torch.float32, device=DEV)
    L.stem_ffn_up_forward(ctx, inp["x"], ids, inp["W_gate"], Wu, inp["W_down"], E, y, G, Up, H)
    L.stem_ffn_up_backward(ctx, inp["dy"], inp["x"], ids, inp["W_gate"], Wu, inp["W_down"], E, G, Up, H, dx, dWg, dWu,
                           dWd, dV)
    y2 = torch.empty_like(y)
    L.stem_ffn_up_forward(ctx, inp["x"], ids, inp["W_gate"], Wu, inp["W_down"], E, y2)   # nothing saved
    L.stem_sync_status(ctx)
    f64 = {k: inputs.to_f64(v) for k, v in inp.items() if k != "ids"}
    ids_np = inp["ids"].cpu().numpy()
    E64 = f64["E"] if with_table else None
    ref, fw = O.up_forward(f64["x"], ids_np, f64["W_gate"], inputs.to_f64(Wu), f64["W_down"], E64)
    bw = O.up_backward(f64["dy"], f64["x"], ids_np, f64["W_gate"], inputs.to_f64(Wu), f64["W_down"], E64)
    errs = {"y": Hn.max_rel(y.float().cpu(), ref), "G": Hn.max_rel(G.float().cpu(), fw["g"]),
            "Up": Hn.max_rel(Up.float().cpu(), fw["up"]), "H": Hn.max_rel(H.float().cpu(), fw["h"]),
            "dx": Hn.max_rel(dx.float().cpu(), bw["dx"]), "dV": Hn.max_rel(dV.float().cpu(), bw["dV"]),
            "dW_gate": Hn.max_rel(dWg.cpu(), bw["dW_gate"]), "dW_up": Hn.max_rel(dWu.cpu(), bw["dW_up"]),
            "dW_down": Hn.max_rel(dWd.cpu(), bw["dW_down"])}
    bad = {k: v for k, v in errs.items() if not v <= Hn.TOL["bf16"]}
    assert not bad, (bad, errs)
    assert torch.equal(y, y2)
    if with_table:   # the table's gradient comes from dV exactly as it comes from dU in the STEM layer
        eg = Hn.hip_embed_grad(ctx, inp["ids"], dV, V)
        U = Hn.check_integers(eg, ids_np)
        assert Hn.max_rel(eg["dE_rows"][:U].cpu(), O.embed_grad(ids_np, bw["dV"])["dE_rows"]) <= Hn.TOL["bf16"]
    ctx.close()


@pytest.mark.parametrize("T,V", [(1, 1), (2, 2), (64, 5), (4096, 50304), (4097, 128256), (16384, 128256),
                                 (65536, 128256), (70001, 64), (5000, (1 << 20) + 3), (3000, 2 ** 31 - 1)])
def test_sort_unique_offsets_bit_exact(T, V):
    if V < 1 << 24:
        ids = inputs.zipf_ids(T, V, seed=T + V)
    else:   # the largest table an int32 id can address: 31 key bits, both ends of the range, repeated ids
        rng = np.random.default_rng(T)
        ids = rng.integers(0, V, T).astype(np.int32)
        ids[[0, 7, T - 1]] = V - 1
        ids[[1, 8, T - 2]] = 0
        ids[100:200] = ids[300:400]
    s = inputs.StemShape("ints", 64, 64, V, 1, T, "bf16")
    ctx = Hn.make_ctx(s, T)
    eg = Hn.hip_embed_grad(ctx, torch.from_numpy(ids).to(DEV), None, V, with_rows=False)
    L.stem_sync_status(ctx)
    Hn.check_integers(eg, ids)
    ctx.close()


def test_segmented_sum_is_bit_reproducible_and_conserves_column_sums():
    s = inputs.StemShape("det", 64, 2112, 3000, 1, 9000, "bf16")
    ids = torch.from_numpy(inputs.zipf_ids(9000, 3000, seed=9)).to(DEV)
    dU = inputs.normal((9000, 2112), 1.0, 10, torch.bfloat16, DEV)
    ctx = Hn.make_ctx(s, 9000)
    a = Hn.hip_embed_grad(ctx, ids, dU, 3000)
    b = Hn.hip_embed_grad(ctx, ids, dU, 3000)
    U = int(a["n_uniq"].item())
    assert torch.equal(a["dE_rows"][:U], b["dE_rows"][:U])
    ref = O.embed_grad(ids.cpu().numpy(), inputs.to_f64(dU))
    assert Hn.max_rel(a["dE_rows"][:U].cpu(), ref["dE_rows"]) <= 1e-5
    col = a["dE_rows"][:U].double().sum(0).cpu().numpy()
    assert Hn.max_rel(col, inputs.to_f64(dU).sum(0)) <= 1e-5
    ctx.close()


@pytest.mark.parametrize("T", [300, 700])   # the few-row and the 256x256-tile forward kernels
def test_bf16_saturated_gate_activations_stay_finite(T):
    """Pre-activations far beyond the range where exp() overflows in fp32 (|g| up to ~200): SiLU and
    its derivative must come out as their limits (0 or g, 0 or 1), never NaN or inf."""
    s = inputs.StemShape("saturated", 192, 320, 400, 1, T, "bf16")
    inp = inputs.layer_inputs(s, seed=19, device=DEV, tokens=T)
    inp["x"] = (inp["x"].float() * 150.0).to(torch.bfloat16)
    ctx = Hn.make_ctx(s, T)
    out = Hn.hip_forward_backward(ctx, inp)
    L.stem_sync_status(ctx)
    f64 = {k: inputs.to_f64(v) for k, v in inp.items() if k != "ids"}
    ids = inp["ids"].cpu().numpy()
    y, fw = O.ffn_forward(f64["x"], ids, f64["W_gate"], f64["W_down"], f64["E"])
    bw = O.ffn_backward(f64["dy"], f64["x"], ids, f64["W_gate"], f64["W_down"], f64["E"])
    assert np.abs(fw["g"]).max() > 120.0          # the case is what it claims to be
    for k in ("y", "G", "H", "dx", "dU", "dW_gate", "dW_down"):
        assert bool(torch.isfinite(out[k].float()).all()), k
    errs = {"y": Hn.max_rel(out["y"].float().cpu(), y), "H": Hn.max_rel(out["H"].float().cpu(), fw["h"]),
            "dx": Hn.max_rel(out["dx"].float().cpu(), bw["dx"]), "dU": Hn.max_rel(out["dU"].float().cpu(), bw["dU"]),
            "dW_gate": Hn.max_rel(out["dW_gate"].cpu(), bw["dW_gate"])}
    assert all(v <= Hn.TOL["bf16"] for v in errs.values()), errs
    ctx.close()


def test_whole_backward_is_bit_reproducible():
    s = inputs.StemShape("det2", 128, 256, 400, 1, 700, "bf16")
    inp = inputs.layer_inputs(s, 11, device=DEV, tokens=700)
    ctx = Hn.make_ctx(s, 700)
    a = Hn.hip_forward_backward(ctx, inp)
    b = Hn.hip_forward_backward(ctx, inp)
    for k in ("y", "dx", "dW_gate", "dW_down", "dU"):
        assert torch.equal(a[k], b[k]), k
    ctx.close()


@pytest.mark.parametrize("T", [90, 1100])   # 1100 tokens: the K-sliced weight-gradient path
def test_weight_gradient_accumulate_flag(T):
    s = inputs.StemShape("acc", 64, 128, 100, 1, T, "bf16")
    inp = inputs.layer_inputs(s, 12, device=DEV, tokens=T)
    ctx = Hn.make_ctx(s, T)
    out = Hn.hip_forward_backward(ctx, inp)
    dWg = out["dW_gate"].clone()
    dWd = out["dW_down"].clone()
    L.stem_ffn_backward(ctx, inp["dy"], inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], inp["E"], out["G"],
                        out["H"], None, dWg, dWd, out["dU"], accumulate=True)
    torch.cuda.synchronize()
    assert torch.equal(dWg, out["dW_gate"] * 2) and torch.equal(dWd, out["dW_down"] * 2)
    ctx.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_knowledge_edit_row_operations(dtype):
    """One-to-one, left-padded, copied and averaged replacement of a source entity's rows: copied
    rows bit for bit, the mean within one rounding of the table's dtype; backup restores the table."""
    V, F = 200, 320
    s = inputs.StemShape("edit", 64, F, V, 1, 8, dtype)
    dt = inputs.torch_dtype(dtype)
    ctx = Hn.make_ctx(s, 8, reserve=L.STEM_RESERVE_EDIT)
    E0 = inputs.normal((V, F), 0.02, 51, dt, DEV)
    E64 = inputs.to_f64(E0)
    rnd = O.bf16_round if dtype == "bf16" else (lambda a: a.astype(np.float32).astype(np.float64))
    cases = [([3, 7, 9], [7, 5, 3], L.STEM_EDIT_REPLACE, O.EDIT_REPLACE),        # overlapping: 3 <-> 7 and 9 <- 3
             ([3, 7, 8, 1], [7, 5], L.STEM_EDIT_PAD_LEFT, O.EDIT_PAD_LEFT),
             ([3, 7, 8, 1, 6], [7, 5], L.STEM_EDIT_COPY, O.EDIT_COPY),
             ([3, 7, 8, 1, 6, 2, 0], [9, 5, 11], L.STEM_EDIT_COPY, O.EDIT_COPY),
             ([3, 7], [5, 6, 11, 150, 199], L.STEM_EDIT_AVERAGE, O.EDIT_AVERAGE),
             ([4], [4], L.STEM_EDIT_AVERAGE, O.EDIT_AVERAGE)]
    for src, tgt, mode, omode in cases:
        E = E0.clone()
        backup = torch.empty(len(src), F, dtype=dt, device=DEV)
        L.stem_edit_rows(ctx, E, src, tgt, mode, pad_id=13, backup=backup)
        torch.cuda.synchronize()
        want, want_backup = O.edit_rows(E64, src, tgt, omode, pad_id=13, round_row=rnd)
        got = inputs.to_f64(E)
        np.testing.assert_array_equal(inputs.to_f64(backup), want_backup)
        if omode == O.EDIT_AVERAGE:
            ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -22
            assert np.abs(got - want).max() <= ulp * np.abs(want).max()
            rest = np.setdiff1d(np.arange(V), src)
            np.testing.assert_array_equal(got[rest], E64[rest])
        else:
            np.testing.assert_array_equal(got, want)
        E[torch.tensor(src, device=DEV)] = backup          # undo
        assert torch.equal(E.view(torch.int16 if dtype == "bf16" else torch.int32),
                           E0.view(torch.int16 if dtype == "bf16" else torch.int32))
    E = E0.clone()
    for bad, status in ((([1, 2], [3, 4, 5], L.STEM_EDIT_COPY), L.STEM_ERR_SHAPE),
                        (([1, 2], [3], L.STEM_EDIT_REPLACE), L.STEM_ERR_SHAPE),
                        (([1, V], [3, 4], L.STEM_EDIT_REPLACE), L.STEM_ERR_ID_RANGE),
                        (([1, 2], [3, -1], L.STEM_EDIT_REPLACE), L.STEM_ERR_ID_RANGE),
                        (([1], [2], 9), L.STEM_ERR_INVALID_ARG),
                        ((list(range(65)), [2], L.STEM_EDIT_AVERAGE), L.STEM_ERR_SHAPE)):
        with pytest.raises(L.StemError) as e:
            L.stem_edit_rows(ctx, E, *bad)
        assert e.value.status == status
    torch.cuda.synchronize()
    assert torch.equal(E, E0)   # a rejected call changes nothing
    ctx.close()


def test_edge_cases_and_error_reporting():
    s = inputs.SHAPES["C1"]
    inp = inputs.layer_inputs(s, 13, device=DEV)
    ctx = Hn.make_ctx(s, s.tokens)
    T, d, F = s.tokens, s.d_model, s.d_ff
    y = torch.full((T, d), 7.0, device=DEV)
    # T = 0 is a no-op
    L.stem_ffn_forward(ctx, inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], inp["E"], y, T=0)
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
    eg = Hn.hip_embed_grad(ctx, inp["ids"][:0], None, s.vocab, with_rows=False)
    assert int(eg["n_uniq"].item()) == 0 and int(eg["seg_offsets"][0].item()) == 0
    # T beyond the context's capacity
    with pytest.raises(L.StemError) as e:
        L.stem_ffn_forward(ctx, inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], inp["E"], y, T=T + 1)
    assert e.value.status == L.STEM_ERR_SHAPE
    # null pointer
    with pytest.raises(L.StemError) as e:
        L.stem_ffn_forward(ctx, inp["x"], inp["ids"], None, inp["W_down"], inp["E"], y)
    assert e.value.status == L.STEM_ERR_INVALID_ARG
    # misaligned pointer
    with pytest.raises(L.StemError) as e:
        L.stem_ffn_forward(ctx, inp["x"].flatten()[1:], inp["ids"], inp["W_gate"], inp["W_down"], inp["E"], y, T=1)
    assert e.value.status == L.STEM_ERR_INVALID_ARG
    # id out of range: no fault, sticky flag reported at the next synchronising status call
    bad = inp["ids"].clone()
    bad[5] = s.vocab
    bad[9] = -3
    L.stem_ffn_forward(ctx, inp["x"], bad, inp["W_gate"], inp["W_down"], inp["E"], y)
    with pytest.raises(L.StemError) as e:
        L.stem_sync_status(ctx)
    assert e.value.status == L.STEM_ERR_ID_RANGE
    L.stem_sync_status(ctx)  # flag was cleared
    # scratch of the optional entry points is reserved explicitly; without it they refuse to run
    cb = L.stem_create(64, 64, 100, L.STEM_BF16, 8, 0)
    z16 = torch.zeros(8, 64, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(L.StemError) as e:
        L.stem_ffn_up_forward(cb, z16, None, z16[:64].repeat(8, 1), z16[:64].repeat(8, 1), z16[:64].repeat(8, 1), None, z16.clone())
    assert e.value.status == L.STEM_ERR_WORKSPACE and "STEM_RESERVE_UP" in str(e.value)
    with pytest.raises(L.StemError) as e:
        L.stem_edit_rows(cb, torch.zeros(100, 64, dtype=torch.bfloat16, device=DEV), [1], [2], L.STEM_EDIT_REPLACE)
    assert e.value.status == L.STEM_ERR_WORKSPACE
    with pytest.raises(L.StemError) as e:
        L.stem_reserve(cb, 64)
    assert e.value.status == L.STEM_ERR_INVALID_ARG
    with pytest.raises(L.StemError) as e:
        L.stem_set_prefetch_mode(cb, 5)
    assert e.value.status == L.STEM_ERR_INVALID_ARG
    cb.close()
    # unsupported widths are refused at creation
    with pytest.raises(L.StemError) as e:
        L.stem_create(100, 256, 10, L.STEM_BF16, 8, 0)
    assert e.value.status == L.STEM_ERR_UNSUPPORTED
    ctx.close()


@pytest.mark.parametrize("dtype,T,d,F", [("bf16", 300, 128, 1024), ("bf16", 256, 192, 320), ("bf16", 700, 192, 576),
                                         ("f32", 100, 72, 132)])
def test_forward_with_residual_out_of_place_and_in_place(dtype, T, d, F):
    """y = residual + layer(x), the sum taken in the down product's epilogue: the few-row kernel with and
    without a K split (T = 300, 256), the 256x256-tile kernel (T = 700), the fp32 path; with a separate
    residual and output, and in place on the layer's own input (a residual stream)."""
    s = inputs.StemShape("residual", d, F, 500, 1, T, dtype)
    inp = inputs.layer_inputs(s, seed=18, device=DEV, tokens=T)
    dt = inp["x"].dtype
    ctx = Hn.make_ctx(s, T)
    f64 = {k: inputs.to_f64(v) for k, v in inp.items() if k != "ids"}
    ids = inp["ids"].cpu().numpy()
    layer, _ = O.ffn_forward(f64["x"], ids, f64["W_gate"], f64["W_down"], f64["E"])
    # a residual of the layer output's own magnitude, so that neither term can hide an error in the other
    res = inputs.normal((T, d), float(np.abs(layer).max()), 19, dt, DEV)
    y = torch.empty(T, d, dtype=dt, device=DEV)
    L.stem_ffn_forward_residual(ctx, inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], inp["E"], res, y)
    L.stem_sync_status(ctx)
    assert Hn.max_rel(y.float().cpu(), inputs.to_f64(res) + layer) <= Hn.TOL[dtype]
    assert Hn.max_rel(y.float().cpu().numpy().astype(np.float64) - inputs.to_f64(res), layer) <= 4 * Hn.TOL[dtype]
    xs = inp["x"].clone()
    L.stem_ffn_forward_residual(ctx, xs, inp["ids"], inp["W_gate"], inp["W_down"], inp["E"], xs, xs)
    L.stem_sync_status(ctx)
    assert Hn.max_rel(xs.float().cpu(), f64["x"] + layer) <= Hn.TOL[dtype]
    with pytest.raises(L.StemError) as e:
        L.stem_ffn_forward_residual(ctx, inp["x"], inp["ids"], inp["W_gate"], inp["W_down"], inp["E"], None, y)
    assert e.value.status == L.STEM_ERR_INVALID_ARG
    ctx.close()


def test_table_gradient_in_two_halves_on_two_streams():
    """The integer half of the table gradient on a second stream, the row sums later on the main one
    (stem_embed_grad with dU = NULL, then stem_embed_grad_presorted): same bits as the single call."""
    T, V, F = 5000, 3000, 320
    s = inputs.StemShape("two-halves", 64, F, V, 1, T, "bf16")
    ctx = Hn.make_ctx(s, T)
    ids_np = inputs.zipf_ids(T, V, seed=20)
    ids = torch.from_numpy(ids_np).to(DEV)
    dU = inputs.normal((T, F), 1.0, 21, torch.bfloat16, DEV)
    want = Hn.hip_embed_grad(ctx, ids, dU, V)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    got = Hn.hip_embed_grad(ctx, ids, None, V, with_rows=False, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    rows = torch.full((min(T, V), F), 7.0, dtype=torch.float32, device=DEV)
    L.stem_embed_grad_presorted(ctx, dU, got["perm"], got["seg_offsets"], rows)
    L.stem_sync_status(ctx)
    U = Hn.check_integers(got, ids_np)
    assert torch.equal(rows[:U], want["dE_rows"][:U]) and bool((rows[U:] == 7.0).all())
    with pytest.raises(L.StemError) as e:      # the context's run index belongs to a call with T tokens
        L.stem_embed_grad_presorted(ctx, dU[:100], got["perm"], got["seg_offsets"], rows)
    assert e.value.status == L.STEM_ERR_INVALID_ARG
    ctx.close()


def _expect_id_range(ctx):
    with pytest.raises(L.StemError) as e:
        L.stem_sync_status(ctx)
    assert e.value.status == L.STEM_ERR_ID_RANGE
    L.stem_sync_status(ctx)   # the flag was cleared


@pytest.mark.parametrize("T,d,F", [(700, 1088, 320), (300, 128, 320)])
def test_bf16_out_of_range_ids_are_clamped_and_reported(T, d, F):
    """Ids outside the table on the bf16 paths: the fused epilogues of the 256x256-tile products (T = 700;
    d_model 1088 also reaches the early touch of the gathered rows, d_ff 320 = 64 mod 128 its narrow last
    column block) and the few-row kernel (T = 300).  No access leaves the table (an id below zero reads
    row 0, one beyond the end the last row), the sticky flag is reported once, every output is finite,
    and the rows of tokens with valid ids match the oracle."""
    V = 257
    s = inputs.StemShape("bf16-bad-ids", d, F, V, 1, T, "bf16")
    inp = inputs.layer_inputs(s, seed=15, device=DEV, tokens=T)
    ids_good = inp["ids"].cpu().numpy()
    bad_at = np.array([0, 5, 63, 64, 255, 256, T - 1])
    bad_val = np.array([V, -3, 2 ** 31 - 1, -2 ** 31, V + 7, -1, V])
    ids_bad = ids_good.copy()
    ids_bad[bad_at] = bad_val
    inp_bad = dict(inp, ids=torch.from_numpy(ids_bad.astype(np.int32)).to(DEV))
    ctx = Hn.make_ctx(s, T)
    dt = inp["x"].dtype
    good = np.setdiff1d(np.arange(T), bad_at)
    f64 = {k: inputs.to_f64(v) for k, v in inp.items() if k != "ids"}
    ref, fw = O.ffn_forward(f64["x"], ids_good, f64["W_gate"], f64["W_down"], f64["E"])
    tol = Hn.TOL["bf16"]
    if T <= 512:   # few-row kernel: forward only
        y = torch.empty(T, d, dtype=dt, device=DEV)
        G, H = (torch.empty(T, F, dtype=dt, device=DEV) for _ in range(2))
        L.stem_ffn_forward(ctx, inp["x"], inp_bad["ids"], inp["W_gate"], inp["W_down"], inp["E"], y, G, H)
        _expect_id_range(ctx)
        for t in (y, G, H):
            assert bool(torch.isfinite(t.float()).all())
        assert Hn.max_rel(y.float().cpu().numpy()[good], ref[good]) <= tol
        assert Hn.max_rel(H.float().cpu().numpy()[good], fw["h"][good]) <= tol
    else:
        # the forward call's flag is collected before the backward call: that call would report it
        # itself (and do nothing else) if the forward kernels happened to have run by then
        out = Hn.hip_forward_backward(ctx, inp_bad, after_forward=lambda: _expect_id_range(ctx))
        _expect_id_range(ctx)   # the fused dH epilogue gathers the same rows
        for t in out.values():
            assert bool(torch.isfinite(t.float()).all())
        bw = O.ffn_backward(f64["dy"], f64["x"], ids_good, f64["W_gate"], f64["W_down"], f64["E"])
        for k, want in (("y", ref), ("H", fw["h"]), ("G", fw["g"]), ("dx", bw["dx"]), ("dU", bw["dU"])):
            assert Hn.max_rel(out[k].float().cpu().numpy()[good], want[good]) <= tol, k
        # the clamp itself: the whole result equals the oracle's on the clamped ids
        ids_cl = np.clip(ids_bad.astype(np.int64), 0, V - 1)
        y_cl, _ = O.ffn_forward(f64["x"], ids_cl, f64["W_gate"], f64["W_down"], f64["E"])
        bw_cl = O.ffn_backward(f64["dy"], f64["x"], ids_cl, f64["W_gate"], f64["W_down"], f64["E"])
        assert Hn.max_rel(out["y"].float().cpu(), y_cl) <= tol
        assert Hn.max_rel(out["dW_gate"].cpu(), bw_cl["dW_gate"]) <= tol
        assert Hn.max_rel(out["dW_down"].cpu(), bw_cl["dW_down"]) <= tol
    ctx.close()


@pytest.mark.parametrize("T", [16384, 20000])
def test_sort_paths_clamp_and_report_out_of_range_ids(T):
    """The one-workgroup sort (T = 16384) and the multi-kernel sort (T = 20000) with ids outside the
    table: the flag is raised, and sort, unique, offsets and the row sums are those of the clamped ids."""
    V, F = 5000, 64
    s = inputs.StemShape("bf16-bad-sort", 64, F, V, 1, T, "bf16")
    ids = inputs.zipf_ids(T, V, seed=16).astype(np.int64)
    ids[[0, 7, 1023, 1024, T // 2, T - 1]] = [V, -1, 2 ** 31 - 1, -2 ** 31, V + 100, -77]
    ids32 = ids.astype(np.int32)
    ctx = Hn.make_ctx(s, T)
    dU = inputs.normal((T, F), 1.0, 17, torch.bfloat16, DEV)
    eg = Hn.hip_embed_grad(ctx, torch.from_numpy(ids32).to(DEV), dU, V)
    _expect_id_range(ctx)
    ids_cl = np.clip(ids, 0, V - 1).astype(np.int32)
    U = Hn.check_integers(eg, ids_cl)
    oeg = O.embed_grad(ids_cl, inputs.to_f64(dU))
    assert bool(torch.isfinite(eg["dE_rows"][:U]).all())
    assert Hn.max_rel(eg["dE_rows"][:U].cpu(), oeg["dE_rows"]) <= 1e-5
    ctx.close()


def test_id_at_last_row_of_table():
    s = inputs.StemShape("lastrow", 64, 64, 33, 1, 40, "bf16")
    ids = np.full(40, 32, np.int32)
    ids[::3] = 0
    _pipeline_case(s, 40, seed=14, ids=ids)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sparse_adamw_three_steps_on_shared_gradients(dtype):
    # Both sides receive the same seeded gradient rows and row list, so the comparison is tight.
    V, F, T = 777, 320, 400
    s = inputs.StemShape("adamw", 64, F, V, 1, T, dtype)
    ctx = Hn.make_ctx(s, T)
    dt = inputs.torch_dtype(dtype)
    E = inputs.normal((V, F), 0.02, 30, dt, DEV)
    E0 = E.clone()
    master = E.float().clone()
    m = torch.zeros(V, F, dtype=torch.float32, device=DEV)
    v = torch.zeros(V, F, dtype=torch.float32, device=DEV)
    p_ref, m_ref, v_ref = inputs.to_f64(E), np.zeros((V, F)), np.zeros((V, F))
    for step in (1, 2, 3):
        uniq = np.unique(inputs.zipf_ids(T, V, seed=40 + step)).astype(np.int32)
        U = len(uniq)
        g = inputs.normal((T, F), 10.0 ** (step - 3), 50 + step, torch.float32, DEV)
        g[0, :7] = 0.0  # exact zeros: the update must still be finite
        d_uniq = torch.zeros(T, dtype=torch.int32, device=DEV)
        d_uniq[:U] = torch.from_numpy(uniq).to(DEV)
        n_uniq = torch.tensor([U], dtype=torch.int32, device=DEV)
        L.stem_embed_sparse_adamw(ctx, d_uniq, n_uniq, g, E, master if dtype == "bf16" else None, m, v,
                                  step=step, **Hn.ADAMW)
        p_ref, m_ref, v_ref = O.sparse_adamw(uniq, g[:U].cpu().numpy(), p_ref, m_ref, v_ref, step=step, **Hn.ADAMW)
    L.stem_sync_status(ctx)
    p_gpu = (master if dtype == "bf16" else E).cpu().numpy()
    assert np.isfinite(p_gpu).all()
    assert Hn.max_rel(p_gpu, p_ref) <= 1e-5
    assert Hn.max_rel(m.cpu().numpy(), m_ref) <= 1e-5
    assert Hn.max_rel(v.cpu().numpy(), v_ref) <= 1e-5
    if dtype == "bf16":
        # working copy = master rounded to nearest-even bf16 on touched rows, untouched rows keep their bits
        want = O.bf16_round(p_gpu)
        touched = np.zeros(V, bool)
        for step in (1, 2, 3):
            touched[np.unique(inputs.zipf_ids(T, V, seed=40 + step))] = True
        got = E.float().cpu().numpy().astype(np.float64)
        np.testing.assert_array_equal(got[touched], want[touched])
        np.testing.assert_array_equal(got[~touched], E0.float().cpu().numpy()[~touched])
    ctx.close()


def test_on_box_peak_measurements_run_and_order_as_expected():
    """stem_measure_peak: every kind returns a positive rate; the MFMA loop on all-zero operands is not
    slower than on unit-normal ones (the chip sustains a lower clock the more operand bits toggle)."""
    a = torch.zeros(1 << 24, dtype=torch.uint8, device=DEV)
    b = torch.empty_like(a)
    assert L.stem_measure_peak(L.STEM_PEAK_MFMA_BF16, a, None, repeats=1) > 100.0
    assert L.stem_measure_peak(L.STEM_PEAK_HBM_READ, a, b, repeats=2) > 100.0
    assert L.stem_measure_peak(L.STEM_PEAK_HBM_COPY, a, b, repeats=2) > 100.0
    sink = torch.zeros(64, device=DEV)
    zeros = torch.zeros(1 << 16, dtype=torch.bfloat16, device=DEV)
    normal = inputs.normal((1 << 16,), 1.0, 5, torch.bfloat16, DEV)
    on_zeros = L.stem_measure_peak(L.STEM_PEAK_MFMA_BF16_DATA, zeros, sink, repeats=2)
    on_normal = L.stem_measure_peak(L.STEM_PEAK_MFMA_BF16_DATA, normal, sink, repeats=2)
    assert on_normal > 100.0 and on_zeros >= 0.98 * on_normal, (on_zeros, on_normal)
    with pytest.raises(L.StemError):   # the data loop needs its second buffer
        L.stem_measure_peak(L.STEM_PEAK_MFMA_BF16_DATA, zeros, None, repeats=1)

