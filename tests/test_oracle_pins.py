"""Pins for the CPU oracle: each check compares it with something other than
itself — a one-hot matmul, finite differences, a library routine (torch's SiLU,
linear and AdamW, scipy's expit, numpy's unique), a closed form or brute force.
All CPU, all tiny.
"""
import itertools

import numpy as np
import pytest
import scipy.special
import torch

from oracle import stem_oracle as O
from paper_2601_10639_amd import inputs


def _tiny(seed=0, T=12, d=8, F=16, V=11, scale=0.5):
    rng = np.random.default_rng(seed)
    x = rng.normal(size=(T, d))
    Wg = rng.normal(size=(F, d)) * scale
    Wd = rng.normal(size=(d, F)) * scale
    E = rng.normal(size=(V, F))
    ids = rng.integers(0, V, size=T).astype(np.int32)
    ids[3] = ids[0]  # make sure at least one id repeats
    r = rng.normal(size=(T, d))
    return x, ids, Wg, Wd, E, r


def _onehot(ids, V):
    P = np.zeros((len(ids), V))
    P[np.arange(len(ids)), ids] = 1.0
    return P


# -- elementary --------------------------------------------------------------
def test_sigmoid_matches_scipy_expit():
    z = np.concatenate([np.linspace(-50, 50, 2001), [-800.0, 800.0, 0.0]])
    np.testing.assert_allclose(O.sigmoid(z), scipy.special.expit(z), rtol=1e-15, atol=0)


def test_silu_matches_torch():
    z = np.linspace(-20, 20, 1001)
    ref = torch.nn.functional.silu(torch.from_numpy(z)).numpy()
    np.testing.assert_allclose(O.silu(z), ref, rtol=1e-14, atol=1e-300)


def test_silu_prime_is_derivative_of_silu():
    z = np.linspace(-8, 8, 321)
    h = 1e-5
    fd = (O.silu(z + h) - O.silu(z - h)) / (2 * h)
    np.testing.assert_allclose(O.silu_prime(z), fd, rtol=0, atol=1e-8)
    ref = torch.from_numpy(z).requires_grad_()
    torch.nn.functional.silu(ref).sum().backward()
    np.testing.assert_allclose(O.silu_prime(z), ref.grad.numpy(), rtol=1e-13, atol=1e-15)


# -- gather and forward ------------------------------------------------------
def test_gather_is_onehot_matmul():
    x, ids, Wg, Wd, E, r = _tiny()
    np.testing.assert_array_equal(O.gather_rows(E, ids), _onehot(ids, E.shape[0]) @ E)


def test_gather_rejects_out_of_range():
    _, ids, _, _, E, _ = _tiny()
    bad = ids.copy(); bad[0] = E.shape[0]
    with pytest.raises(IndexError):
        O.gather_rows(E, bad)
    bad[0] = -1
    with pytest.raises(IndexError):
        O.gather_rows(E, bad)


def test_forward_scalar_closed_form():
    # d = F = 1:  y = w_d * (w_g x) * sigmoid(w_g x) * e
    wg, wd, e, x = 0.7, -1.3, 2.5, 0.9
    y, _ = O.ffn_forward([[x]], [0], [[wg]], [[wd]], [[e]])
    z = wg * x
    assert y.shape == (1, 1)
    assert y[0, 0] == pytest.approx(wd * z / (1 + np.exp(-z)) * e, rel=1e-15)


def test_forward_reduces_to_dense_swiglu_on_constant_input():
    # If every token carries the same hidden state c and every table row equals
    # W_up c, the STEM layer is the SwiGLU FFN on c.  The SwiGLU side is written
    # with torch's library routines, not with the oracle.
    rng = np.random.default_rng(3)
    T, d, F, V = 7, 6, 10, 5
    c = rng.normal(size=d)
    Wg, Wu, Wd = rng.normal(size=(F, d)), rng.normal(size=(F, d)), rng.normal(size=(d, F))
    E = np.tile(Wu @ c, (V, 1))
    ids = rng.integers(0, V, size=T)
    x = np.tile(c, (T, 1))
    y, _ = O.ffn_forward(x, ids, Wg, Wd, E)
    tc = torch.from_numpy(c)
    lin = torch.nn.functional.linear
    ref = lin(torch.nn.functional.silu(lin(tc, torch.from_numpy(Wg))) * lin(tc, torch.from_numpy(Wu)),
              torch.from_numpy(Wd)).numpy()
    np.testing.assert_allclose(y, np.tile(ref, (T, 1)), rtol=1e-12, atol=1e-13)
    # and the oracle's own dense SwiGLU agrees with the same library expression
    np.testing.assert_allclose(O.swiglu_forward(x, Wg, Wu, Wd), np.tile(ref, (T, 1)), rtol=1e-12, atol=1e-13)


def test_forward_against_per_token_loops():
    # brute force: scalar loops straight from the layer's equation
    x, ids, Wg, Wd, E, _ = _tiny(seed=5, T=5, d=3, F=4, V=6)
    y, _ = O.ffn_forward(x, ids, Wg, Wd, E)
    for i in range(x.shape[0]):
        h = []
        for f in range(Wg.shape[0]):
            z = sum(Wg[f, k] * x[i, k] for k in range(x.shape[1]))
            h.append(z / (1.0 + np.exp(-z)) * E[ids[i], f])
        for a in range(Wd.shape[0]):
            want = sum(Wd[a, f] * h[f] for f in range(len(h)))
            assert y[i, a] == pytest.approx(want, rel=1e-12, abs=1e-14)


def test_forward_linear_in_table_and_zero_row():
    x, ids, Wg, Wd, E, _ = _tiny(seed=1)
    E2 = np.random.default_rng(9).normal(size=E.shape)
    y1, _ = O.ffn_forward(x, ids, Wg, Wd, E)
    y2, _ = O.ffn_forward(x, ids, Wg, Wd, E2)
    y12, _ = O.ffn_forward(x, ids, Wg, Wd, 2.0 * E - 3.0 * E2)
    np.testing.assert_allclose(y12, 2.0 * y1 - 3.0 * y2, rtol=1e-12, atol=1e-12)
    Ez = E.copy(); Ez[ids[0]] = 0.0
    yz, _ = O.ffn_forward(x, ids, Wg, Wd, Ez)
    assert np.all(yz[ids == ids[0]] == 0.0)
    np.testing.assert_array_equal(yz[ids != ids[0]], y1[ids != ids[0]])


def test_forward_token_permutation_equivariance():
    x, ids, Wg, Wd, E, _ = _tiny(seed=2)
    perm = np.random.default_rng(4).permutation(len(ids))
    y, _ = O.ffn_forward(x, ids, Wg, Wd, E)
    yp, _ = O.ffn_forward(x[perm], ids[perm], Wg, Wd, E)
    np.testing.assert_array_equal(yp, y[perm])


def test_stem_dagger_special_cases():
    # zero up-projection -> the STEM layer; zero table -> the dense SwiGLU FFN
    x, ids, Wg, Wd, E, _ = _tiny(seed=6)
    Wu = np.random.default_rng(7).normal(size=Wg.shape)
    y_stem, _ = O.ffn_forward(x, ids, Wg, Wd, E)
    np.testing.assert_array_equal(O.stem_dagger_forward(x, ids, Wg, np.zeros_like(Wu), Wd, E), y_stem)
    np.testing.assert_array_equal(O.stem_dagger_forward(x, ids, Wg, Wu, Wd, np.zeros_like(E)),
                                  O.swiglu_forward(x, Wg, Wu, Wd))
    both = O.stem_dagger_forward(x, ids, Wg, Wu, Wd, E)
    np.testing.assert_allclose(both, y_stem + O.swiglu_forward(x, Wg, Wu, Wd), rtol=1e-12, atol=1e-12)


# -- backward ----------------------------------------------------------------
def _loss(x, ids, Wg, Wd, E, r):
    y, _ = O.ffn_forward(x, ids, Wg, Wd, E)
    return float((y * r).sum())


@pytest.mark.parametrize("which", ["x", "W_gate", "W_down", "E"])
def test_backward_matches_central_finite_differences(which):
    x, ids, Wg, Wd, E, r = _tiny(seed=11, T=9, d=5, F=7, V=6)
    grads = O.ffn_backward(r, x, ids, Wg, Wd, E)
    eg = O.embed_grad(ids, grads["dU"])
    dE = np.zeros_like(E)
    dE[eg["uniq_ids"]] = eg["dE_rows"]
    analytic = {"x": grads["dx"], "W_gate": grads["dW_gate"], "W_down": grads["dW_down"], "E": dE}[which]
    params = {"x": x, "W_gate": Wg, "W_down": Wd, "E": E}
    target = params[which]
    h = 1e-6
    fd = np.zeros_like(target)
    for idx in itertools.product(*[range(n) for n in target.shape]):
        old = target[idx]
        target[idx] = old + h
        lp = _loss(params["x"], ids, params["W_gate"], params["W_down"], params["E"], r)
        target[idx] = old - h
        lm = _loss(params["x"], ids, params["W_gate"], params["W_down"], params["E"], r)
        target[idx] = old
        fd[idx] = (lp - lm) / (2 * h)
    scale = np.abs(fd).max()
    assert scale > 0
    assert np.abs(analytic - fd).max() / scale < 1e-7


def test_backward_against_torch_autograd():
    x, ids, Wg, Wd, E, r = _tiny(seed=12)
    tx, tWg, tWd, tE = (torch.from_numpy(a.copy()).requires_grad_() for a in (x, Wg, Wd, E))
    u = torch.nn.functional.embedding(torch.from_numpy(ids.astype(np.int64)), tE)
    y = torch.nn.functional.linear(torch.nn.functional.silu(torch.nn.functional.linear(tx, tWg)) * u, tWd)
    (y * torch.from_numpy(r)).sum().backward()
    g = O.ffn_backward(r, x, ids, Wg, Wd, E)
    np.testing.assert_allclose(g["dx"], tx.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(g["dW_gate"], tWg.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(g["dW_down"], tWd.grad.numpy(), rtol=1e-11, atol=1e-12)
    eg = O.embed_grad(ids, g["dU"])
    dE = np.zeros_like(E); dE[eg["uniq_ids"]] = eg["dE_rows"]
    np.testing.assert_allclose(dE, tE.grad.numpy(), rtol=1e-11, atol=1e-12)


# -- embedding gradient ------------------------------------------------------
def test_up_variants_forward_and_backward_against_torch_autograd():
    # dense SwiGLU and the additive variant, written with torch's own silu / linear / embedding
    rng = np.random.default_rng(21)
    T, d, F, V = 9, 5, 7, 6
    x, Wg, Wu, Wd = rng.normal(size=(T, d)), rng.normal(size=(F, d)), rng.normal(size=(F, d)), rng.normal(size=(d, F))
    E, dy = rng.normal(size=(V, F)), rng.normal(size=(T, d))
    ids = rng.integers(0, V, T)
    for table in (None, E):
        tx, tWg, tWu, tWd = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, Wg, Wu, Wd))
        tE = torch.tensor(E, dtype=torch.float64, requires_grad=True)
        v = torch.nn.functional.linear(tx, tWu)
        if table is not None:
            v = v + torch.nn.functional.embedding(torch.tensor(ids), tE)
        y = torch.nn.functional.linear(torch.nn.functional.silu(torch.nn.functional.linear(tx, tWg)) * v, tWd)
        (y * torch.tensor(dy)).sum().backward()
        y_o, _ = O.up_forward(x, ids, Wg, Wu, Wd, table)
        bw = O.up_backward(dy, x, ids, Wg, Wu, Wd, table)
        np.testing.assert_allclose(y_o, y.detach().numpy(), rtol=1e-12, atol=1e-12)
        for name, t in (("dx", tx), ("dW_gate", tWg), ("dW_up", tWu), ("dW_down", tWd)):
            np.testing.assert_allclose(bw[name], t.grad.numpy(), rtol=1e-11, atol=1e-12, err_msg=name)
        if table is not None:   # the table's gradient is the per-row sum of dV
            np.testing.assert_allclose(O.embed_grad(ids, bw["dV"])["dE_rows"],
                                       tE.grad.numpy()[np.unique(ids)], rtol=1e-11, atol=1e-12)


def test_up_variants_reduce_to_the_stem_layer_and_to_each_other():
    rng = np.random.default_rng(22)
    T, d, F, V = 8, 4, 6, 5
    x, Wg, Wu, Wd = rng.normal(size=(T, d)), rng.normal(size=(F, d)), rng.normal(size=(F, d)), rng.normal(size=(d, F))
    E, dy = rng.normal(size=(V, F)), rng.normal(size=(T, d))
    ids = rng.integers(0, V, T)
    # W_up = 0: the STEM layer, forward and every gradient it has
    y0, _ = O.up_forward(x, ids, Wg, np.zeros_like(Wu), Wd, E)
    np.testing.assert_array_equal(y0, O.ffn_forward(x, ids, Wg, Wd, E)[0])
    b0, bs = O.up_backward(dy, x, ids, Wg, np.zeros_like(Wu), Wd, E), O.ffn_backward(dy, x, ids, Wg, Wd, E)
    for a, b in (("dx", "dx"), ("dW_gate", "dW_gate"), ("dW_down", "dW_down"), ("dV", "dU"), ("dG", "dG")):
        np.testing.assert_allclose(b0[a], bs[b], rtol=1e-13, atol=1e-14)
    # all-zero table: the dense FFN; and the published forward functions agree
    y1, _ = O.up_forward(x, ids, Wg, Wu, Wd, np.zeros_like(E))
    np.testing.assert_array_equal(y1, O.up_forward(x, ids, Wg, Wu, Wd, None)[0])
    np.testing.assert_array_equal(y1, O.swiglu_forward(x, Wg, Wu, Wd))
    np.testing.assert_array_equal(O.up_forward(x, ids, Wg, Wu, Wd, E)[0], O.stem_dagger_forward(x, ids, Wg, Wu, Wd, E))
    # one finite difference through W_up (the term the STEM layer does not have)
    h = 1e-6
    Wp, Wm = Wu.copy(), Wu.copy()
    Wp[2, 1] += h
    Wm[2, 1] -= h
    fd = ((O.up_forward(x, ids, Wg, Wp, Wd, E)[0] - O.up_forward(x, ids, Wg, Wm, Wd, E)[0]) * dy).sum() / (2 * h)
    assert abs(fd - O.up_backward(dy, x, ids, Wg, Wu, Wd, E)["dW_up"][2, 1]) < 1e-7


def test_embed_grad_is_onehot_transpose_matmul():
    x, ids, Wg, Wd, E, r = _tiny(seed=13)
    dU = O.ffn_backward(r, x, ids, Wg, Wd, E)["dU"]
    eg = O.embed_grad(ids, dU)
    dense = _onehot(ids, E.shape[0]).T @ dU
    touched = np.zeros(E.shape[0], bool); touched[eg["uniq_ids"]] = True
    np.testing.assert_allclose(eg["dE_rows"], dense[eg["uniq_ids"]], rtol=1e-13, atol=1e-14)
    assert np.all(dense[~touched] == 0.0)
    assert set(eg["uniq_ids"].tolist()) == set(ids.tolist())


def test_embed_grad_all_equal_and_all_distinct():
    rng = np.random.default_rng(14)
    dU = rng.normal(size=(10, 6))
    eg = O.embed_grad(np.full(10, 4, np.int32), dU)
    assert eg["n_uniq"] == 1 and eg["uniq_ids"].tolist() == [4] and eg["seg_offsets"].tolist() == [0, 10]
    np.testing.assert_allclose(eg["dE_rows"][0], dU.sum(axis=0), rtol=1e-14)
    ids = rng.permutation(10).astype(np.int32)
    eg = O.embed_grad(ids, dU)
    assert eg["n_uniq"] == 10 and eg["uniq_ids"].tolist() == list(range(10))
    np.testing.assert_array_equal(eg["dE_rows"], dU[np.argsort(ids)])


def test_sort_and_segments_brute_force_and_invariants():
    rng = np.random.default_rng(15)
    for T, V in [(1, 1), (1, 9), (17, 3), (64, 1000), (200, 7)]:
        ids = rng.integers(0, V, size=T).astype(np.int32)
        s, perm = O.sort_ids(ids)
        want = sorted((int(t), i) for i, t in enumerate(ids))
        assert s.tolist() == [t for t, _ in want]
        assert perm.tolist() == [i for _, i in want]
        assert sorted(perm.tolist()) == list(range(T))
        uniq, offs = O.unique_segments(s)
        assert uniq.tolist() == sorted(set(ids.tolist()))
        assert offs[0] == 0 and offs[-1] == T and np.all(np.diff(offs) > 0)
        counts = np.bincount(ids, minlength=V)
        assert np.diff(offs).tolist() == counts[uniq].tolist()
        for j, t in enumerate(uniq):
            assert np.all(s[offs[j]:offs[j + 1]] == t)
    # empty input
    s, perm = O.sort_ids(np.zeros(0, np.int32))
    uniq, offs = O.unique_segments(s)
    assert s.size == 0 and perm.size == 0 and uniq.size == 0 and offs.tolist() == [0]


def test_embed_grad_column_sum_conservation():
    rng = np.random.default_rng(16)
    ids = inputs.zipf_ids(300, 50, seed=1)
    dU = rng.normal(size=(300, 5))
    eg = O.embed_grad(ids, dU)
    np.testing.assert_allclose(eg["dE_rows"].sum(axis=0), dU.sum(axis=0), rtol=1e-12)


# -- AdamW -------------------------------------------------------------------
HP = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def test_adamw_all_rows_touched_equals_torch_adamw():
    rng = np.random.default_rng(17)
    V, F = 6, 5
    p0 = rng.normal(size=(V, F))
    tp = torch.from_numpy(p0.copy()).requires_grad_()
    opt = torch.optim.AdamW([tp], lr=HP["lr"], betas=(HP["beta1"], HP["beta2"]), eps=HP["eps"],
                            weight_decay=HP["weight_decay"])
    p, m, v = p0, np.zeros((V, F)), np.zeros((V, F))
    for step in range(1, 5):
        g = rng.normal(size=(V, F)) * (10.0 ** rng.integers(-3, 2))
        tp.grad = torch.from_numpy(g.copy())
        opt.step()
        p, m, v = O.sparse_adamw(np.arange(V), g, p, m, v, step=step, **HP)
        np.testing.assert_allclose(p, tp.detach().numpy(), rtol=1e-12, atol=1e-15)
        st = opt.state[tp]
        np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-18)


def test_adamw_step_one_closed_form_and_untouched_rows():
    rng = np.random.default_rng(18)
    V, F = 9, 4
    p0 = rng.normal(size=(V, F)); m0 = np.zeros((V, F)); v0 = np.zeros((V, F))
    uniq = np.array([1, 4, 7], np.int32)
    g = rng.normal(size=(3, F))
    p, m, v = O.sparse_adamw(uniq, g, p0, m0, v0, step=1, **HP)
    want = p0[uniq] * (1 - HP["lr"] * HP["weight_decay"]) - HP["lr"] * g / (np.abs(g) + HP["eps"])
    np.testing.assert_allclose(p[uniq], want, rtol=1e-12)
    rest = np.setdiff1d(np.arange(V), uniq)
    np.testing.assert_array_equal(p[rest], p0[rest])
    assert np.all(m[rest] == 0) and np.all(v[rest] == 0)
    # a touched row with zero gradient still decays its weight and moments
    m1 = rng.normal(size=(V, F)); v1 = rng.random(size=(V, F))
    p2, m2, v2 = O.sparse_adamw(np.array([2]), np.zeros((1, F)), p0, m1, v1, step=3, **HP)
    np.testing.assert_allclose(m2[2], HP["beta1"] * m1[2], rtol=1e-15)
    np.testing.assert_allclose(v2[2], HP["beta2"] * v1[2], rtol=1e-15)
    assert not np.array_equal(p2[2], p0[2])


def test_adamw_rows_form_equals_table_form():
    rng = np.random.default_rng(19)
    V, F = 8, 3
    p0, m0, v0 = rng.normal(size=(V, F)), rng.normal(size=(V, F)), rng.random(size=(V, F))
    uniq = np.array([0, 3, 6]); g = rng.normal(size=(3, F))
    p, m, v = O.sparse_adamw(uniq, g, p0, m0, v0, step=5, **HP)
    pr, mr, vr = O.sparse_adamw_rows(g, p0[uniq], m0[uniq], v0[uniq], step=5, **HP)
    np.testing.assert_array_equal(pr, p[uniq]); np.testing.assert_array_equal(mr, m[uniq])
    np.testing.assert_array_equal(vr, v[uniq])


def test_bf16_round_matches_torch():
    rng = np.random.default_rng(20)
    a = np.concatenate([rng.normal(size=5000), rng.normal(size=2000) * 1e-30, rng.normal(size=2000) * 1e30,
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, np.inf, -np.inf]]).astype(np.float32)
    # exact ties: mantissa low half == 0x8000
    ties = (rng.integers(0, 2 ** 15, size=2000).astype(np.uint32) << np.uint32(16) | np.uint32(0x8000)).view(np.float32)
    ties = ties[np.isfinite(ties)]
    a = np.concatenate([a, ties])
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.bf16_round(a), ref)


# -- prefetch dedup and decode chain ------------------------------------------
def test_dedup_remap_matches_numpy_unique():
    ids = inputs.zipf_ids(500, 97, seed=3)
    uniq, remap = O.dedup_remap(ids)
    u2, inv = np.unique(ids, return_inverse=True)
    np.testing.assert_array_equal(uniq, u2)
    np.testing.assert_array_equal(remap, inv)
    np.testing.assert_array_equal(uniq[remap], ids)


def test_cost_model_reproduces_the_printed_saving_fractions():
    # golden values: percentages the paper prints for five published model configurations
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "train_saving_fractions.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                name, d, dff, L, pct, status = line.split()
                rows.append((name, int(d), int(dff), int(L), float(pct), status))
    assert len(rows) == 5
    for name, d, dff, L, pct, status in rows:
        got = 100.0 * O.train_saving_fraction(d, dff, L)
        assert abs(got - 100.0 * dff / (4 * d + 2 * L + 3 * dff)) < 1e-9          # the closed form
        if status == "ok":
            assert abs(got - pct) <= 0.05, (name, got, pct)
        else:   # the one printed value the paper's own formula does not give
            assert round(got, 1) == 22.3 and pct == 22.8
    # the FFN part alone: exactly one third fewer multiply-adds, whatever the widths
    for d, dff in ((1024, 4096), (2048, 8192), (1536, 8960)):
        assert 3 * O.ffn_macs_per_token(d, dff, True) == 2 * O.ffn_macs_per_token(d, dff, False)
        assert O.train_flops_per_layer(3, 7, d, dff, False) - O.train_flops_per_layer(3, 7, d, dff, True) == 3 * 7 * d * dff


def test_lfu_row_cache_serves_right_rows_and_keeps_the_most_frequent():
    # simulate the device buffer [cache slots | staging] and check every token finds its row;
    # check the LFU property after every batch; check the hit rate on a Zipf stream
    V, F, n_slots, T = 400, 3, 40, 300
    rng = np.random.default_rng(31)
    table = rng.normal(size=(V, F))
    dev = np.full((n_slots + T, F), np.nan)
    cache = O.LfuRowCache(V, n_slots)
    hit_tokens = total = 0
    for b in range(12):
        ids = inputs.zipf_ids(T, V, seed=100 + b, perm_seed=5)
        cached_before = dict(cache.slot_of)
        remap, misses, installs = cache.step(ids)
        dev[n_slots:n_slots + len(misses)] = table[misses]          # the copy of the missed rows
        np.testing.assert_array_equal(dev[remap], table[ids])        # every token reads its own row
        assert len(set(misses.tolist())) == len(misses) and not set(misses.tolist()) & set(cached_before)
        first_use = [t for k, t in enumerate(ids.tolist()) if t not in ids[:k].tolist() and t not in cached_before]
        assert misses.tolist() == first_use                          # copy order = order of first use
        for t, slot, j in installs:                                  # promotion from the staging area
            assert misses[j] == t
            dev[slot] = dev[n_slots + j]
        for t, slot in cache.slot_of.items():
            assert cache.id_in_slot[slot] == t
            np.testing.assert_array_equal(dev[slot], table[t])
        # LFU: no id of this batch left outside is more frequent than a cached row the batch did not use
        outside = [t for t in misses.tolist() if t not in cache.slot_of]
        cold = [t for t in cache.slot_of if t not in set(ids.tolist())]
        if outside and cold:
            assert max(cache.freq[t] for t in outside) <= min(cache.freq[t] for t in cold)
        if b >= 6:
            hit_tokens += sum(1 for t in ids.tolist() if t in cached_before)
            total += T
    assert sum(s >= 0 for s in cache.id_in_slot) == n_slots
    # the 40 hottest of 400 Zipf(1.1) ids carry about 62 % of the token mass
    assert 0.5 < hit_tokens / total < 0.75, hit_tokens / total


def test_lfu_row_cache_hand_worked_tie_breaks():
    """Four batches worked out by hand from the stated policy (3 slots, ids below 10): every remap,
    miss list and slot content is written out here, not computed.  The batches are chosen so that the
    order of equally frequent candidates (id ascending) and of equally cold victims (id ascending)
    decides the outcome, and so that a candidate which fails ends the update."""
    c = O.LfuRowCache(10, 3)
    # batch 1: empty cache, everything misses in order of first use; counts 5:3, 3:2, 7:1, 9:1.
    # Offered 5, 3, then 7 before 9 (equal counts, lower id first): 7 takes the last free slot,
    # 9 finds neither a free slot nor a cached row the batch did not use, and the update ends.
    remap, misses, installs = c.step([5, 3, 5, 7, 3, 5, 9])
    assert remap.tolist() == [3, 4, 3, 5, 4, 3, 6] and misses.tolist() == [5, 3, 7, 9]
    assert installs == [(5, 0, 0), (3, 1, 1), (7, 2, 2)] and c.id_in_slot == [5, 3, 7]
    # batch 2: 5 hits slot 0; misses 9, 2, 8.  Counts now 9:3, 8:2, 2:1, 5:4; cached and unused: 7 (1), 3 (2).
    # 9 (3) replaces the coldest, 7; 8 (2) is not strictly more frequent than 3 (2): it fails, the update ends.
    remap, misses, installs = c.step([9, 9, 2, 5, 8, 8])
    assert remap.tolist() == [3, 3, 4, 0, 5, 5] and misses.tolist() == [9, 2, 8]
    assert installs == [(9, 2, 0)] and c.id_in_slot == [5, 3, 9]
    # batch 3: misses 6, 1, 4 with counts 6:3, 1:3, 4:1; cached and unused: 3 (2), 9 (3), 5 (4).
    # Equal counts: 1 is offered before 6 and replaces 3; 6 (3) is not above 9 (3) and fails.
    remap, misses, installs = c.step([6, 6, 6, 1, 1, 1, 4])
    assert remap.tolist() == [3, 3, 3, 4, 4, 4, 5] and misses.tolist() == [6, 1, 4]
    assert installs == [(1, 1, 1)] and c.id_in_slot == [5, 1, 9]
    # batch 4: 6 reaches count 5; cached and unused: 1 (3), 9 (3), 5 (4).  Equally cold: the lower id, 1, goes.
    remap, misses, installs = c.step([6, 6])
    assert remap.tolist() == [3, 3] and misses.tolist() == [6]
    assert installs == [(6, 1, 0)] and c.id_in_slot == [5, 6, 9]
    assert c.freq.tolist() == [0, 3, 1, 2, 1, 4, 5, 1, 2, 3]


def test_edit_target_index_follows_the_stated_rules():
    # one to one; left padding; "each target token repeated floor(n_s / n_t) times, the last one
    # repeated as needed to cover the n_s source positions"
    assert O.edit_target_index(3, 3, O.EDIT_REPLACE) == [0, 1, 2]
    assert O.edit_target_index(4, 2, O.EDIT_PAD_LEFT) == [-1, -1, 0, 1]
    assert O.edit_target_index(4, 2, O.EDIT_COPY) == [0, 0, 1, 1]
    assert O.edit_target_index(5, 2, O.EDIT_COPY) == [0, 0, 1, 1, 1]
    assert O.edit_target_index(7, 3, O.EDIT_COPY) == [0, 0, 1, 1, 2, 2, 2]
    assert O.edit_target_index(3, 3, O.EDIT_COPY) == [0, 1, 2] == O.edit_target_index(3, 3, O.EDIT_PAD_LEFT)
    assert O.edit_target_index(4, 9, O.EDIT_AVERAGE) is None
    for n_s, n_t in itertools.product(range(1, 9), repeat=2):
        if n_s >= n_t:
            idx = O.edit_target_index(n_s, n_t, O.EDIT_COPY)
            counts = [idx.count(k) for k in range(n_t)]
            assert len(idx) == n_s and idx == sorted(idx)
            assert counts[:-1] == [n_s // n_t] * (n_t - 1) and counts[-1] == n_s - (n_s // n_t) * (n_t - 1)
    for bad in ((2, 3, O.EDIT_REPLACE), (2, 3, O.EDIT_COPY), (2, 3, O.EDIT_PAD_LEFT), (0, 1, O.EDIT_COPY)):
        with pytest.raises(ValueError):
            O.edit_target_index(*bad)


def test_edit_rows_equals_substituting_the_tokens():
    # editing the table rows of the source tokens is the same layer as feeding the target tokens
    # at the source positions (when the source tokens occur nowhere else); sources and targets may overlap
    rng = np.random.default_rng(41)
    V, F, d = 12, 5, 4
    E, Wg, Wd = rng.normal(size=(V, F)), rng.normal(size=(F, d)), rng.normal(size=(d, F))
    src, tgt, pad = [3, 7, 8, 1], [7, 5], 0
    for mode in (O.EDIT_PAD_LEFT, O.EDIT_COPY):
        edited, backup = O.edit_rows(E, src, tgt, mode, pad)
        np.testing.assert_array_equal(backup, E[src])
        idx = O.edit_target_index(len(src), len(tgt), mode)
        ids = np.asarray([2] + src + [9])
        sub = np.asarray([2] + [pad if k < 0 else tgt[k] for k in idx] + [9])
        x = rng.normal(size=(len(ids), d))
        np.testing.assert_array_equal(O.ffn_forward(x, ids, Wg, Wd, edited)[0], O.ffn_forward(x, sub, Wg, Wd, E)[0])
        untouched = [t for t in range(V) if t not in src]
        np.testing.assert_array_equal(edited[untouched], E[untouched])
    swapped, _ = O.edit_rows(E, [3, 7], [7, 3], O.EDIT_REPLACE)          # a swap reads the old rows
    np.testing.assert_array_equal(swapped[[3, 7]], E[[7, 3]])
    avg, _ = O.edit_rows(E, src, [5, 6, 11], O.EDIT_AVERAGE)
    np.testing.assert_allclose(avg[src], np.tile(np.mean(E[[5, 6, 11]], axis=0), (4, 1)), rtol=1e-15)
    undone = avg.copy()
    undone[src] = O.edit_rows(E, src, [5, 6, 11], O.EDIT_AVERAGE)[1]
    np.testing.assert_array_equal(undone, E)


def test_decode_chain_composes_layers_with_rounded_residual():
    rng = np.random.default_rng(21)
    T, d, F, V = 4, 8, 16, 5
    ids = rng.integers(0, V, size=T)
    layers = [(rng.normal(size=(F, d)) * .3, rng.normal(size=(d, F)) * .3, rng.normal(size=(V, F))) for _ in range(3)]
    x0 = O.bf16_round(rng.normal(size=(T, d)))
    outs = O.decode_chain(x0, ids, layers)
    x = x0
    for l, (Wg, Wd, E) in enumerate(layers):
        y, _ = O.ffn_forward(x, ids, Wg, Wd, E)
        x = torch.from_numpy((x + y).astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
        np.testing.assert_array_equal(outs[l], x)


# -- input generators ----------------------------------------------------------
def test_zipf_ids_follow_the_power_law():
    V, n = 1000, 200000
    ids = inputs.zipf_ids(n, V, seed=5, permute=False)
    assert ids.dtype == np.int32 and ids.min() >= 0 and ids.max() < V
    w = np.arange(1, V + 1, dtype=np.float64) ** -1.1
    p = w / w.sum()
    freq = np.bincount(ids, minlength=V) / n
    assert abs(freq[0] - p[0]) < 5 * np.sqrt(p[0] * (1 - p[0]) / n)
    assert abs(freq[:10].sum() - p[:10].sum()) < 0.01
    # the permuted stream has the same multiset of frequencies
    idp = inputs.zipf_ids(n, V, seed=5, permute=True)
    assert sorted(np.bincount(idp, minlength=V).tolist()) == sorted(np.bincount(ids, minlength=V).tolist())
    np.testing.assert_array_equal(inputs.zipf_ids(100, V, seed=5), inputs.zipf_ids(100, V, seed=5))
