"""Pins for the floating-point half of the CPU oracle (no GPU).

The oracle computes each expert's FFN densely on exactly the tokens routed to it.  It is pinned here by
(i) a dense all-experts-masked brute force in float64 (every expert applied to every token, then gated),
(ii) torch float64 autograd on that dense formulation, a third implementation, for every gradient,
(iii) central finite differences, (iv) special cases that reduce to a textbook MLP (two library GEMMs),
(v) closed-form values of the activation.
"""
import math

import numpy as np
import pytest
import torch

from dmoe_inputs import small_config, make_inputs, bf16_bits_to_f32, f32_to_bf16_bits
from oracle import dmoe_oracle as orc


def _f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


def _route(cfg, inp):
    return orc.route(inp["x"], inp["w_router"], inp["router_bias"], cfg.top_k, cfg.normalize_topk)


def _dense_masked_forward(cfg, inp, idx, w):
    """y = sum_e G[t,e] * FFN_e(x_t) with FFN_e evaluated for ALL (t, e) pairs."""
    x, w1, w2 = _f64(inp["x"]), _f64(inp["w1"]), _f64(inp["w2"])
    T, d = x.shape
    E, h = cfg.num_experts, cfg.ffn_hidden
    G = np.zeros((T, E))
    for t in range(T):
        for s in range(cfg.top_k):
            G[t, idx[t, s]] += w[t, s]
    y = np.zeros((T, d))
    for e in range(E):
        hid = x @ w1[:, e * h:(e + 1) * h]
        act = np.array([[0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in row] for row in hid])
        y += G[:, e:e + 1] * (act @ w2[e * h:(e + 1) * h, :])
    return y


CASES = [
    small_config("k1", T=70, d=128, h=128, E=4, k=1, seed=21),
    small_config("k2norm", T=90, d=128, h=256, E=5, k=2, normalize_topk=1, seed=22),
    small_config("k3raw_skew", T=60, d=128, h=128, E=6, k=3, zipf_s=1.5, seed=23),
]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_forward_equals_dense_masked_brute_force(cfg):
    inp = make_inputs(cfg)
    logits, idx, w, p = _route(cfg, inp)
    y = orc.forward(inp["x"], inp["w1"], inp["w2"], idx, w, cfg.ffn_hidden)
    ref = _dense_masked_forward(cfg, inp, idx, w)
    assert np.abs(y - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())


def test_single_expert_is_the_textbook_mlp():
    cfg = small_config("one", T=150, d=128, h=256, E=1, k=1, seed=31)
    inp = make_inputs(cfg)
    logits, idx, w, p = _route(cfg, inp)
    assert np.all(idx == 0) and np.allclose(w, 1.0)
    y = orc.forward(inp["x"], inp["w1"], inp["w2"], idx, w, cfg.ffn_hidden)
    hid = torch.from_numpy(_f64(inp["x"])) @ torch.from_numpy(_f64(inp["w1"]))
    ref = torch.nn.functional.gelu(hid) @ torch.from_numpy(_f64(inp["w2"]))
    assert np.allclose(y, ref.numpy(), rtol=1e-12, atol=1e-13)


def test_identical_experts_with_normalised_weights_ignore_routing():
    cfg = small_config("same", T=80, d=128, h=128, E=4, k=2, normalize_topk=1, seed=32)
    inp = make_inputs(cfg)
    h = cfg.ffn_hidden
    inp["w1"] = np.tile(inp["w1"][:, :h], (1, cfg.num_experts))
    inp["w2"] = np.tile(inp["w2"][:h, :], (cfg.num_experts, 1))
    logits, idx, w, p = _route(cfg, inp)
    y = orc.forward(inp["x"], inp["w1"], inp["w2"], idx, w, h)
    ref = orc.gelu(_f64(inp["x"]) @ _f64(inp["w1"][:, :h])) @ _f64(inp["w2"][:h, :])
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-13)


def test_permuting_tokens_permutes_outputs():
    cfg = CASES[1]
    inp = make_inputs(cfg)
    logits, idx, w, p = _route(cfg, inp)
    y = orc.forward(inp["x"], inp["w1"], inp["w2"], idx, w, cfg.ffn_hidden)
    perm = np.random.default_rng(0).permutation(cfg.num_tokens)
    inp2 = dict(inp, x=inp["x"][perm])
    l2, idx2, w2, p2 = _route(cfg, inp2)
    assert np.array_equal(idx2, idx[perm])
    y2 = orc.forward(inp2["x"], inp["w1"], inp["w2"], idx2, w2, cfg.ffn_hidden)
    assert np.allclose(y2, y[perm], rtol=1e-12, atol=1e-14)


def test_gelu_values_and_derivative():
    assert orc.gelu(np.array([0.0]))[0] == 0.0
    assert orc.gelu_grad(np.array([0.0]))[0] == 0.5
    big = np.array([12.0, 30.0])
    assert np.allclose(orc.gelu(big), big) and np.allclose(orc.gelu_grad(big), 1.0)
    assert np.all(np.abs(orc.gelu(-big)) < 1e-30) and np.all(np.abs(orc.gelu_grad(-big)) < 1e-30)
    v = np.linspace(-6, 6, 241)
    ref = np.array([0.5 * t * (1.0 + math.erf(t / math.sqrt(2.0))) for t in v])
    assert np.allclose(orc.gelu(v), ref, rtol=1e-14, atol=1e-16)
    assert abs(orc.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15        # Phi(1)
    eps = 1e-6
    fd = (orc.gelu(v + eps) - orc.gelu(v - eps)) / (2 * eps)
    assert np.allclose(orc.gelu_grad(v), fd, rtol=1e-8, atol=1e-9)


# ----------------------------------------------------------------------------- gradients
def _torch_dense(cfg, inp, idx, activation=0):
    """Differentiable dense masked formulation in torch float64 (routing indices held constant)."""
    E, h = cfg.num_experts, cfg.ffn_hidden
    leaves = {k: torch.tensor(_f64(inp[k]), requires_grad=True) for k in ("x", "w_router", "w1", "w2")}
    x, wr, w1, w2 = leaves["x"], leaves["w_router"], leaves["w1"], leaves["w2"]
    z = x @ wr
    if inp["router_bias"] is not None:
        z = z + torch.tensor(inp["router_bias"].astype(np.float64))
    p = torch.softmax(z, dim=1)
    ti = torch.tensor(idx.astype(np.int64))
    sel = p.gather(1, ti)
    if cfg.normalize_topk:
        sel = sel / sel.sum(dim=1, keepdim=True)
    G = torch.zeros_like(p).scatter(1, ti, sel)
    y = 0
    for e in range(E):
        hid = torch.nn.functional.gelu(x @ w1[:, e * h:(e + 1) * h], approximate="tanh" if activation else "none")
        y = y + G[:, e:e + 1] * (hid @ w2[e * h:(e + 1) * h, :])
    return leaves, y, sel


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_backward_equals_torch_autograd_on_dense_formulation(cfg):
    inp = make_inputs(cfg)
    logits, idx, w, p = _route(cfg, inp)
    g = orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, cfg.ffn_hidden,
                     cfg.normalize_topk)
    leaves, y, sel = _torch_dense(cfg, inp, idx)
    sel.retain_grad()
    y.backward(torch.tensor(_f64(inp["dy"])))
    # the oracle's probabilities come from float32 scores, torch's from float64 ones: agreement to ~1e-6
    for name, leaf in (("dx", "x"), ("dw_router", "w_router"), ("dw1", "w1"), ("dw2", "w2")):
        ref = leaves[leaf].grad.numpy()
        assert np.abs(g[name] - ref).max() <= 2e-5 * np.abs(ref).max() + 1e-12, name


def test_backward_against_central_finite_differences():
    cfg = small_config("fd", T=40, d=128, h=128, E=3, k=2, normalize_topk=1, seed=41)
    inp = make_inputs(cfg)
    logits, idx, w, p = _route(cfg, inp)
    srt = -np.sort(-logits.astype(np.float64), axis=1)
    assert np.all(srt[:, 1] - srt[:, 2] > 1e-3)         # no routing decision can flip under the perturbation
    g = orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, cfg.ffn_hidden, 1)
    dy = _f64(inp["dy"])
    rng = np.random.default_rng(1)

    def loss(t):
        # float64 evaluation of the layer at perturbed parameters, indices fixed
        z = t["x"] @ t["w_router"]
        ez = np.exp(z - z.max(axis=1, keepdims=True))
        pp = ez / ez.sum(axis=1, keepdims=True)
        sel = np.take_along_axis(pp, idx.astype(np.int64), axis=1)
        sel = sel / sel.sum(axis=1, keepdims=True)
        h = cfg.ffn_hidden
        y = np.zeros_like(t["x"])
        for tok in range(cfg.num_tokens):
            for s in range(cfg.top_k):
                e = idx[tok, s]
                y[tok] += sel[tok, s] * (orc.gelu(t["x"][tok] @ t["w1"][:, e * h:(e + 1) * h]) @ t["w2"][e * h:(e + 1) * h, :])
        return float((dy * y).sum())

    base = {k: _f64(inp[k]) for k in ("x", "w_router", "w1", "w2")}
    for name, key in (("dx", "x"), ("dw_router", "w_router"), ("dw1", "w1"), ("dw2", "w2")):
        v = rng.standard_normal(base[key].shape)
        v /= np.linalg.norm(v)
        eps = 1e-5
        plus = dict(base); plus[key] = base[key] + eps * v
        minus = dict(base); minus[key] = base[key] - eps * v
        fd = (loss(plus) - loss(minus)) / (2 * eps)
        an = float((g[name] * v).sum())
        assert abs(fd - an) <= 2e-5 * max(abs(an), np.linalg.norm(g[name]) * 1e-2), (name, fd, an)


def test_backward_is_linear_in_upstream_gradient_and_zero_for_empty_experts():
    cfg = small_config("lin", T=50, d=128, h=128, E=6, k=1, zipf_s=3.0, seed=51)
    inp = make_inputs(cfg)
    logits, idx, w, p = _route(cfg, inp)
    n = np.bincount(idx.reshape(-1), minlength=cfg.num_experts)
    assert (n == 0).any()
    g1 = orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, cfg.ffn_hidden, 0)
    dy2 = f32_to_bf16_bits(2.0 * bf16_bits_to_f32(inp["dy"]))
    g2 = orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], dy2, idx, w, p, cfg.ffn_hidden, 0)
    h = cfg.ffn_hidden
    for name in ("dx", "dw_router", "dw1", "dw2"):
        assert np.allclose(g2[name], 2.0 * g1[name], rtol=1e-12, atol=1e-300)
    for e in np.flatnonzero(n == 0):
        assert np.all(g1["dw1"][:, e * h:(e + 1) * h] == 0.0) and np.all(g1["dw2"][e * h:(e + 1) * h, :] == 0.0)


def test_top1_with_normalised_weight_gives_router_no_gradient():
    cfg = small_config("nograd", T=30, d=128, h=128, E=4, k=1, normalize_topk=1, seed=52)
    inp = make_inputs(cfg)
    logits, idx, w, p = _route(cfg, inp)
    assert np.all(w == 1.0)
    g = orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, cfg.ffn_hidden, 1)
    assert np.abs(g["dw_router"]).max() < 1e-12


def test_slices_equal_the_full_computation():
    cfg = CASES[1]
    inp = make_inputs(cfg)
    logits, idx, w, p = _route(cfg, inp)
    h = cfg.ffn_hidden
    y = orc.forward(inp["x"], inp["w1"], inp["w2"], idx, w, h)
    g = orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, h, cfg.normalize_topk)
    toks = [0, 7, 33, 89]
    assert np.allclose(orc.forward_rows(inp["x"], inp["w1"], inp["w2"], idx, w, h, toks), y[toks], rtol=1e-11, atol=1e-14)
    dxs, dws, dls = orc.backward_rows(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, h,
                                      cfg.normalize_topk, toks)
    assert np.allclose(dxs, g["dx"][toks], rtol=1e-10, atol=1e-14)
    assert np.allclose(dws, g["dweights"][toks], rtol=1e-10, atol=1e-14)
    assert np.allclose(dls, g["dlogits"][toks], rtol=1e-10, atol=1e-16)
    for e in range(cfg.num_experts):
        cols = [1, 5, 130, 255]
        a, b = orc.weight_grad_panel(inp["x"], inp["w1"], inp["w2"], inp["dy"], idx, w, h, e, cols)
        assert np.allclose(a, g["dw1"][:, e * h + np.array(cols)], rtol=1e-10, atol=1e-14)
        assert np.allclose(b, g["dw2"][e * h + np.array(cols), :], rtol=1e-10, atol=1e-14)


def test_weight_gradients_add_up_over_micro_batches():
    """Gradient accumulation (Section 6.2): the layer treats every token independently, so the weight gradients of
    two micro-batches taken as one batch are the sum of the micro-batches' own gradients.  This pins what
    dmoe_backward_accumulate is compared with (start + g1 + g2) to the oracle's single-batch gradient."""
    from dmoe_inputs import small_config, make_inputs
    cfg = small_config("mb", T=90, d=128, h=128, E=5, k=2, normalize_topk=1, zipf_s=0.8, seed=411)
    a, b = make_inputs(cfg), make_inputs(small_config("mb", 90, 128, 128, 5, 2, 1, 0.8, 412))
    for key in ("w_router", "w1", "w2", "router_bias"):
        b[key] = a[key]

    def grads(c, inp):
        _, idx, w, p = orc.route(inp["x"], inp["w_router"], inp["router_bias"], c.top_k, c.normalize_topk)
        return orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, c.ffn_hidden,
                            c.normalize_topk)

    ga, gb = grads(cfg, a), grads(cfg, b)
    joined = dict(a)
    for key in ("x", "dy"):
        joined[key] = np.concatenate([a[key], b[key]], axis=0)
    gj = grads(small_config("mb", 180, 128, 128, 5, 2, 1, 0.8, 411), joined)
    for k in ("dw1", "dw2", "dw_router"):
        assert np.abs(gj[k]).max() > 0
        assert np.allclose(ga[k] + gb[k], gj[k], rtol=1e-10, atol=1e-12 * np.abs(gj[k]).max()), k
    assert np.allclose(np.concatenate([ga["dx"], gb["dx"]]), gj["dx"], rtol=1e-10, atol=1e-14)


# ----------------------------------------------------------------------------- the tanh form (activation = 1)
def test_tanh_gelu_values_and_derivative():
    """The tanh form against torch's own (an independent library routine), its limits, its distance from the exact
    form (close, but not the same function), and its derivative against central differences."""
    v = np.linspace(-8, 8, 321)
    ref = torch.nn.functional.gelu(torch.tensor(v), approximate="tanh").numpy()
    assert np.allclose(orc.gelu_tanh(v), ref, rtol=1e-13, atol=1e-15)
    assert orc.gelu_tanh(np.array([0.0]))[0] == 0.0 and orc.gelu_tanh_grad(np.array([0.0]))[0] == 0.5
    big = np.array([12.0, 30.0])
    assert np.allclose(orc.gelu_tanh(big), big) and np.allclose(orc.gelu_tanh_grad(big), 1.0)
    assert np.all(np.abs(orc.gelu_tanh(-big)) < 1e-30) and np.all(np.abs(orc.gelu_tanh_grad(-big)) < 1e-30)
    gap = np.abs(orc.gelu_tanh(v) - orc.gelu(v)).max()
    assert 1e-4 < gap < 1e-3
    eps = 1e-6
    fd = (orc.gelu_tanh(v + eps) - orc.gelu_tanh(v - eps)) / (2 * eps)
    assert np.allclose(orc.gelu_tanh_grad(v), fd, rtol=1e-8, atol=1e-9)
    assert orc.activation_pair(0) == (orc.gelu, orc.gelu_grad) and orc.activation_pair(1) == (orc.gelu_tanh, orc.gelu_tanh_grad)
    with pytest.raises(ValueError):
        orc.activation_pair(2)


def test_tanh_form_forward_and_backward_equal_torch_autograd():
    cfg = CASES[1]
    inp = make_inputs(cfg)
    logits, idx, w, p = _route(cfg, inp)
    y = orc.forward(inp["x"], inp["w1"], inp["w2"], idx, w, cfg.ffn_hidden, activation=1)
    g = orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, cfg.ffn_hidden,
                     cfg.normalize_topk, activation=1)
    leaves, yt, sel = _torch_dense(cfg, inp, idx, activation=1)
    yt.backward(torch.tensor(_f64(inp["dy"])))
    assert np.abs(y - yt.detach().numpy()).max() <= 2e-5 * np.abs(y).max()
    for name, leaf in (("dx", "x"), ("dw_router", "w_router"), ("dw1", "w1"), ("dw2", "w2")):
        ref = leaves[leaf].grad.numpy()
        assert np.abs(g[name] - ref).max() <= 2e-5 * np.abs(ref).max() + 1e-12, name
    # and it is not the exact form in disguise
    y0 = orc.forward(inp["x"], inp["w1"], inp["w2"], idx, w, cfg.ffn_hidden)
    assert np.abs(y - y0).max() > 1e-7 * np.abs(y0).max()
