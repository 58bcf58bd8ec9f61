"""Pins for the token-dropping variant of the oracle (Section 2.2: a fixed expert capacity, tokens beyond it dropped,
unused capacity padded).  No GPU.

The variant is pinned against things other than itself: the capacity equation's values, the dropless layer (a capacity
nobody reaches changes nothing), a keep mask derived a second way (cumulative one-hot counts), a dense
all-experts-masked float64 brute force gated by that mask, torch float64 autograd on the gated dense formulation,
and the structural invariants of the permutation (kept = min(load, capacity), dropped rows marked, fixed shape with
padding to capacity).
"""
import math

import numpy as np
import pytest
import torch

from dmoe_inputs import small_config, make_inputs, bf16_bits_to_f32
from oracle import dmoe_oracle as orc


def _f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


def _route(cfg, inp):
    return orc.route(inp["x"], inp["w_router"], inp["router_bias"], cfg.top_k, cfg.normalize_topk)


def _keep_by_cumulative_counts(idx, E, capacity):
    """Second derivation of the keep mask: position of f inside its expert = (running one-hot count) - 1."""
    flat = idx.reshape(-1).astype(np.int64)
    onehot = np.zeros((flat.size, E), dtype=np.int64)
    onehot[np.arange(flat.size), flat] = 1
    position = (np.cumsum(onehot, axis=0) - 1)[np.arange(flat.size), flat]
    return (position < capacity).reshape(idx.shape)


CASES = [
    (small_config("cap_k1", T=90, d=128, h=128, E=4, k=1, zipf_s=1.0, seed=61), 1.0),
    (small_config("cap_k2norm", T=80, d=128, h=256, E=5, k=2, normalize_topk=1, zipf_s=1.2, seed=62), 1.0),
    (small_config("cap_k2raw", T=70, d=128, h=128, E=6, k=2, zipf_s=0.8, seed=63), 1.5),
]


def test_capacity_equation_values():
    # expert_capacity = num_tokens / num_experts x capacity_factor  (Section 2.2)
    assert orc.expert_capacity(6, 3, 1.0) == 2              # the setting drawn in Figure 2: three experts, factor 1
    assert orc.expert_capacity(8192, 64, 1.0) == 128
    assert orc.expert_capacity(8192, 64, 1.5) == 192
    assert orc.expert_capacity(8192, 64, 2.0) == 256
    assert orc.expert_capacity(100, 64, 1.0) == 1           # rounded down, but never zero
    assert orc.expert_capacity(16384, 64, 1.0, top_k=2) == 512


@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0].name)
def test_keep_mask_and_permutation_invariants(case):
    cfg, factor = case
    inp = make_inputs(cfg)
    _, idx, w, p = _route(cfg, inp)
    E, k = cfg.num_experts, cfg.top_k
    C = orc.expert_capacity(cfg.num_tokens, E, factor, k)
    keep = orc.capacity_keep_mask(idx, E, C)
    assert np.array_equal(keep, _keep_by_cumulative_counts(idx, E, C))
    load = np.bincount(idx.reshape(-1), minlength=E)
    assert (load > C).any(), "the case must actually drop something"
    for pad in (False, True):
        n, off, row_of, token_of = orc.permutation_capacity(idx, E, C, pad)
        assert np.array_equal(n, np.minimum(load, C))
        rows = np.diff(off)
        if pad:
            assert (rows == -(-C // 128) * 128).all()                  # every expert owns the capacity's worth of rows
        else:
            assert np.array_equal(rows, -(-n.astype(np.int64) // 128) * 128)
        assert np.array_equal(row_of >= 0, keep.reshape(-1))             # dropped assignments, and only they, have no row
        kept_f = np.flatnonzero(keep.reshape(-1))
        assert np.array_equal(token_of[row_of[kept_f]], kept_f)          # inverse on the kept ones
        assert (token_of >= 0).sum() == kept_f.size
        for e in range(E):                                               # stable: ascending f, padding at the tail
            seg = token_of[off[e]:off[e + 1]]
            assert (seg[:n[e]] >= 0).all() and (seg[n[e]:] == -1).all() and (np.diff(seg[:n[e]]) > 0).all()
            assert (idx.reshape(-1)[seg[:n[e]]] == e).all()
            # the kept ones are the FIRST assignments of the expert
            assert np.array_equal(seg[:n[e]], np.flatnonzero(idx.reshape(-1) == e)[:n[e]])


def test_a_capacity_nobody_reaches_is_the_dropless_layer():
    cfg = small_config("roomy", T=60, d=128, h=128, E=4, k=2, normalize_topk=1, seed=64)
    inp = make_inputs(cfg)
    _, idx, w, p = _route(cfg, inp)
    C = cfg.num_tokens * cfg.top_k
    keep = orc.capacity_keep_mask(idx, cfg.num_experts, C)
    assert keep.all()
    a = orc.permutation(idx, cfg.num_experts)
    b = orc.permutation_capacity(idx, cfg.num_experts, C, False)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    h = cfg.ffn_hidden
    y0 = orc.forward(inp["x"], inp["w1"], inp["w2"], idx, w, h)
    y1 = orc.forward(inp["x"], inp["w1"], inp["w2"], idx, w, h, keep_mask=keep)
    assert np.array_equal(y0, y1)
    g0 = orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, h, 1)
    g1 = orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, h, 1, keep_mask=keep)
    for name in g0:
        assert np.array_equal(g0[name], g1[name]), name


@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0].name)
def test_forward_equals_gated_dense_brute_force(case):
    cfg, factor = case
    inp = make_inputs(cfg)
    _, idx, w, p = _route(cfg, inp)
    E, h, k = cfg.num_experts, cfg.ffn_hidden, cfg.top_k
    C = orc.expert_capacity(cfg.num_tokens, E, factor, k)
    keep = orc.capacity_keep_mask(idx, E, C)
    y = orc.forward(inp["x"], inp["w1"], inp["w2"], idx, w, h, keep_mask=keep)
    mask2 = _keep_by_cumulative_counts(idx, E, C)
    x, w1, w2 = _f64(inp["x"]), _f64(inp["w1"]), _f64(inp["w2"])
    G = np.zeros((cfg.num_tokens, E))
    for t in range(cfg.num_tokens):
        for s in range(k):
            if mask2[t, s]:
                G[t, idx[t, s]] += w[t, s]
    ref = np.zeros_like(y)
    for e in range(E):
        hid = x @ w1[:, e * h:(e + 1) * h]
        act = np.array([[0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in row] for row in hid])
        ref += G[:, e:e + 1] * (act @ w2[e * h:(e + 1) * h, :])
    assert np.abs(y - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())
    if k == 1:                      # a dropped token's output is exactly zero (Figure 2)
        assert not y[~keep[:, 0]].any() and y[keep[:, 0]].any()


@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0].name)
def test_backward_equals_torch_autograd_on_gated_dense_formulation(case):
    cfg, factor = case
    inp = make_inputs(cfg)
    _, idx, w, p = _route(cfg, inp)
    E, h, k = cfg.num_experts, cfg.ffn_hidden, cfg.top_k
    C = orc.expert_capacity(cfg.num_tokens, E, factor, k)
    keep = orc.capacity_keep_mask(idx, E, C)
    g = orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, h, cfg.normalize_topk,
                     keep_mask=keep)
    leaves = {n: torch.tensor(_f64(inp[n]), requires_grad=True) for n in ("x", "w_router", "w1", "w2")}
    x, wr, w1, w2 = leaves["x"], leaves["w_router"], leaves["w1"], leaves["w2"]
    z = x @ wr
    if inp["router_bias"] is not None:
        z = z + torch.tensor(inp["router_bias"].astype(np.float64))
    pt = torch.softmax(z, dim=1)
    ti = torch.tensor(idx.astype(np.int64))
    sel = pt.gather(1, ti)
    if cfg.normalize_topk:
        sel = sel / sel.sum(dim=1, keepdim=True)                 # over all k chosen experts, dropped or not
    gate = sel * torch.tensor(_keep_by_cumulative_counts(idx, E, C).astype(np.float64))
    G = torch.zeros_like(pt).scatter_add(1, ti, gate)
    y = 0
    for e in range(E):
        y = y + G[:, e:e + 1] * (torch.nn.functional.gelu(x @ w1[:, e * h:(e + 1) * h]) @ w2[e * h:(e + 1) * h, :])
    y.backward(torch.tensor(_f64(inp["dy"])))
    for name, leaf in (("dx", "x"), ("dw_router", "w_router"), ("dw1", "w1"), ("dw2", "w2")):
        ref = leaves[leaf].grad.numpy()
        assert np.abs(g[name] - ref).max() <= 2e-5 * np.abs(ref).max() + 1e-12, name
    assert not g["dweights"][~keep].any()                        # no gradient through a dropped assignment
    full = orc.backward(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p, h, cfg.normalize_topk)
    assert np.abs(full["dw1"] - g["dw1"]).max() > 0              # and dropping does change the result
