"""Pins for the integer half of the CPU oracle: routing decisions, permutation, sparse-matrix encoding.

None of these tests touch a GPU.  Each pin is something other than the oracle's own formula: a brute
force in another precision, a library routine (scipy.sparse), a hand-derived fixture, or an invariant
stated by the paper (no token dropped; groups padded to the block size; row-wise block order).
"""
import json
import os

import numpy as np
import pytest
import scipy.sparse as sp

from dmoe_inputs import small_config, make_inputs, bf16_bits_to_f32, f32_to_bf16_bits, CONFIGS
from oracle import dmoe_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- inputs module
def test_bf16_round_trip_and_rounding():
    vals = np.array([1.0, -2.5, 0.0, 3.140625, 1e-3], dtype=np.float32)
    bits = f32_to_bf16_bits(vals)
    back = bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[1] == -2.5 and back[2] == 0.0 and back[3] == 3.140625
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: ties go to the even mantissa (1.0)
    assert bf16_bits_to_f32(f32_to_bf16_bits(np.array([1.0 + 2.0 ** -8], np.float32)))[0] == 1.0
    # 1 + 3*2^-8 ties between 1+2^-7 (odd) and 1+2^-6 (even)
    assert bf16_bits_to_f32(f32_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], np.float32)))[0] == 1.0 + 2.0 ** -6
    assert np.all(orc.widen_bf16(bits, np.float32) == back)


def test_inputs_are_seeded_and_shaped():
    cfg = small_config(T=50, d=128, h=128, E=3, k=1, zipf_s=1.0, seed=11)
    a, b = make_inputs(cfg), make_inputs(cfg)
    for key in ("x", "w_router", "w1", "w2", "dy", "router_bias"):
        assert np.array_equal(a[key], b[key])
    assert a["x"].shape == (50, 128) and a["w1"].shape == (128, 3 * 128) and a["w2"].shape == (3 * 128, 128)
    assert abs(float(np.exp(a["router_bias"].astype(np.float64)).sum()) - 1.0) < 1e-6
    x = bf16_bits_to_f32(a["x"])
    assert 0.8 < x.std() < 1.2
    w = bf16_bits_to_f32(a["w1"])
    assert 0.015 < w.std() < 0.025


# ----------------------------------------------------------------------------- routing
def test_logits_accumulate_in_ascending_index_order_in_float32():
    # 1 + 2^30 rounds to 2^30 in float32, so ascending order gives exactly 0; the exact sum and the
    # descending order both give 1.  All values are bf16-representable.
    x = f32_to_bf16_bits(np.array([[1.0, 2.0 ** 30, -(2.0 ** 30)]], np.float32))
    wr = f32_to_bf16_bits(np.ones((3, 2), np.float32))
    out = orc.router_logits(x, wr, None)
    assert out.dtype == np.float32 and np.all(out == 0.0)
    x2 = f32_to_bf16_bits(np.array([[2.0 ** 30, -(2.0 ** 30), 1.0]], np.float32))
    assert np.all(orc.router_logits(x2, wr, None) == 1.0)
    assert np.all(orc.router_logits(x2, wr, np.array([0.5, -1.0], np.float32)) == np.array([[1.5, 0.0]], np.float32))


def test_topk_ties_go_to_lowest_expert_and_are_distinct():
    logits = np.array([[1.0, 3.0, 3.0, 0.0], [2.0, 2.0, 2.0, 2.0], [0.0, -1.0, 5.0, 5.0]], np.float32)
    idx = orc.top_k_greedy(logits, 3)
    assert idx.tolist() == [[1, 2, 0], [0, 1, 2], [2, 3, 0]]


@pytest.mark.parametrize("k,E,norm,zipf", [(1, 4, 0, 0.0), (2, 8, 1, 1.2), (3, 5, 0, 0.0), (2, 64, 1, 1.0)])
def test_routing_against_float64_stable_sort(k, E, norm, zipf):
    cfg = small_config(T=400, d=128, h=128, E=E, k=k, normalize_topk=norm, zipf_s=zipf, seed=3 + E)
    inp = make_inputs(cfg)
    logits, idx, w, p = orc.route(inp["x"], inp["w_router"], inp["router_bias"], k, norm)
    z = bf16_bits_to_f32(inp["x"]).astype(np.float64) @ bf16_bits_to_f32(inp["w_router"]).astype(np.float64)
    if inp["router_bias"] is not None:
        z = z + inp["router_bias"].astype(np.float64)
    assert np.abs(logits - z).max() < 1e-5 * max(1.0, np.abs(z).max())
    order = np.argsort(-z, axis=1, kind="stable")
    srt = -np.sort(-z, axis=1)
    clear = np.all(srt[:, :k] - srt[:, 1:k + 1] > 1e-4, axis=1) if E > k else np.ones(len(z), bool)
    assert clear.sum() > 0.9 * len(z)
    assert np.array_equal(idx[clear], order[clear, :k])
    # each token's experts are distinct; weights are the softmax probabilities of the chosen experts
    for t in range(len(idx)):
        assert len(set(idx[t].tolist())) == k
    ez = np.exp(z - z.max(axis=1, keepdims=True))
    p64 = ez / ez.sum(axis=1, keepdims=True)
    assert np.allclose(p, p64, rtol=1e-5, atol=1e-9)
    sel = np.take_along_axis(p64, idx.astype(np.int64), axis=1)
    if norm:
        sel = sel / sel.sum(axis=1, keepdims=True)
        assert np.allclose(w.sum(axis=1), 1.0, atol=1e-12)
    assert np.all(w > 0) and np.allclose(w, sel, rtol=1e-5)
    # slot order is descending score
    assert np.all(np.diff(np.take_along_axis(logits, idx.astype(np.int64), axis=1), axis=1) <= 0)


# ----------------------------------------------------------------------------- permutation
def _check_permutation(idx, E, block=128):
    n, off, row_of, token_of = orc.permutation(idx, E, block)
    flat = idx.reshape(-1)
    F = flat.size
    assert n.sum() == F                                         # no token dropped, none duplicated
    assert np.array_equal(n, np.bincount(flat, minlength=E))
    padded = np.diff(off)
    assert np.array_equal(padded, -(-n // block) * block)       # ceil(n_e / block) * block, 0 stays 0
    P = off[-1]
    assert token_of.shape == (P,)
    assert len(set(row_of.tolist())) == F                       # injective
    assert np.array_equal(token_of[row_of], np.arange(F))
    assert (token_of == -1).sum() == P - F
    for e in range(E):
        seg = token_of[off[e]:off[e + 1]]
        real = seg[:n[e]]
        assert np.all(seg[n[e]:] == -1)                         # padding is the tail of the group
        assert np.all(real >= 0) and np.all(np.diff(real) > 0)  # ascending f: the stable order
        assert np.all(flat[real] == e)
    return n, off, row_of, token_of


@pytest.mark.parametrize("case", ["random", "empty_experts", "one_takes_all", "exact_blocks", "block_pm1", "top2"])
def test_permutation_invariants(case):
    rng = np.random.default_rng(5)
    E = 6
    if case == "random":
        idx = rng.integers(0, E, size=(1000, 1))
    elif case == "empty_experts":
        idx = rng.choice([1, 4], size=(700, 1))
    elif case == "one_takes_all":
        idx = np.full((513, 1), 3)
    elif case == "exact_blocks":
        idx = np.repeat(np.arange(E), [128, 256, 0, 128, 384, 128])[:, None]
        idx = idx[rng.permutation(len(idx))]
    elif case == "block_pm1":
        idx = np.repeat(np.arange(E), [127, 129, 1, 255, 257, 0])[:, None]
        idx = idx[rng.permutation(len(idx))]
    else:
        a = rng.integers(0, E, size=900)
        b = (a + rng.integers(1, E, size=900)) % E
        idx = np.stack([a, b], axis=1)
    _check_permutation(idx.astype(np.int32), E)


def test_permutation_against_stable_argsort():
    rng = np.random.default_rng(9)
    idx = rng.integers(0, 7, size=(2000, 2)).astype(np.int32)
    n, off, row_of, token_of = orc.permutation(idx, 7)
    order = np.argsort(idx.reshape(-1), kind="stable")          # library routine: stable sort by expert
    assert np.array_equal(token_of[token_of >= 0], order)


# ----------------------------------------------------------------------------- topology
def test_topology_hand_worked_example():
    g = json.load(open(os.path.join(GOLDEN, "topology_small.json")))
    topo = orc.topology(np.array(g["padded_offsets"], np.int32), g["ffn_hidden"])
    for key in ("row_offsets", "column_indices", "row_indices", "column_offsets_t", "row_indices_t",
                "block_offsets_t", "counts"):
        assert topo[key].tolist() == g[key], key


def test_encode_mask_against_scipy_on_arbitrary_masks():
    rng = np.random.default_rng(2)
    for shape in [(5, 7), (1, 9), (12, 3), (8, 8)]:
        mask = (rng.random(shape) < 0.4).astype(np.uint8)
        enc = orc.encode_mask(mask)
        csr = sp.csr_matrix(mask)
        csr.sort_indices()
        assert np.array_equal(enc["row_offsets"], csr.indptr)
        assert np.array_equal(enc["column_indices"], csr.indices)
        assert np.array_equal(enc["row_indices"], sp.coo_matrix(mask).row)      # COO in row-major order
        # transposed metadata = CSR of the transpose; offsets point back into the primary numbering
        numbered = sp.csr_matrix((np.arange(1, csr.nnz + 1), csr.indices, csr.indptr), shape=shape)
        csc = numbered.tocsc()
        csc.sort_indices()
        assert np.array_equal(enc["column_offsets_t"], csc.indptr)
        assert np.array_equal(enc["row_indices_t"], csc.indices)
        assert np.array_equal(enc["block_offsets_t"], csc.data - 1)


@pytest.mark.parametrize("rows,hb", [([2, 0, 1], 2), ([0, 0, 3, 1], 4), ([1], 8), ([0, 0], 2), ([5, 1, 0, 2, 0, 0, 7], 3)])
def test_topology_generic_equals_closed_form_and_invariants(rows, hb):
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32) * 128
    topo = orc.topology(off, hb * 128)
    closed = orc.topology_closed_form(off, hb * 128)
    for key, val in closed.items():
        assert np.array_equal(topo[key], val), key
    R, nnz = sum(rows), sum(rows) * hb
    assert topo["counts"].tolist() == [R * 128, R, nnz, 0]
    assert topo["column_indices"].size == nnz
    # row-wise order: (row, col) pairs strictly increasing => valid as both BCSR and BCOO
    key = topo["row_indices"].astype(np.int64) * (len(rows) * hb) + topo["column_indices"]
    assert np.all(np.diff(key) > 0)
    # transpose indices: a permutation of the blocks; each points at a block in its own column and row
    bot = topo["block_offsets_t"]
    assert sorted(bot.tolist()) == list(range(nnz))
    cot = topo["column_offsets_t"]
    for c in range(len(rows) * hb):
        seg = slice(cot[c], cot[c + 1])
        assert np.all(topo["column_indices"][bot[seg]] == c)
        assert np.array_equal(topo["row_indices"][bot[seg]], topo["row_indices_t"][seg])
        assert np.all(np.diff(topo["row_indices_t"][seg]) > 0)
    # transposing twice gives the primary arrays back
    mask = orc.block_mask(off, hb)
    back = orc.encode_mask(mask.T.copy())
    assert np.array_equal(back["column_offsets_t"], topo["row_offsets"])
    assert np.array_equal(back["row_indices_t"], topo["column_indices"])


def test_tiny_benchmark_config_padding_and_block_count():
    """Each expert's padded row count is ceil(n_e/128)*128 on the tiny benchmark configuration."""
    cfg = CONFIGS[0]
    inp = make_inputs(cfg)
    logits, idx, w, p = orc.route(inp["x"], inp["w_router"], inp["router_bias"], cfg.top_k, cfg.normalize_topk)
    n, off, row_of, token_of = _check_permutation(idx, cfg.num_experts)
    assert n.sum() == cfg.num_tokens * cfg.top_k
    topo = orc.topology(off, cfg.ffn_hidden)
    assert topo["counts"][2] == (off[-1] // 128) * (cfg.ffn_hidden // 128)
