"""Parity of the token-dropping variant (Section 2.2: a fixed expert capacity, tokens beyond it dropped, unused
capacity padded) with its CPU oracle.  Same kernels, same bars as the dropless layer: every index array bit-exact
(row_of = -1 on dropped assignments), values within 1e-2 of the tensor maximum, tile by tile."""
import numpy as np
import pytest
import torch

from dmoe_inputs import small_config, make_inputs
from oracle import dmoe_oracle as orc
from tests._harness import full_parity, run_gpu

pytestmark = pytest.mark.gpu


def _with_capacity(name, factor, pad, **kw):
    base = small_config(name, **kw)
    cap = orc.expert_capacity(base.num_tokens, base.num_experts, factor, base.top_k)
    return small_config(name, expert_capacity=cap, pad_to_capacity=pad, **kw)


CASES = [
    _with_capacity("k1_cf1", 1.0, 0, T=900, d=128, h=256, E=6, k=1, zipf_s=1.0, seed=601),
    _with_capacity("k1_cf1_padded", 1.0, 1, T=900, d=128, h=256, E=6, k=1, zipf_s=1.0, seed=601),
    _with_capacity("k2norm_cf1.5_padded", 1.5, 1, T=700, d=256, h=128, E=5, k=2, normalize_topk=1, zipf_s=1.2, seed=602),
    _with_capacity("k2raw_cf2", 2.0, 0, T=640, d=128, h=384, E=8, k=2, zipf_s=1.5, seed=603),
    _with_capacity("E64_cf1_padded_moe_shape", 1.0, 1, T=8192, d=256, h=256, E=64, k=1, seed=604),   # capacity 128 = one block
    _with_capacity("E64_cf1.5_padded", 1.5, 1, T=4096, d=128, h=256, E=64, k=1, zipf_s=0.8, seed=605),  # capacity 96 < a block
    _with_capacity("k3_cf0.5", 0.5, 0, T=500, d=128, h=128, E=7, k=3, seed=606),
    small_config("capacity_one", T=300, d=128, h=128, E=4, k=2, seed=607, expert_capacity=1, pad_to_capacity=1),
]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_token_dropping_cases(cfg):
    errs, gpu, ref = full_parity(cfg)
    idx = ref["expert_idx"]
    load = np.bincount(idx.reshape(-1), minlength=cfg.num_experts)
    assert np.array_equal(ref["tokens_per_expert"], np.minimum(load, cfg.expert_capacity))
    dropped = np.asarray(gpu["topo"]["row_of"]) < 0
    assert dropped.sum() == int(np.maximum(load - cfg.expert_capacity, 0).sum())
    if cfg.pad_to_capacity:
        rows = -(-cfg.expert_capacity // 128) * 128
        assert (np.diff(np.asarray(gpu["topo"]["padded_offsets"])) == rows).all()
    if cfg.top_k == 1 and dropped.any():                 # outputs of dropped tokens are exactly zero (Figure 2)
        assert not gpu["y"][dropped].any()
    print(cfg.name, "dropped %d of %d" % (dropped.sum(), dropped.size), errs)


def test_a_capacity_nobody_reaches_changes_nothing():
    base = small_config("roomy", T=800, d=256, h=256, E=6, k=2, normalize_topk=1, zipf_s=1.0, seed=608)
    roomy = small_config("roomy", T=800, d=256, h=256, E=6, k=2, normalize_topk=1, zipf_s=1.0, seed=608,
                         expert_capacity=1600)
    inp = make_inputs(base)
    a, b = run_gpu(base, inp), run_gpu(roomy, inp)
    for name in ("y", "dx", "dw1", "dw2", "dw_router"):
        assert np.array_equal(a[name], b[name]), name
    for name in ("row_of", "token_of", "padded_offsets", "tokens_per_expert", "column_indices", "block_offsets_t"):
        assert np.array_equal(np.asarray(a["topo"][name]), np.asarray(b["topo"][name])), name
