"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

Configurations 2-4 (64 experts) are compared against the oracle in full.  Configuration 5 (0.94 G weights per
matrix) is too large for a float64 dense oracle in test time: all of its indices are compared in full, and the
values on seeded samples that the oracle computes one by one -- output rows of y and dx, and for every expert a
128-column panel of hidden units, which fixes 128 columns of dW1 and 128 rows of dW2."""
import numpy as np
import pytest
import torch

from dmoe_inputs import CONFIGS, make_inputs
from oracle import dmoe_oracle as orc
from tests._harness import full_parity, run_gpu, run_oracle_indices, check_indices, check_values, bf16_to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg", CONFIGS[1:4], ids=lambda c: c.name)
def test_sixty_four_expert_configs_in_full(cfg):
    errs, gpu, ref = full_parity(cfg)
    n = ref["tokens_per_expert"]
    print(cfg.name, "P=%d nnz=%d empty=%d max_load=%d" % (ref["counts"][0], ref["counts"][2], int((n == 0).sum()), n.max()),
          {k: "%.2e" % v for k, v in errs.items()})
    if cfg.zipf_s >= 1.2:       # the skewed top-2 workload: several experts empty, some above 4x the mean load
        assert (n == 0).sum() >= 3 and n.max() > 4 * n.mean()


def test_large_expert_config_on_samples():
    cfg = CONFIGS[4]
    inp = make_inputs(cfg)
    ref = run_oracle_indices(cfg, inp)
    gpu = run_gpu(cfg, inp)
    check_indices(gpu["topo"], ref)
    h, k = cfg.ffn_hidden, cfg.top_k
    idx, w, p = ref["expert_idx"], ref["weights"], ref["probs"]
    rng = np.random.default_rng(55)
    toks = sorted(rng.choice(cfg.num_tokens, size=6, replace=False).tolist())
    y_rows = orc.forward_rows(inp["x"], inp["w1"], inp["w2"], idx, w, h, toks)
    dx_rows, dw_rows, dl_rows = orc.backward_rows(inp["x"], inp["w_router"], inp["w1"], inp["w2"], inp["dy"], idx, w, p,
                                                  h, cfg.normalize_topk, toks)
    scale_y = np.abs(gpu["y"]).max()
    scale_dx = np.abs(gpu["dx"]).max()
    assert np.abs(gpu["y"][toks] - y_rows).max() <= 1e-2 * max(np.abs(y_rows).max(), 0.25 * scale_y)
    assert np.abs(gpu["dx"][toks] - dx_rows).max() <= 1e-2 * max(np.abs(dx_rows).max(), 0.25 * scale_dx)
    for e in range(cfg.num_experts):
        c0 = int(rng.integers(0, h // 128)) * 128 + int(rng.integers(0, 2)) * 64   # straddles or fills a block
        cols = np.arange(c0, min(c0 + 128, h))
        dw1_c, dw2_c = orc.weight_grad_panel(inp["x"], inp["w1"], inp["w2"], inp["dy"], idx, w, h, e, cols)
        check_values("dw1[e=%d]" % e, gpu["dw1"][:, e * h + cols], dw1_c)
        check_values("dw2[e=%d]" % e, gpu["dw2"][e * h + cols, :], dw2_c)
