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


@pytest.mark.timeout(900)
def test_large_expert_shape_in_full_on_a_short_batch():
    """The largest configuration's d, h, E and k (hb = 112, db = 32, K up to 14 336) on 2 048 tokens, where the float64
    oracle is affordable: every tensor, dw_router included, compared in full and tile by tile."""
    from dmoe_inputs import Config
    big = CONFIGS[4]
    cfg = Config("large_expert_shape_short", 2048, big.d_model, big.ffn_hidden, big.num_experts, big.top_k, seed=1905)
    errs, gpu, ref = full_parity(cfg)
    assert "dw_router" in errs
    print(cfg.name, "P=%d nnz=%d" % (ref["counts"][0], ref["counts"][2]), {k: "%.2e" % v for k, v in errs.items()})


@pytest.mark.timeout(900)
def test_large_expert_config_on_samples():
    """Indices in full.  Values: one token out of every 256 (128 tokens) through the oracle's forward and backward on
    that sub-batch (a token's y and dx depend on no other token), one 128-column panel of hidden units per expert for
    dW1 / dW2, the router's dscores on the sampled tokens, and dw_router against x^T dscores taken in float64 from the
    library's own dscores (which the sampled rows pin)."""
    cfg = CONFIGS[4]
    inp = make_inputs(cfg)
    ref = run_oracle_indices(cfg, inp)
    gpu = run_gpu(cfg, inp)
    check_indices(gpu["topo"], ref)
    h, k, T, E = cfg.ffn_hidden, cfg.top_k, cfg.num_tokens, cfg.num_experts
    idx, w, p = ref["expert_idx"], ref["weights"], ref["probs"]
    rng = np.random.default_rng(55)
    toks = np.sort(np.arange(0, T, 256) + rng.integers(0, 256, size=T // 256))
    sub = lambda a: np.ascontiguousarray(a[toks])
    y_rows = orc.forward(sub(inp["x"]), inp["w1"], inp["w2"], sub(idx), sub(w), h)
    g = orc.backward(sub(inp["x"]), inp["w_router"], inp["w1"], inp["w2"], sub(inp["dy"]), sub(idx), sub(w), sub(p), h,
                     cfg.normalize_topk)
    scale_y, scale_dx = np.abs(gpu["y"]).max(), np.abs(gpu["dx"]).max()
    assert np.abs(gpu["y"][toks] - y_rows).max() <= 1e-2 * max(np.abs(y_rows).max(), 0.25 * scale_y)
    assert np.abs(gpu["dx"][toks] - g["dx"]).max() <= 1e-2 * max(np.abs(g["dx"]).max(), 0.25 * scale_dx)
    # the router's gradient: dscores rows from the library's scratch (still intact after the call) against the oracle's
    ws = gpu["ws"]
    dl_gpu = _scratch_dlogits(ws, T, E)
    assert np.abs(dl_gpu[toks] - g["dlogits"]).max() <= 1e-2 * np.abs(g["dlogits"]).max()
    from dmoe_inputs import bf16_bits_to_f32
    dwr_expect = bf16_bits_to_f32(inp["x"]).astype(np.float64).T @ dl_gpu
    check_values("dw_router", gpu["dw_router"], dwr_expect)
    for e in range(cfg.num_experts):
        c0 = int(rng.integers(0, h // 128)) * 128 + int(rng.integers(0, 2)) * 64   # straddles or fills a block
        cols = np.arange(c0, min(c0 + 128, h))
        dw1_c, dw2_c = orc.weight_grad_panel(inp["x"], inp["w1"], inp["w2"], inp["dy"], idx, w, h, e, cols)
        check_values("dw1[e=%d]" % e, gpu["dw1"][:, e * h + cols], dw1_c)
        check_values("dw2[e=%d]" % e, gpu["dw2"][e * h + cols, :], dw2_c)


def _scratch_dlogits(ws, T, E):
    """The fp32 dscores [T, E] that dmoe_backward left in the caller's scratch buffer."""
    import ctypes
    import paper_2211_15841_amd as dm
    off = ctypes.c_size_t()
    rc = dm.load_library().dmoe_debug_scratch_offset(ctypes.byref(ws.cfg), b"dlogits", ctypes.byref(off))
    assert rc == 0, dm.dmoe_last_error()
    torch.cuda.synchronize()
    return ws.scratch[off.value:off.value + 4 * T * E].view(torch.float32).cpu().numpy().reshape(T, E).astype(np.float64)
