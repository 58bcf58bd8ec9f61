"""dmoe_topology_static (the entry point that uses the library's built-in scratch instead of a caller buffer) gives
exactly what dmoe_topology gives: every routing and topology array bit for bit, on two calls in a row, the second
on a smaller input (the built-in array keeps the first call's contents), and then forward + backward run on its
topology.  Sizes beyond the built-in scratch are refused before anything is enqueued."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2211_15841_amd as dm
from dmoe_inputs import Config, make_inputs
from tests._harness import to_dev

pytestmark = pytest.mark.gpu

KEYS = ["expert_idx", "weights", "logits", "tokens_per_expert", "padded_offsets", "row_of", "token_of", "row_offsets",
        "column_indices", "row_indices", "column_offsets_t", "row_indices_t", "block_offsets_t", "counts",
        "expert_order", "group_offsets", "row_group", "sched"]


def _both(cfg):
    inp = make_inputs(cfg)
    x, wr = to_dev(inp["x"]), to_dev(inp["w_router"])
    bias = torch.from_numpy(inp["router_bias"]).cuda() if inp["router_bias"] is not None else None
    out = []
    for static in (False, True):
        ws = dm.Workspace(cfg.num_tokens, cfg.d_model, cfg.ffn_hidden, cfg.num_experts, cfg.top_k, cfg.normalize_topk,
                          guard_bytes=1 << 16)
        ws.topology_mem.fill_(0xFF)
        if static:
            ws.scratch.fill_(0x5A)
            ws.topology_static(x, wr, bias)
        else:
            ws.topology(x, wr, bias)
        arrays = {k: v.numpy().copy() for k, v in ws.topology_arrays().items()}
        if static:                               # the caller's scratch was not touched by the static variant
            assert bool((ws.scratch == 0x5A).all())
        ws.check_guards()
        out.append((ws, arrays))
    return inp, out


def test_static_scratch_matches_caller_scratch_twice_in_a_row():
    big = Config("noalloc_big", 5000, 256, 512, 64, 2, normalize_topk=1, zipf_s=1.0, seed=311)
    small = Config("noalloc_small", 333, 128, 256, 5, 1, seed=312)
    for cfg in (big, small):
        inp, ((ws_a, a), (ws_b, b)) = _both(cfg)
        for k in KEYS:
            ga, gb = np.asarray(a[k]), np.asarray(b[k])
            assert ga.shape == gb.shape and ga.dtype == gb.dtype, k
            assert np.array_equal(ga.view(np.uint8), gb.view(np.uint8)), "%s differs (%s)" % (k, cfg.name)
        # the layer runs on the topology of the static call and agrees with the run on the other one, bit for bit
        dev = {k: to_dev(inp[k]) for k in ("x", "w_router", "w1", "w2", "dy")}
        res = []
        for ws in (ws_a, ws_b):
            ws.forward(dev["x"], dev["w1"], dev["w2"])
            ws.backward(dev["x"], dev["w_router"], dev["w1"], dev["w2"], dev["dy"])
            torch.cuda.synchronize()
            ws.check_guards()
            res.append([t.clone() for t in (ws.y, ws.dx, ws.dw1, ws.dw2, ws.dw_router)])
        for ta, tb in zip(*res):
            assert torch.equal(ta.view(torch.uint8), tb.view(torch.uint8))


def test_sizes_beyond_the_built_in_scratch_are_refused():
    cfg = dm.DMoEConfig(1 << 20, 128, 128, 256, 8, 128, 0, 0)      # 32 768 chunks x 256 experts x 4 bytes = 32 MiB
    s = dm.dmoe_sizes(cfg)
    fake = 0x7f0000000000
    topo = dm.dmoe_topology_bind(cfg, fake, s["topology_bytes"])
    rc = dm.load_library().dmoe_topology_static(ctypes.byref(cfg), fake, fake, None, ctypes.byref(topo), None)
    assert rc == -2 and "built-in" in dm.dmoe_last_error()
