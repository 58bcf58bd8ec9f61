"""The three calls of the layer only enqueue kernels on the stream they are given: no allocation, no host
synchronisation, no memset.  So one step can be captured into a HIP graph and replayed; every replay must give,
bit for bit, what the eager calls give on the same inputs (routing included: the grids are sized for the upper bounds
and the kernels take the actual counts from device memory, so a replay follows a new routing)."""
import numpy as np
import pytest
import torch

import paper_2211_15841_amd as dm
from dmoe_inputs import small_config, make_inputs
from tests._harness import to_dev

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.detach().clone().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def test_a_step_can_be_captured_and_replayed():
    cfg = small_config("graph", T=700, d=256, h=256, E=6, k=2, normalize_topk=1, zipf_s=0.8, seed=501)
    inputs = [make_inputs(cfg), make_inputs(small_config("graph", 700, 256, 256, 6, 2, 1, 0.8, 502))]
    for key in ("w_router", "w1", "w2", "router_bias"):
        inputs[1][key] = inputs[0][key]
    ws = dm.Workspace(cfg.num_tokens, cfg.d_model, cfg.ffn_hidden, cfg.num_experts, cfg.top_k, cfg.normalize_topk)
    w = {k: to_dev(inputs[0][k]) for k in ("w_router", "w1", "w2")}
    bias = torch.from_numpy(inputs[0]["router_bias"]).cuda()
    x, dy = to_dev(inputs[0]["x"]).clone(), to_dev(inputs[0]["dy"]).clone()      # static buffers of the graph

    def step():
        ws.topology(x, w["w_router"], bias)
        ws.forward(x, w["w1"], w["w2"])
        ws.backward(x, w["w_router"], w["w1"], w["w2"], dy)

    def outputs():
        torch.cuda.synchronize()
        topo = ws.topology_arrays()
        return {"y": _bits(ws.y), "dx": _bits(ws.dx), "dw1": _bits(ws.dw1), "dw2": _bits(ws.dw2),
                "dw_router": _bits(ws.dw_router), "row_of": topo["row_of"].clone(),
                "column_indices": topo["column_indices"].clone(), "counts": topo["counts"].clone()}

    def load(i):
        x.copy_(to_dev(inputs[i]["x"]))
        dy.copy_(to_dev(inputs[i]["dy"]))

    eager = []
    for i in range(2):                       # eager results for both inputs (also the warm-up of every kernel variant)
        load(i)
        step()
        eager.append(outputs())
    assert not torch.equal(eager[0]["row_of"], eager[1]["row_of"]), "the two inputs should route differently"

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        step()
    for i in (1, 0, 1):                      # replays with the program's own eager work and synchronisations in between
        load(i)
        for t in (ws.y, ws.dx, ws.dw1, ws.dw2):
            t.view(torch.int16).fill_(0x7FC1)
        ws.dw_router.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        got = outputs()
        for key, ref in eager[i].items():
            assert got[key].shape == ref.shape and torch.equal(got[key], ref), "replay with input %d: %s differs" % (i, key)
