#!/usr/bin/env python3
"""Benchmark of the MI355X dMoE layer: one step = dmoe_topology + dmoe_forward + dmoe_backward on one batch.

Prints ONE JSON line.  `value` is useful TFLOP/s = 12*T*k*d*h / time (six block-sparse products of 2*T*k*d*h
flops each; padding rows, the router and the permutation kernels are not counted as useful work) with every
input already resident in HBM.  `roofline` describes the slowest block-sparse product of the step, timed with
HIP events recorded around that kernel on the stream it runs on, inside the timed steps.  `cpu_baseline` is the
CPU oracle (fp64 numpy) timed on the host cores, on the whole workload when that takes seconds and on a stated
slice of it (a prefix of the batch's tokens against the full expert weights) for the largest configuration.
The headline is the largest configuration, large_expert_top2; the other four are reported beside it under
`other_workloads`, each with its own timed steps (median and mean) and roofline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config large_expert_top2] [--also tiny,xs,...] [--no-cpu]
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
MATMUL_STAGES = ["sdd", "dsd", "sddt", "dstd", "dsdt", "ddts"]
# Configurations whose block-sparse products are bound by HBM (weights are read once per ~128 rows: about
# 128 flop/byte, below the 312 flop/byte ridge); the others are bound by the MFMA pipes.
HBM_BOUND = {"tiny", "xs"}
# HBM traffic per launch (bytes) of each block-sparse product, from the rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# summaries under profiles/ (dmoe_<workload>_hbm_bytes.txt): FETCH_SIZE * 2.0 + WRITE_SIZE * 1.0 KiB, the factors
# being what the same counters read for a 1 GiB elementwise copy (--copy-calibration) in the same runs.
MEASURED_TRAFFIC = {
    ("xs", "dsdt"): 210515149, ("xs", "sdd"): 260303667, ("xs", "ddts"): 186822042,
    ("xs", "dstd"): 186810778, ("xs", "dsd"): 207908864, ("xs", "sddt"): 260336640,
    ("small_zipf1.0", "ddts"): 988802662, ("small_zipf1.0", "dstd"): 1011044557, ("small_zipf1.0", "dsdt"): 777336422,
    ("small_zipf1.0", "sdd"): 639211315, ("small_zipf1.0", "dsd"): 874702029, ("small_zipf1.0", "sddt"): 639066931,
    ("medium_zipf1.2_top2", "sdd"): 2429830144, ("medium_zipf1.2_top2", "ddts"): 2759092634, ("medium_zipf1.2_top2", "dstd"): 2761476096,
    ("medium_zipf1.2_top2", "sddt"): 2585897779, ("medium_zipf1.2_top2", "dsdt"): 2617261875, ("medium_zipf1.2_top2", "dsd"): 2576706970,
    ("large_expert_top2", "sdd"): 24057967411, ("large_expert_top2", "dsd"): 16102725018, ("large_expert_top2", "dsdt"): 15117702144,
    ("large_expert_top2", "dstd"): 13325429146, ("large_expert_top2", "sddt"): 27807969894, ("large_expert_top2", "ddts"): 13869480960,
}


class HipEvents:
    """Minimal access to hipEvent_* of the HIP runtime that torch already loaded."""

    def __init__(self):
        import torch
        path = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
        self.hip = ctypes.CDLL(path if os.path.exists(path) else "libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        e = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(e))
        assert rc == 0, "hipEventCreate failed: %d" % rc
        return e

    def elapsed_ms(self, a, b) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        assert rc == 0, "hipEventElapsedTime failed: %d" % rc
        return ms.value


def algorithmic_bytes(stage: str, T, k, d, h, E, P, active) -> float:
    """Bytes a kernel must move at least once (bf16 = 2 bytes): its dense operand rows, the weights of the
    experts that own at least one token, the sparse blocks it reads or writes."""
    pd, ph, w = P * d * 2.0, P * h * 2.0, active * d * h * 2.0
    return {
        "sdd": pd + w + 2 * ph,          # read Xp, W1; write H and gelu(H)
        "dsd": ph + w + pd,              # read A, W2; write Yp
        "sddt": pd + w + 2 * ph,         # read dYp, W2, H; write dH
        "dstd": ph + pd + E * d * h * 2.0,   # read A, dYp; write all of dW2 (zeros for empty experts)
        "dsdt": ph + w + pd,             # read dH, W1; write dXp
        "ddts": pd + ph + E * d * h * 2.0,   # read Xp, dH; write all of dW1
    }[stage]


CPU_SLICE_TOKENS = 2048     # tokens of the batch that the oracle is timed on when the whole workload would take minutes


def run_config(cfg, steps, warmup, hipev, with_cpu, verbose=True, accumulate=False):
    import numpy as np
    import torch
    import paper_2211_15841_amd as dm
    from dmoe_inputs import make_inputs

    def log(*a):
        if verbose:
            print(*a, file=sys.stderr, flush=True)

    t0 = time.time()
    inp = make_inputs(cfg)
    log("[bench] %s: inputs drawn in %.1fs" % (cfg.name, time.time() - t0))
    to_dev = lambda b: torch.from_numpy(b.view(np.int16)).cuda().view(torch.bfloat16)
    x, wr, w1, w2, dy = (to_dev(inp[k]) for k in ("x", "w_router", "w1", "w2", "dy"))
    bias = torch.from_numpy(inp["router_bias"]).cuda() if inp["router_bias"] is not None else None
    ws = dm.Workspace(cfg.num_tokens, cfg.d_model, cfg.ffn_hidden, cfg.num_experts, cfg.top_k, cfg.normalize_topk,
                      expert_capacity=cfg.expert_capacity, pad_to_capacity=cfg.pad_to_capacity)

    if accumulate:     # fp32 accumulators of a training loop with gradient accumulation (never zeroed here: timing only)
        acc = [torch.zeros(s_, dtype=torch.float32, device="cuda")
               for s_ in ((cfg.d_model, cfg.num_experts), (cfg.d_model, cfg.num_experts * cfg.ffn_hidden),
                          (cfg.num_experts * cfg.ffn_hidden, cfg.d_model))]

    def step():
        ws.topology(x, wr, bias)
        ws.forward(x, w1, w2)
        if accumulate:
            ws.backward_accumulate(x, wr, w1, w2, dy, *acc)
        else:
            ws.backward(x, wr, w1, w2, dy)

    nst = len(dm.STAGE_NAMES)
    EvArr = ctypes.c_void_p * (2 * nst)

    # -- warm-up, with a per-stage timing pass to find the slowest block-sparse product --------------------
    for _ in range(max(1, warmup // 2)):
        step()
    torch.cuda.synchronize()
    stage_ms = {n: 0.0 for n in dm.STAGE_NAMES}
    nprobe = max(3, warmup - warmup // 2)
    for _ in range(nprobe):
        evs = EvArr(*[hipev.create() for _ in range(2 * nst)])
        dm.dmoe_set_stage_events(evs)
        step()
        dm.dmoe_set_stage_events(None)
        torch.cuda.synchronize()
        for i, n in enumerate(dm.STAGE_NAMES):
            stage_ms[n] += hipev.elapsed_ms(evs[2 * i], evs[2 * i + 1]) / nprobe
        for e in evs:
            hipev.hip.hipEventDestroy(e)
    dominant = max(MATMUL_STAGES, key=lambda n: stage_ms[n])
    di = dm.STAGE_NAMES.index(dominant)

    # -- timed region: exactly `steps` steps, events only around the dominant kernel -----------------------
    ev_sets = []
    for _ in range(steps):
        arr = EvArr()
        arr[2 * di], arr[2 * di + 1] = hipev.create(), hipev.create()
        ev_sets.append(arr)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]   # step boundaries, for the median
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    marks[0].record()
    for i, arr in enumerate(ev_sets):
        dm.dmoe_set_stage_events(arr)
        step()
        marks[i + 1].record()
    dm.dmoe_set_stage_events(None)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    median_ms = 0.5 * (step_ms[(steps - 1) // 2] + step_ms[steps // 2])
    kernel_ms = sum(hipev.elapsed_ms(a[2 * di], a[2 * di + 1]) for a in ev_sets) / steps
    for a in ev_sets:
        hipev.hip.hipEventDestroy(a[2 * di]); hipev.hip.hipEventDestroy(a[2 * di + 1])

    topo = ws.topology_arrays()
    P, R, nnz, _ = (int(v) for v in topo["counts"])
    n_e = topo["tokens_per_expert"].numpy()
    active = int((n_e > 0).sum())
    T, k, d, h, E = cfg.num_tokens, cfg.top_k, cfg.d_model, cfg.ffn_hidden, cfg.num_experts
    ms = elapsed * 1e3 / steps
    useful = cfg.useful_flops
    if cfg.expert_capacity > 0:      # token dropping: only the kept assignments are useful work
        useful = 12.0 * float(n_e.sum()) * d * h
    res = {
        "workload": cfg.name, "steps": steps, "ms_per_step": ms, "ms_per_step_median": median_ms,
        "useful_tflops": useful / (ms * 1e-3) / 1e12,
        "useful_tflops_median": useful / (median_ms * 1e-3) / 1e12,
        "pct_mfma_peak": 100.0 * useful / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "padded_tflops": 12.0 * P * d * h / (ms * 1e-3) / 1e12,
        "P": P, "nnz_blocks": nnz, "active_experts": active, "max_tokens_per_expert": int(n_e.max()),
        "expert_capacity": cfg.expert_capacity, "kept_assignments": int(n_e.sum()),
        "stage_ms": {n: round(v, 5) for n, v in stage_ms.items()},
        "matmul_ms": round(sum(stage_ms[n] for n in MATMUL_STAGES), 5),
    }
    if cfg.name.split("@")[0] in HBM_BOUND:
        ab = algorithmic_bytes(dominant, T, k, d, h, E, P, active)
        ach = ab / (kernel_ms * 1e-3) / 1e9
        res["roofline"] = {"kernel": dominant, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": ach / PEAK_HBM_GBS, "traffic": MEASURED_TRAFFIC.get((cfg.name, dominant)),
                           "kernel_ms": kernel_ms, "algorithmic_bytes": ab}
    else:
        fl = useful / 6.0
        ach = fl / (kernel_ms * 1e-3) / 1e12
        res["roofline"] = {"kernel": dominant, "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                           "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                           "traffic": MEASURED_TRAFFIC.get((cfg.name, dominant)), "kernel_ms": kernel_ms,
                           "algorithmic_flops": fl}
    log("[bench] %s: %.3f ms/step, %.1f useful TFLOP/s (%.1f%% of bf16 peak); stages %s" %
        (cfg.name, ms, res["useful_tflops"], res["pct_mfma_peak"], res["stage_ms"]))

    if with_cpu:
        from threadpoolctl import threadpool_info
        from oracle import dmoe_oracle as orc
        # The oracle as it stands: route + permute + topology + forward + backward in fp64 numpy.  The whole workload
        # when that is seconds of work (repeated until about ten seconds have been timed, at most eight passes);
        # otherwise a slice of it: the first CPU_SLICE_TOKENS tokens of the batch, routed by the same router, against
        # the full expert weights (each token's rows are independent dense computations, so a prefix of the batch is
        # the same work per token; its useful flops are 12 * tokens * k * d * h).
        whole = useful <= 5e12
        n_tok = T if whole else min(T, CPU_SLICE_TOKENS)
        xs_, dys_ = inp["x"][:n_tok], inp["dy"][:n_tok]
        cpu_s, passes = 0.0, 0
        while passes < (8 if whole else 1) and (passes == 0 or cpu_s < 10.0):
            t1 = time.perf_counter()
            logits, idx, w, p = orc.route(xs_, inp["w_router"], inp["router_bias"], k, cfg.normalize_topk)
            n, off, row_of, token_of = orc.permutation(idx, E)
            orc.topology(off, h)
            orc.forward(xs_, inp["w1"], inp["w2"], idx, w, h)
            orc.backward(xs_, inp["w_router"], inp["w1"], inp["w2"], dys_, idx, w, p, h, cfg.normalize_topk)
            cpu_s += time.perf_counter() - t1
            passes += 1
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        cpu_s /= passes
        # backward() recomputes the forward to get its intermediates: 18*tokens*k*d*h flops of matmul in total
        what = ("the whole %s workload" % cfg.name) if whole else \
            ("the first %d of the %d tokens of %s (%d assignments) against all %d experts' full weights"
             % (n_tok, T, cfg.name, n_tok * k, E))
        res["cpu_baseline"] = {"value": 12.0 * n_tok * k * d * h / cpu_s / 1e12, "unit": "TFLOP/s", "cores": threads,
                               "kind": "oracle",
                               "sample": "%s (route + permute + topology + forward + backward, fp64 numpy), %d "
                                         "pass(es) of %.2f s each, host has %d cpus"
                                         % (what, passes, cpu_s, os.cpu_count())}
        log("[bench] %s: oracle %.2f s on %d threads (%s)" % (cfg.name, cpu_s, threads, what))
    del ws, x, wr, w1, w2, dy
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--config", default="large_expert_top2",
                    help="headline workload: name (see dmoe_inputs.CONFIGS) or 1-based index; default = the largest")
    ap.add_argument("--also", default="tiny,xs,small_zipf1.0,medium_zipf1.2_top2,xs@cf1.0",
                    help="comma-separated extra workloads reported under 'other_workloads' ('' for none); "
                         "name@cfF = that workload as the token-dropping MoE of Section 2.2 with capacity factor F, "
                         "every expert padded to its capacity")
    ap.add_argument("--also-steps", type=int, default=30, help="timed steps of each extra workload (>= 20)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-probe", action="store_true",
                    help="skip the register-only MFMA peak probe (keeps its kernel out of rocprofv3 summaries)")
    ap.add_argument("--tile-mode", type=int, default=0, choices=(0, 1, 2, 3),
                    help="0: the library's own tile choice (default); 1 / 2: force 128x128 / 256x256 tiles; 3: 256x256 tiles on the "
                         "two-stage loop instead of the slab ring (experiments)")
    ap.add_argument("--accumulate", action="store_true",
                    help="time dmoe_backward_accumulate (fp32 weight-gradient accumulators) instead of dmoe_backward; "
                         "a variant for context, not the headline step")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel (reference for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from dmoe_inputs import CONFIGS, CONFIG_BY_NAME
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    def pick(name):
        if "@cf" in name:            # expert_capacity = num_tokens * top_k / num_experts * capacity_factor (Section 2.2)
            import dataclasses
            base_name, factor = name.split("@cf")
            base = pick(base_name)
            cap = max(1, int(base.num_tokens * base.top_k / base.num_experts * float(factor)))
            return dataclasses.replace(base, name=name, expert_capacity=cap, pad_to_capacity=1)
        return CONFIGS[int(name) - 1] if name.isdigit() else CONFIG_BY_NAME[name]

    if args.copy_calibration:      # a kernel whose HBM traffic is known: reads 1 GiB, writes 1 GiB
        src = torch.empty(1 << 28, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)   # an elementwise kernel: distinct from the runtime's own copy kernels
        torch.cuda.synchronize()
        del src, dst

    import paper_2211_15841_amd as dm
    if args.tile_mode:
        dm.dmoe_set_tile_mode(args.tile_mode)
    # register-only MFMA loop on this machine (context for % of peak); left out of profiled runs with --no-probe
    measured_peak = None if args.no_probe else dm.dmoe_probe_mfma_tflops()
    # the same instruction on operands that toggle like real data, after half a second of sustained load: the rate
    # and shader clock the device holds under its power management (the published peak assumes 2.4 GHz)
    sustained = (None, None) if args.no_probe else dm.dmoe_probe_mfma_sustained(0.5)
    hipev = HipEvents()
    cfg = pick(args.config)
    main_res = run_config(cfg, args.steps, args.warmup, hipev, with_cpu=not args.no_cpu, accumulate=args.accumulate)
    others = []
    for name in [n for n in args.also.split(",") if n and n != cfg.name]:
        others.append(run_config(pick(name), max(20, args.also_steps), max(6, args.warmup), hipev, with_cpu=False,
                                 accumulate=args.accumulate))

    line = {
        "metric": "dMoE FFN fwd+bwd useful TFLOP/s (bf16) + % MFMA peak, 1 MI355X",
        "value": main_res["useful_tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "ms_per_step_median": main_res["ms_per_step_median"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "num_tokens": cfg.num_tokens, "d_model": cfg.d_model,
                   "ffn_hidden": cfg.ffn_hidden, "num_experts": cfg.num_experts, "top_k": cfg.top_k,
                   "block": 128, "routing": "zipf(%.1f)-biased router" % cfg.zipf_s if cfg.zipf_s else "random router"},
        "backward": "dmoe_backward_accumulate (fp32 accumulators)" if args.accumulate else "dmoe_backward",
        "pct_mfma_peak": main_res["pct_mfma_peak"],
        "mfma_peak_measured_tflops": round(measured_peak, 1) if measured_peak else None,
        "pct_mfma_peak_measured": round(100.0 * main_res["useful_tflops"] / measured_peak, 2) if measured_peak else None,
        "mfma_sustained_tflops": round(sustained[0], 1) if sustained[0] else None,
        "mfma_sustained_shader_ghz": round(sustained[1], 3) if sustained[0] else None,
        "pct_mfma_sustained": round(100.0 * main_res["useful_tflops"] / sustained[0], 2) if sustained[0] else None,
        "roofline": {k: main_res["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")},
        "roofline_kernel": main_res["roofline"]["kernel"], "roofline_kernel_ms": main_res["roofline"]["kernel_ms"],
        "cpu_baseline": main_res.get("cpu_baseline"),
        "detail": {k: main_res[k] for k in ("padded_tflops", "P", "nnz_blocks", "active_experts",
                                            "max_tokens_per_expert", "stage_ms", "matmul_ms")},
        "other_workloads": others,
        "paper_context": "MegaBlocks reports up to 40% end-to-end speedup over Tutel and up to 2.4x over Megatron-LM "
                         "on 8x A100 SXM4 80GB (fp16, CUDA 11.5); no absolute kernel throughput is published",
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
