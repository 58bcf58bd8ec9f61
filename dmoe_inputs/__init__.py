"""Seeded synthetic inputs for the dMoE layer, shared by the CPU oracle's tests and the HIP path's tests.

This module holds no arithmetic of the method itself (no routing, no permutation, no matmul): it only
names the workload shapes and draws the random tensors, so that both sides consume the very same bf16
bit patterns.  The shapes follow the paper's MoE model table (Table 2: 64 experts, top-1, hidden sizes
512/1024/1536 with ffn_hidden = 4 x hidden, Table 1) and the sequence length of Section 3 (1024); the
paper's token stream (The Pile) is replaced by Gaussian activations.

Tensors are returned as numpy uint16 arrays holding bfloat16 bit patterns (round-to-nearest-even from
float32 draws), except the optional router bias, which is float32.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict
import numpy as np

BLOCK = 128


@dataclass(frozen=True)
class Config:
    """One synthetic dMoE layer workload."""
    name: str
    num_tokens: int
    d_model: int
    ffn_hidden: int
    num_experts: int
    top_k: int
    normalize_topk: int = 0      # 1: confidence weights divided by their sum over the k slots
    zipf_s: float = 0.0          # > 0: log-Zipf popularity added to the router logits through the bias
    seed: int = 0
    block: int = BLOCK
    activation: int = 0          # 0: exact (erf) GELU
    expert_capacity: int = 0     # > 0: the token-dropping variant, at most this many assignments per expert
    pad_to_capacity: int = 0     # 1: every expert owns the capacity's worth of rows

    def as_dict(self):
        return asdict(self)

    @property
    def useful_flops(self) -> float:
        """Six matmuls of 2*T*k*d*h flops each (two forward, four backward; Section 5.1)."""
        return 12.0 * self.num_tokens * self.top_k * self.d_model * self.ffn_hidden


# Index i is configuration i+1 of the benchmark list.
CONFIGS = [
    Config("tiny", 1024, 256, 1024, 4, 1, seed=1001),
    Config("xs", 8192, 512, 2048, 64, 1, seed=1002),
    Config("small_zipf1.0", 16384, 1024, 4096, 64, 1, zipf_s=1.0, seed=1003),
    Config("medium_zipf1.2_top2", 16384, 1536, 6144, 64, 2, normalize_topk=1, zipf_s=1.2, seed=1004),
    Config("large_expert_top2", 32768, 4096, 14336, 8, 2, seed=1005),
]
CONFIG_BY_NAME = {c.name: c for c in CONFIGS}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24                              # bounded temporaries for the 0.5 G-element weights
    for s in range(0, n, step):
        m = min(step, n - s)
        v = rng.standard_normal(m, dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        out[s:s + m] = f32_to_bf16_bits(v)
    return out.reshape(shape)


def zipf_bias(rng: np.random.Generator, num_experts: int, s: float) -> np.ndarray:
    """log of a Zipf(s) popularity over a seeded random ranking of the experts, as float32 [E]."""
    rank = rng.permutation(num_experts) + 1
    pop = rank.astype(np.float64) ** (-s)
    pop /= pop.sum()
    return np.log(pop).astype(np.float32)


def make_inputs(cfg: Config, with_grad: bool = True) -> dict:
    """Draw x, w_router, w1, w2, (dy), (router_bias) for `cfg`, in that order, from PCG64(cfg.seed).

    x [T,d] ~ N(0,1); w_router [d,E], w1 [d,E*h], w2 [E*h,d] ~ N(0,0.02); dy [T,d] ~ N(0,1) (the upstream
    gradient); router_bias float32 [E] or None.
    """
    rng = np.random.default_rng(cfg.seed)
    T, d, h, E = cfg.num_tokens, cfg.d_model, cfg.ffn_hidden, cfg.num_experts
    out = {
        "x": _normal_bf16(rng, (T, d), 1.0),
        "w_router": _normal_bf16(rng, (d, E), 0.02),
        "w1": _normal_bf16(rng, (d, E * h), 0.02),
        "w2": _normal_bf16(rng, (E * h, d), 0.02),
    }
    out["dy"] = _normal_bf16(rng, (T, d), 1.0) if with_grad else None
    out["router_bias"] = zipf_bias(rng, E, cfg.zipf_s) if cfg.zipf_s > 0 else None
    return out


def small_config(name="case", T=300, d=128, h=256, E=5, k=2, normalize_topk=0, zipf_s=0.0, seed=7,
                 expert_capacity=0, pad_to_capacity=0) -> Config:
    """Helper for tests: an arbitrary small configuration."""
    return Config(name, T, d, h, E, k, normalize_topk=normalize_topk, zipf_s=zipf_s, seed=seed,
                  expert_capacity=expert_capacity, pad_to_capacity=pad_to_capacity)
