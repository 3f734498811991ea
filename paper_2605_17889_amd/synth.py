"""Seeded synthetic inputs for one MoE layer.

This module only draws random tensors of the stated shapes and distributions. It holds
none of the layer's arithmetic (no routing, no FFN): both the CPU oracle's tests and the
HIP path's tests/bench consume the same bytes produced here.

Shapes follow the five benchmark configurations: a Tiny layer, a Mixtral-8x7B-shaped
batched decode step, a Mixtral-8x22B-shaped prefill chunk, the coalesced-vs-micro-batched
comparison, and the Zipf(1.2)-skewed routing case; two more presets have many small experts. The paper's own workloads are real
checkpoints (Mixtral-8x7B-Instruct, DeepSeek-V2-Lite, Qwen3-30B-A3B; Section 6.1) and a
BIG-Bench-Hard expert-load histogram (Fig. 3(c)); none of those are available, so these
random layers of the same shape and a Zipf-shaped expert load stand in for them.

Distributions: x ~ N(0,1) rounded to bf16; router W_r[d,E] ~ N(0,0.02) fp32;
W1,W3[E,f,d], W2[E,d,f] ~ N(0,0.02) rounded to bf16; optional per-expert router bias.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Callable, Dict, Optional, Sequence

import torch


@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int               # tokens in the ordinary (coalesced) batch
    d_model: int         # paper's d_h
    d_ff: int            # paper's d_e
    E: int               # experts
    k: int               # experts selected per token
    seed: int
    micro_tokens: Optional[int] = None   # m of the micro-batched comparison, if any
    zipf_s: Optional[float] = None       # exponent of the target expert-load law, if skewed
    empty_expert: bool = False           # skewed variant in which one expert gets no token

    @property
    def R(self) -> int:                  # routed rows
        return self.T * self.k

    def with_T(self, T: int) -> "LayerConfig":
        return replace(self, T=T)


PRESETS: Dict[str, LayerConfig] = {
    "tiny": LayerConfig("tiny", 256, 512, 1024, 8, 2, seed=0),
    "mixtral8x7b_decode": LayerConfig("mixtral8x7b_decode", 256, 4096, 14336, 8, 2, seed=1),
    "mixtral8x22b_prefill": LayerConfig("mixtral8x22b_prefill", 8192, 6144, 16384, 8, 2, seed=2),
    "mixtral8x22b_coalesce": LayerConfig("mixtral8x22b_coalesce", 4096, 6144, 16384, 8, 2, seed=3,
                                         micro_tokens=256),
    "mixtral8x22b_zipf": LayerConfig("mixtral8x22b_zipf", 16384, 6144, 16384, 8, 2, seed=4,
                                     zipf_s=1.2),
    "mixtral8x22b_zipf_empty": LayerConfig("mixtral8x22b_zipf_empty", 16384, 6144, 16384, 8, 2,
                                           seed=5, zipf_s=1.2, empty_expert=True),
    # Layers with numerous smaller experts, shaped like the paper's other two models
    # (Section 6.1). The paper prints no dimensions; these are the public model cards' values:
    # Qwen3-30B-A3B: hidden 2048, expert dim 768, 128 experts, top-8; DeepSeek-V2-Lite: hidden
    # 2048, expert dim 1408, 64 routed experts, top-6 (its two always-on shared experts are a
    # plain dense FFN and not part of the routed path).
    "qwen3_30b_a3b_prefill": LayerConfig("qwen3_30b_a3b_prefill", 8192, 2048, 768, 128, 8, seed=6),
    "deepseek_v2_lite_prefill": LayerConfig("deepseek_v2_lite_prefill", 8192, 2048, 1408, 64, 6,
                                            seed=7),
}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _normal_bf16(shape, std: float, gen: torch.Generator, device) -> torch.Tensor:
    """N(0, std) drawn in fp32, rounded to bf16 (round-to-nearest-even)."""
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    n = flat.numel()
    step = 1 << 26                        # bound the fp32 temporary to 256 MiB
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        t = torch.randn(hi - lo, generator=gen, device=device, dtype=torch.float32)
        if std != 1.0:
            t.mul_(std)
        flat[lo:hi] = t.to(torch.bfloat16)
    return out


def make_tokens(cfg: LayerConfig, device="cpu", T: Optional[int] = None) -> torch.Tensor:
    """x[T, d_model] bf16 ~ N(0,1)."""
    T = cfg.T if T is None else T
    return _normal_bf16((T, cfg.d_model), 1.0, _gen(device, cfg.seed * 1000 + 1), device)


def make_router(cfg: LayerConfig, device="cpu") -> torch.Tensor:
    """W_r[d_model, E] fp32 ~ N(0, 0.02)."""
    g = _gen(device, cfg.seed * 1000 + 2)
    return torch.randn((cfg.d_model, cfg.E), generator=g, device=device, dtype=torch.float32) * 0.02


def make_experts(cfg: LayerConfig, device="cpu"):
    """(W1[E,f,d], W3[E,f,d], W2[E,d,f]) bf16 ~ N(0, 0.02)."""
    E, f, d = cfg.E, cfg.d_ff, cfg.d_model
    W1 = _normal_bf16((E, f, d), 0.02, _gen(device, cfg.seed * 1000 + 3), device)
    W3 = _normal_bf16((E, f, d), 0.02, _gen(device, cfg.seed * 1000 + 4), device)
    W2 = _normal_bf16((E, d, f), 0.02, _gen(device, cfg.seed * 1000 + 5), device)
    return W1, W3, W2


def make_layer(cfg: LayerConfig, device="cpu") -> Dict[str, torch.Tensor]:
    """All tensors of one layer. `bias` is None here; skewed configs attach it with
    `calibrate_expert_bias` because the calibration needs a routing count callback."""
    W1, W3, W2 = make_experts(cfg, device)
    return {"x": make_tokens(cfg, device), "w_router": make_router(cfg, device), "bias": None,
            "W1": W1, "W3": W3, "W2": W2}


def zipf_target_counts(cfg: LayerConfig) -> torch.Tensor:
    """Target routed-row count per expert: proportional to rank^(-s) over the experts that
    receive tokens, summing to T*k, ranks assigned to experts by a seeded shuffle. With
    `empty_expert`, the expert shuffled to the last position gets zero."""
    assert cfg.zipf_s is not None
    g = _gen("cpu", cfg.seed * 1000 + 6)
    order = torch.randperm(cfg.E, generator=g)
    n_live = cfg.E - 1 if cfg.empty_expert else cfg.E
    share = torch.tensor([(r + 1) ** (-cfg.zipf_s) for r in range(n_live)], dtype=torch.float64)
    share = share / share.sum()
    target = torch.zeros(cfg.E, dtype=torch.float64)
    target[order[:n_live]] = share * cfg.R
    return target


def calibrate_expert_bias(cfg: LayerConfig, count_fn: Callable[[torch.Tensor], Sequence[int]],
                          rel_tol: float = 0.01, max_iter: int = 200) -> torch.Tensor:
    """Per-expert router bias (fp32[E], CPU) under which the expert load follows the Zipf
    target. `count_fn(bias)` must return the per-expert routed-row counts that the caller's
    router produces with that bias; this function only runs the damped fixed-point update
    bias_e += step*log(target_e/count_e) (step 0.5, shrinking) and returns the best bias seen,
    stopping once every live expert is within `rel_tol`."""
    target = zipf_target_counts(cfg)
    live = target > 0
    bias = torch.zeros(cfg.E, dtype=torch.float32)
    bias[~live] = -1.0e9
    best, best_err, step = bias.clone(), float("inf"), 0.5
    for it in range(max_iter):
        counts = torch.as_tensor(list(count_fn(bias)), dtype=torch.float64)
        err = ((counts - target).abs() / target.clamp(min=1.0))[live].max().item()
        if counts[~live].sum().item() == 0 and err < best_err:
            best, best_err = bias.clone(), err
        if best_err <= rel_tol:
            break
        upd = torch.log(target[live] / counts[live].clamp(min=0.5))
        bias[live] = (bias[live].double() + step * upd).float()
        bias[live] -= bias[live].mean()          # the routing is invariant to a common shift
        if it % 20 == 19:
            step *= 0.7                          # shrink the step if the iteration keeps hunting
    return best


def expert_ffn_flops(R: int, d_model: int, d_ff: int) -> int:
    """FLOPs of the three expert GEMMs over R routed rows (Table 1, row 3: 6*rows*d_h*d_e)."""
    return 6 * R * d_model * d_ff


def expert_weight_bytes(E: int, d_model: int, d_ff: int) -> int:
    """bf16 bytes of one layer's expert weights (Table 1, row 3: 6*d_h*d_e per expert)."""
    return 6 * d_model * d_ff * E


def bf16_bits(t: torch.Tensor):
    """numpy uint16 view of a bf16 tensor's raw bits (host copy)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view("uint16")
