"""Seeded synthetic inputs for the MoTE layer: shapes, value distributions and routing
structure of the five benchmark configurations.

This module only draws random tensors.  It holds none of the method's arithmetic
(no quantiser, no softmax, no top-k, no expert evaluation) and is the one module
that the CPU oracle's tests and the GPU path's tests / benchmark both use.

Every tensor comes from its own torch CPU generator whose seed is a fixed function of
(config seed, tensor tag, expert, matrix), so any tensor can be drawn alone and in any
order -- large configurations never need all latent weights in memory at once.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch


@dataclass(frozen=True)
class MoteConfig:
    name: str
    d_model: int
    d_ff: int
    n_experts: int
    top_k: int
    n_tokens: int
    seed: int
    sigma_shared: float = 0.02     # std of the bf16 shared-expert weights
    sigma_latent: float = 0.02     # std of the fp32 latent routed-expert weights
    outlier_channels: int = 0      # channels of x scaled by outlier_scale
    outlier_scale: float = 20.0
    bias_kind: str = "none"        # "none" | "subset" | "zipf"
    bias_subset: int = 0           # "subset": number of experts that can be selected
    zipf_s: float = 1.2            # "zipf": exponent
    zipf_tau: float = 1.0          # "zipf": temperature on the log-rank bias
    x_seed: int = -1               # >= 0: draw x from this seed instead of `seed` (weights unchanged)
    d_ff_shared: int = 0           # hidden width of the shared expert; 0: the same as d_ff (all benchmark shapes)

    @property
    def f_shared(self) -> int:
        return self.d_ff_shared or self.d_ff

    def with_tokens(self, n_tokens: int, **kw) -> "MoteConfig":
        return replace(self, n_tokens=n_tokens, **kw)


# The five configurations of the benchmark definition.
C1 = MoteConfig("c1_tiny", 256, 512, 4, 2, 64, seed=0)
C2 = MoteConfig("c2_qwen0.5b", 896, 4864, 8, 2, 2048, seed=1, sigma_shared=0.012,
                outlier_channels=4)
C3 = MoteConfig("c3_qwen3b_prefill", 2048, 11008, 16, 2, 8192, seed=2, sigma_shared=0.015)
C4 = MoteConfig("c4_qwen3b_decode", 2048, 11008, 16, 2, 64, seed=2, sigma_shared=0.015,
                bias_kind="subset", bias_subset=16)
C5 = MoteConfig("c5_qwen7b_skew", 3584, 18944, 16, 2, 16384, seed=4, sigma_shared=0.01,
                bias_kind="zipf", zipf_tau=0.45)
# The paper's own layer (Section 4.1, Figure 1): four routed ternary experts, top-1 gating, one
# shared expert, sequences of 2048 tokens, at the Qwen2.5-0.5B / 1.5B / 3B widths.
P05 = MoteConfig("paper_0.5b_top1", 896, 4864, 4, 1, 2048, seed=21, sigma_shared=0.012)
P15 = MoteConfig("paper_1.5b_top1", 1536, 8960, 4, 1, 2048, seed=22, sigma_shared=0.012)
P3 = MoteConfig("paper_3b_top1", 2048, 11008, 4, 1, 2048, seed=23, sigma_shared=0.012)

CONFIGS = {c.name: c for c in (C1, C2, C3, C4, C5, P05, P15, P3)}


# x seeds for which the decode batch really touches all n_distinct selectable experts
_DECODE_X_SEEDS = {(16, 16): 10}


def decode_config(n_tokens: int, n_distinct: int) -> MoteConfig:
    """C4 at batch n_tokens (same weights as C3), router biased so that only n_distinct
    experts are selectable; x is drawn from a seed for which all of them are hit."""
    return replace(C4, name=f"c4_decode_T{n_tokens}_n{n_distinct}", n_tokens=n_tokens,
                   bias_subset=n_distinct, x_seed=_DECODE_X_SEEDS.get((n_tokens, n_distinct), 0))


_TAGS = {"x": 1, "router": 2, "shared": 3, "latent": 4, "outlier": 5, "bias": 6}


def _gen(cfg: MoteConfig, tag: str, a: int = 0, b: int = 0) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(((cfg.seed * 1_000_003 + _TAGS[tag]) * 1_009 + a) * 7 + b)
    return g


def make_x(cfg: MoteConfig) -> torch.Tensor:
    """Hidden states entering the layer: bf16 [T, d], N(0,1); optional outlier channels."""
    g = _gen(cfg, "x") if cfg.x_seed < 0 else _gen(replace(cfg, seed=1000 + cfg.x_seed), "x")
    x = torch.randn(cfg.n_tokens, cfg.d_model, generator=g, dtype=torch.float32)
    if cfg.outlier_channels:
        ch = torch.randperm(cfg.d_model, generator=_gen(cfg, "outlier"))[: cfg.outlier_channels]
        x[:, ch] *= cfg.outlier_scale
    return x.to(torch.bfloat16)


def make_router(cfg: MoteConfig) -> torch.Tensor:
    """Router projection bf16 [d, E], N(0, 1/sqrt(d)) so that logits are about N(0,1)."""
    w = torch.randn(cfg.d_model, cfg.n_experts, generator=_gen(cfg, "router"), dtype=torch.float32)
    return (w * cfg.d_model ** -0.5).to(torch.bfloat16)


def make_router_bias(cfg: MoteConfig):
    """fp32 [E] additive logit bias shaping the synthetic routing, or None.

    "subset": +30 on a seeded subset of bias_subset experts (decode: a step touches
    exactly that many distinct experts once enough tokens are present).
    "zipf":   -tau * s * ln(rank_e) with a seeded rank permutation (skewed loads)."""
    if cfg.bias_kind == "none":
        return None
    perm = torch.randperm(cfg.n_experts, generator=_gen(cfg, "bias"))
    bias = torch.zeros(cfg.n_experts, dtype=torch.float32)
    if cfg.bias_kind == "subset":
        bias[perm[: cfg.bias_subset]] = 30.0
    elif cfg.bias_kind == "zipf":
        rank = torch.empty(cfg.n_experts, dtype=torch.float32)
        rank[perm] = torch.arange(1, cfg.n_experts + 1, dtype=torch.float32)
        bias = -cfg.zipf_tau * cfg.zipf_s * torch.log(rank)
    else:
        raise ValueError(cfg.bias_kind)
    return bias


def make_shared(cfg: MoteConfig):
    """Shared expert, bf16: W_gate [F,d], W_up [F,d], W_down [d,F], N(0, sigma_shared)."""
    shapes = [(cfg.f_shared, cfg.d_model), (cfg.f_shared, cfg.d_model), (cfg.d_model, cfg.f_shared)]
    return tuple(
        (torch.randn(*s, generator=_gen(cfg, "shared", m), dtype=torch.float32) * cfg.sigma_shared)
        .to(torch.bfloat16) for m, s in enumerate(shapes))


def make_latent(cfg: MoteConfig, expert: int, matrix: int) -> torch.Tensor:
    """fp32 latent weights of one routed-expert matrix (0 gate [F,d], 1 up [F,d], 2 down [d,F]),
    N(0, sigma_latent).  Ternarised by the code under test, never here."""
    shape = (cfg.d_ff, cfg.d_model) if matrix < 2 else (cfg.d_model, cfg.d_ff)
    return torch.randn(*shape, generator=_gen(cfg, "latent", expert, matrix),
                       dtype=torch.float32) * cfg.sigma_latent


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """torch bf16 tensor -> numpy uint16 bit patterns (a view, no arithmetic)."""
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)
