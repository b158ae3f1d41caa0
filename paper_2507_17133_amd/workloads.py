"""Seeded synthetic inputs for one BrownoutMoE layer.

This module only draws random tensors of the stated shapes and distributions;
it contains none of the method's arithmetic (no gating, no routing, no FFN), so
the GPU library, the tests and the CPU oracle's callers can all take their
inputs from it.

Recipe (one torch.Generator per tensor, seeded ``seed*1000 + tensor_id`` on the
device the tensor is created on, so a tensor does not depend on which others
were drawn):
  x        [T,d]    N(0,1), stored bf16
  gate_w   [m,d]    N(0,1/d) fp32 (row i = centroid e_i), times alpha if skewed
  gate_b   [m]      ln p_pi(i) fp32 if skewed, else None
  w1,w3    [n,F,d]  N(0,1/d) bf16       w2 [n,d,F]  N(0,1/d) bf16
Skewed expert popularity: p_r ~ r^(-s) over ranks r=1..m, assigned to experts by
a seeded permutation pi (hot experts are not contiguous, which matters because
united-expert groups are contiguous in index); logits become alpha*(x.e_i) +
ln p_pi(i) with alpha = pi/sqrt(6), i.e. Gaussian noise with the variance of a
Gumbel variable, so top-K picks approximate sampling without replacement from p.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Optional, Tuple

import torch

_TID = {"x": 1, "gate_w": 2, "perm": 3, "w1": 4, "w3": 5, "w2": 6, "uw1": 7, "uw3": 8, "uw2": 9,
        "sw1": 10, "sw3": 11, "sw2": 12, "calib": 13}


@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int
    d: int
    F: int
    m: int
    K: int
    way: int
    n_shared: int = 0
    F_s: int = 0
    score_fn: int = 0            # 0 softmax over the K winners, 1 sigmoid renormalised
    zipf_s: Optional[float] = None
    brownout_fractions: Tuple[float, ...] = (0.0,)

    @property
    def G(self) -> int:
        return (self.m + self.way - 1) // self.way

    def with_(self, **kw) -> "LayerConfig":
        return replace(self, **kw)


CONFIGS = {
    "tiny": LayerConfig("tiny", T=64, d=256, F=512, m=8, K=2, way=8, brownout_fractions=(0.0, 0.25, 1.0)),
    "mixtral_prefill": LayerConfig("mixtral_prefill", T=4096, d=4096, F=14336, m=8, K=2, way=8,
                                   zipf_s=1.2, brownout_fractions=(0.3, 0.0)),
    "qwen3_30b_a3b": LayerConfig("qwen3_30b_a3b", T=8192, d=2048, F=768, m=128, K=8, way=8,
                                 zipf_s=1.0, brownout_fractions=(0.0, 0.5)),
    "mixtral_decode": LayerConfig("mixtral_decode", T=256, d=4096, F=14336, m=8, K=2, way=8,
                                  brownout_fractions=(0.0, 0.25, 0.5, 0.75, 1.0)),
    "deepseek_v3": LayerConfig("deepseek_v3", T=16384, d=7168, F=2048, m=256, K=8, way=8,
                               n_shared=1, F_s=2048, score_fn=1, zipf_s=1.1,
                               brownout_fractions=(0.4, 0.0)),
    # The paper's own evaluation model (Model and server configurations): 60 routed experts per layer.
    # The other dimensions are those of the public Qwen1.5-MoE-A2.7B model card (hidden 2048, expert
    # width 1408, top-4, one shared expert of width 5632; its sigmoid gate on the shared output is not
    # modelled: the shared expert enters with weight 1).  way = 8 leaves a ragged last group of 4.
    # The paper's (way, threshold) settings (2, 0), (4, 0.2), (8, 0.4) are fractions 1.0, 0.8, 0.6.
    "qwen15_moe_a27b": LayerConfig("qwen15_moe_a27b", T=8192, d=2048, F=1408, m=60, K=4, way=8,
                                   n_shared=1, F_s=5632, zipf_s=1.0, brownout_fractions=(0.6, 0.0)),
}


def _gen(seed: int, name: str, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000 + _TID[name])
    return g


def _normal_bf16(shape, std: float, seed: int, name: str, device) -> torch.Tensor:
    """N(0,std^2) in bf16, drawn slab by slab along dim 0 to bound the fp32 temporary."""
    g = _gen(seed, name, device)
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    if len(shape) == 3:
        for i in range(shape[0]):
            out[i] = (torch.randn(shape[1:], generator=g, device=device, dtype=torch.float32) * std).to(torch.bfloat16)
    else:
        out.copy_((torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std).to(torch.bfloat16))
    return out


@dataclass
class Layer:
    cfg: LayerConfig
    x: torch.Tensor
    gate_w: torch.Tensor
    gate_b: Optional[torch.Tensor]
    experts: Tuple[torch.Tensor, torch.Tensor, torch.Tensor]
    shared: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = None
    popularity: Optional[torch.Tensor] = field(default=None)


def make_activations(cfg: LayerConfig, seed: int = 0, device="cpu", name: str = "x", n: Optional[int] = None):
    n = cfg.T if n is None else n
    return _normal_bf16((n, cfg.d), 1.0, seed, name, device)


def make_gate(cfg: LayerConfig, seed: int = 0, device="cpu"):
    g = _gen(seed, "gate_w", device)
    gate_w = torch.randn((cfg.m, cfg.d), generator=g, device=device, dtype=torch.float32) / math.sqrt(cfg.d)
    if cfg.zipf_s is None:
        return gate_w, None, None
    gp = _gen(seed, "perm", "cpu")
    perm = torch.randperm(cfg.m, generator=gp)                    # expert i has popularity rank perm[i]+1
    p = (perm.to(torch.float64) + 1.0) ** (-float(cfg.zipf_s))
    p = p / p.sum()
    gate_b = torch.log(p).to(torch.float32).to(device)
    gate_w = gate_w * (math.pi / math.sqrt(6.0))
    return gate_w, gate_b, p


def make_ffn_weights(n: int, d: int, F: int, seed: int, prefix: str, device="cpu"):
    """n SwiGLU experts: (w1 [n,F,d], w3 [n,F,d], w2 [n,d,F]), each N(0,1/d), bf16."""
    std = 1.0 / math.sqrt(d)
    w1 = _normal_bf16((n, F, d), std, seed, prefix + "w1", device)
    w3 = _normal_bf16((n, F, d), std, seed, prefix + "w3", device)
    w2 = _normal_bf16((n, d, F), std, seed, prefix + "w2", device)
    return w1, w3, w2


def make_layer(cfg: LayerConfig, seed: int = 0, device="cpu") -> Layer:
    x = make_activations(cfg, seed, device)
    gate_w, gate_b, p = make_gate(cfg, seed, device)
    experts = make_ffn_weights(cfg.m, cfg.d, cfg.F, seed, "", device)
    shared = make_ffn_weights(cfg.n_shared, cfg.d, cfg.F_s, seed, "s", device) if cfg.n_shared else None
    return Layer(cfg, x, gate_w, gate_b, experts, shared, p)


def make_random_united(cfg: LayerConfig, seed: int = 0, device="cpu"):
    """G united experts with independent random weights (the forward pass accepts any)."""
    return make_ffn_weights(cfg.G, cfg.d, cfg.F, seed, "u", device)
