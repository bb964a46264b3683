"""Seeded synthetic inputs for the sparse feed-forward verification (Sec. 3.4).

Only builds inputs (serves both the CPU oracle and the HIP path) and holds none of the method's
arithmetic: no projections, no activation, no threshold.

A gated feed-forward layer: x [M][d_model] (the draft tokens' hidden states), w_gate and w_up
[d_ff][d_model], w_down_t [d_ff][d_model] (the down projection stored channel-major: row i is
what hidden channel i adds to the output), optional biases.  Weights and x are bf16, biases fp32.

Value recipe.  x ~ N(0, 1); w_up rows ~ N(0, 1/d_model); w_down_t ~ N(0, 1/d_ff).  The gate
rows carry a per-channel scale: row c ~ N(0, s_c^2 / d_model) with ln s_c ~ N(-1.6, 1.5^2), so
that the gate pre-activation of channel c is ~ N(0, s_c^2) for every token.  That spread of
scales is fitted to the mean FFN sparsity the paper reports for its thresholds (Table 3:
tau = 0.01 / 0.05 / 0.1 -> 0.18 / 0.47 / 0.64 with SiLU), and, like a trained model's "mostly
quiet" channels, it makes the same channels fall under the threshold for all draft tokens of a
step - which is what lets a verification step skip their weights.

Shapes:
  1  tiny          M=3   d_model=128   d_ff=96     SiLU, biases
  2  expert        M=8   d_model=2048  d_ff=768    one expert of the MoE model of Sec. 4.2 (SFFN is applied per expert)
  3  dense_8b      M=8   d_model=4096  d_ff=14336  the feed-forward layer of the 8B target model of Sec. 4.1 (bench)
  4  dense_8b_tree M=60  d_model=4096  d_ff=14336  the same under a 60-node draft tree
"""
from __future__ import annotations

import dataclasses
from typing import Dict

import torch

BASE_SEED = 251221911 + 77

GATE_LOG_SCALE_MEAN = -1.6
GATE_LOG_SCALE_STD = 1.5


@dataclasses.dataclass(frozen=True)
class FfnConfig:
    name: str
    cfg_id: int
    M: int
    d_model: int
    d_ff: int
    act: str = "silu"          # "silu" | "gelu"
    bias: bool = False
    tau: float = 0.05

    def scaled(self, **kw) -> "FfnConfig":
        return dataclasses.replace(self, **kw)


FFN_CONFIGS: Dict[int, FfnConfig] = {
    1: FfnConfig("ffn1_tiny", 1, 3, 128, 96, "silu", True, 0.05),
    2: FfnConfig("ffn2_expert", 2, 8, 2048, 768),
    3: FfnConfig("ffn3_dense_8b", 3, 8, 4096, 14336),
    4: FfnConfig("ffn4_dense_8b_tree", 4, 60, 4096, 14336),
}


def _gen(cfg: FfnConfig, layer: int, stream: int, device: str) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED + 1000 * cfg.cfg_id + layer + 7919 * stream)
    return g


def make_ffn(cfg: FfnConfig, layer: int = 0, device: str = "cpu") -> Dict[str, object]:
    """Inputs of one layer.  The same (cfg, layer, device kind) always gives the same tensors; CPU and
    GPU generators differ, so a comparison must move one side's tensors to the other."""
    def randn(stream, *shape):
        return torch.randn(*shape, generator=_gen(cfg, layer, stream, device), device=device, dtype=torch.float32)

    dm, df = cfg.d_model, cfg.d_ff
    x = randn(1, cfg.M, dm).to(torch.bfloat16)
    scale = torch.exp(GATE_LOG_SCALE_MEAN + GATE_LOG_SCALE_STD * randn(2, df, 1))
    w_gate = (randn(3, df, dm) * (scale / dm ** 0.5)).to(torch.bfloat16)
    w_up = (randn(4, df, dm) / dm ** 0.5).to(torch.bfloat16)
    w_down_t = (randn(5, df, dm) / df ** 0.5).to(torch.bfloat16)
    out = {"x": x, "w_gate": w_gate, "w_up": w_up, "w_down_t": w_down_t, "b_gate": None, "b_up": None, "b_down": None}
    if cfg.bias:
        out["b_gate"] = randn(6, df) * 0.02
        out["b_up"] = randn(7, df) * 0.1
        out["b_down"] = randn(8, dm) * 0.1
    return out


def weight_bytes(cfg: FfnConfig) -> int:
    """Bytes of the three weight matrices (what a dense layer must read)."""
    return 3 * cfg.d_ff * cfg.d_model * 2
