"""Seeded synthetic inputs for the expert-skipping rule (Sec. 3.5) and the acceptance / resampling
rule (Sec. 2.1).  Only builds inputs: none of the rules' arithmetic lives here.

Routing weights: the setting of Sec. 4.3 - 256 routed experts, 8 per token: logits ~ N(0, s^2) per
expert with a per-token temperature, the 8 largest kept, their softmax values renormalised over
the 8 (what a router hands to the experts).
Distributions: the setting of Sec. 4.3 / 4.1 - draft length 4 (or 8), a vocabulary of 129 280 (or
128 256) tokens: target logits ~ N(0, 3^2), draft logits = target logits + N(0, noise^2), both
through a softmax; the draft token is drawn from the draft distribution; uniforms are drawn here
and passed to both implementations.
"""
from __future__ import annotations

import torch

BASE_SEED = 251221911 + 555


def _gen(seed: int, device: str) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED + seed)
    return g


def routing_weights(T: int, k: int = 8, n_experts: int = 256, seed: int = 0, device: str = "cpu") -> torch.Tensor:
    """fp32 [T][k]: the routing weights of the k experts each token is routed to, in router order
    (not sorted by weight)."""
    g = _gen(seed, device)
    temp = torch.exp(0.5 * torch.randn(T, 1, generator=g, device=device))
    logits = torch.randn(T, n_experts, generator=g, device=device) * temp
    top = torch.topk(logits, k, dim=1).values
    w = torch.softmax(top, dim=1)
    perm = torch.argsort(torch.rand(T, k, generator=g, device=device), dim=1)      # router order, not weight order
    return torch.gather(w, 1, perm).contiguous()


def acceptance_inputs(B: int, gamma: int, V: int, noise: float = 0.7, seed: int = 0, device: str = "cpu"):
    """dict(p_target, p_draft fp32 [B][gamma][V], draft_tokens int32 [B][gamma], u_accept fp32 [B][gamma],
    u_resample fp32 [B])."""
    g = _gen(1000 + seed, device)
    lt = 3.0 * torch.randn(B, gamma, V, generator=g, device=device)
    ld = lt + noise * torch.randn(B, gamma, V, generator=g, device=device)
    pt = torch.softmax(lt, dim=-1)
    pd = torch.softmax(ld, dim=-1)
    tok = torch.multinomial(pd.reshape(-1, V), 1, generator=g).reshape(B, gamma).to(torch.int32)
    ua = torch.rand(B, gamma, generator=g, device=device)
    ur = torch.rand(B, generator=g, device=device)
    return {"p_target": pt.contiguous(), "p_draft": pd.contiguous(), "draft_tokens": tok, "u_accept": ua, "u_resample": ur}
