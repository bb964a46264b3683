"""Seeded synthetic workloads for the sparse verification-attention path.

This module only *builds inputs*: it serves both the CPU oracle and the HIP
path and holds none of the method's arithmetic (no block means, no scores, no
top-k, no softmax).  The one place it looks at the queries is to point the
planted key shift along the first draft token's per-KV-head query direction,
which is part of the input recipe, not of the method.

Every tensor is produced from ``torch.Generator`` streams seeded from
``BASE_SEED + 1000 * cfg + layer`` so that CPU tests, GPU tests and the bench
all see the same data for the same (cfg, layer).

Shapes follow the five benchmark configurations:

  cfg 1  fp32  B=1 Hq=8  Hkv=2 d=64  T=1024    Bs=16  gamma=4  k=8   contiguous
  cfg 2  bf16  B=1 Hq=32 Hkv=8 d=128 T=8192    Bs=64  gamma=5  k=16  contiguous
  cfg 3  bf16  B=4 Hq=32 Hkv=8 d=128 T=32768   Bs=64  gamma=8  k=32  pages of 16, 32 layers, anchors every 2nd
  cfg 4  bf16  B=1 Hq=32 Hkv=8 d=128 T=131072  Bs=128 16-node tree, k=32, pages of 64
  cfg 5  bf16  B=8 Hq=32 Hkv=4 d=128 L~U[16384,65536] Bs=64 gamma=6 k=32 pages of 16, 48 layers, anchors every 4th
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import torch

BASE_SEED = 251221911


@dataclasses.dataclass(frozen=True)
class VerifyConfig:
    """Static description of one verification workload (one transformer layer's shape)."""

    name: str
    cfg_id: int
    dtype: str            # "f32" | "bf16"
    B: int
    Hq: int
    Hkv: int
    d: int
    T: int                # maximum prefix length (allocation size per sequence)
    block_size: int
    gamma: int            # number of draft tokens / tree nodes
    k_blocks: int         # budget per (batch, KV-head), in blocks
    page_size: int        # 0 => contiguous [B][T][Hkv][d]
    planted: float        # >=1: absolute number of planted blocks; <1: fraction of the sequence's blocks
    shift: float
    n_layers: int = 1
    anchor_every: int = 1  # layer l is an anchor iff l % anchor_every == 0
    tree_depth: int = 0    # 0 => linear causal drafts
    min_len: int = 0       # 0 => every sequence has length T; else lengths ~ U[min_len, T]
    n_sink: int = 0
    n_local: int = 0

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def nb_max(self) -> int:
        return -(-self.T // self.block_size)

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def is_anchor(self, layer: int) -> bool:
        return layer % self.anchor_every == 0

    def scaled(self, **kw) -> "VerifyConfig":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[int, VerifyConfig] = {
    1: VerifyConfig("cfg1_tiny_f32", 1, "f32", 1, 8, 2, 64, 1024, 16, 4, 8, 0, 3, 2.0),
    2: VerifyConfig("cfg2_llama8b_8k", 2, "bf16", 1, 32, 8, 128, 8192, 64, 5, 16, 0, 0.05, 1.5),
    3: VerifyConfig("cfg3_long_batch_32k", 3, "bf16", 4, 32, 8, 128, 32768, 64, 8, 32, 16, 0.05, 1.5,
                    n_layers=32, anchor_every=2),
    4: VerifyConfig("cfg4_tree_128k", 4, "bf16", 1, 32, 8, 128, 131072, 128, 16, 32, 64, 0.05, 1.5,
                    tree_depth=5),
    5: VerifyConfig("cfg5_moe_varlen", 5, "bf16", 8, 32, 4, 128, 65536, 64, 6, 32, 16, 0.05, 1.5,
                    n_layers=48, anchor_every=4, min_len=16384),
}


def _gen(cfg: VerifyConfig, layer: int, stream: int, device: str) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED + 1000 * cfg.cfg_id + layer + 7919 * stream)
    return g


def seq_lens_for(cfg: VerifyConfig) -> torch.Tensor:
    """Prefix lengths (CPU int32 [B]); shared by all layers of a config."""
    if cfg.min_len <= 0:
        return torch.full((cfg.B,), cfg.T, dtype=torch.int32)
    g = _gen(cfg, 0, 11, "cpu")
    return torch.randint(cfg.min_len, cfg.T + 1, (cfg.B,), generator=g, dtype=torch.int32)


def draft_tree(cfg: VerifyConfig) -> Optional[torch.Tensor]:
    """Parent index per draft node (CPU int64 [gamma], root has parent -1), or None for linear drafts.

    Nodes 0..depth form a chain; every other node picks a uniformly random earlier
    node whose depth is below the maximum, so parents always precede children.
    """
    if cfg.tree_depth <= 0:
        return None
    g = _gen(cfg, 0, 13, "cpu")
    n = cfg.gamma
    parent = [-1] * n
    depth = [0] * n
    for i in range(1, n):
        if i <= cfg.tree_depth:
            p = i - 1
        else:
            cand = [j for j in range(i) if depth[j] < cfg.tree_depth]
            p = cand[int(torch.randint(0, len(cand), (1,), generator=g))]
        parent[i] = p
        depth[i] = depth[p] + 1
    return torch.tensor(parent, dtype=torch.int64)


def mask_from_parents(parent: torch.Tensor) -> List[int]:
    """Ancestor-or-self attention mask per node as Python ints (bit t set: node may attend node t)."""
    masks: List[int] = []
    for i, p in enumerate(parent.tolist()):
        masks.append((1 << i) | (masks[p] if p >= 0 else 0))
    return masks


def causal_masks(gamma: int) -> List[int]:
    return [(1 << (i + 1)) - 1 for i in range(gamma)]


def draft_masks_for(cfg: VerifyConfig) -> List[int]:
    parent = draft_tree(cfg)
    return causal_masks(cfg.gamma) if parent is None else mask_from_parents(parent)


def masks_to_tensor(masks: List[int]) -> torch.Tensor:
    """uint64 bit masks stored in an int64 tensor (two's complement for bit 63)."""
    return torch.tensor([m - (1 << 64) if m >= (1 << 63) else m for m in masks], dtype=torch.int64)


def paging_for(cfg: VerifyConfig, seq_lens: torch.Tensor):
    """Page table for a config: (block_table int32 [B][max_pages], n_pool_pages, poison_page).

    Contiguous configs return (None, B, None).  Paged configs use one global pool in a
    random physical permutation; table entries past a sequence's last page point at a
    dedicated poison page (filled with NaN by ``make_layer``) so that a stray read
    shows up as NaN in the output instead of going out of bounds.
    """
    if cfg.page_size == 0:
        return None, cfg.B, None
    ps = cfg.page_size
    max_pages = -(-cfg.T // ps)
    used = [-(-int(L) // ps) for L in seq_lens.tolist()]
    total = sum(used)
    g = _gen(cfg, 0, 17, "cpu")
    perm = torch.randperm(total, generator=g)
    poison = total
    table = torch.full((cfg.B, max_pages), poison, dtype=torch.int32)
    off = 0
    for b, u in enumerate(used):
        table[b, :u] = perm[off:off + u].to(torch.int32)
        off += u
    return table, total + 1, poison


def planted_blocks(cfg: VerifyConfig, layer: int, seq_lens: torch.Tensor) -> List[List[torch.Tensor]]:
    """Planted block ids per (b, h).  Positions are shared inside a reuse group of layers."""
    group = (layer // cfg.anchor_every) * cfg.anchor_every
    g = _gen(cfg, group, 19, "cpu")
    out: List[List[torch.Tensor]] = []
    for b in range(cfg.B):
        nb = -(-int(seq_lens[b]) // cfg.block_size)
        n_p = int(cfg.planted) if cfg.planted >= 1 else int(round(cfg.planted * nb))
        row = []
        for _h in range(cfg.Hkv):
            row.append(torch.randperm(nb, generator=g)[:n_p].sort().values)
        out.append(row)
    return out


def make_layer(cfg: VerifyConfig, layer: int = 0, device: str = "cpu") -> Dict[str, object]:
    """All inputs of one layer's verification step, already rounded to the config's dtype.

    Returns a dict with
      q         [B][gamma][Hq][d]
      k_pool    [n_pool_pages][page][Hkv][d]  (contiguous: [B][T][Hkv][d]), same for v_pool
      k_draft   [B][gamma][Hkv][d], v_draft
      block_table  int32 [B][max_pages] or None
      seq_lens  int32 [B]
      draft_mask   int64 [gamma] (uint64 bit patterns)
      masks     the same masks as Python ints
      planted   planted block ids per (b, h)
    Random normal draws happen on ``device``; structure (lengths, pages, tree, planted
    positions) always comes from CPU generators so it is identical on both devices.
    """
    dt = cfg.torch_dtype
    seq_lens = seq_lens_for(cfg)
    table, n_pages, poison = paging_for(cfg, seq_lens)
    masks = draft_masks_for(cfg)
    planted = planted_blocks(cfg, layer, seq_lens)
    g = _gen(cfg, layer, 1, device)
    B, Hq, Hkv, d, G = cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.G

    def randn(*shape):
        return torch.randn(*shape, generator=g, device=device, dtype=torch.float32)

    q = randn(B, cfg.gamma, Hq, d).to(dt)
    k_draft = randn(B, cfg.gamma, Hkv, d).to(dt)
    v_draft = randn(B, cfg.gamma, Hkv, d).to(dt)

    # direction of the planted shift: the first draft token's queries, averaged over the
    # query heads that share a KV head, normalised (taken from the dtype-rounded q)
    q0 = q[:, 0].float().view(B, Hkv, G, d).mean(dim=2)
    u = q0 / q0.norm(dim=-1, keepdim=True).clamp_min(1e-20)

    ps = cfg.page_size if cfg.page_size else cfg.T
    k_pool = torch.empty(n_pages, ps, Hkv, d, device=device, dtype=dt)
    v_pool = torch.empty(n_pages, ps, Hkv, d, device=device, dtype=dt)
    if poison is not None:
        k_pool[poison] = float("nan")
        v_pool[poison] = float("nan")
    for b in range(B):
        L = int(seq_lens[b])
        n_pg = -(-L // ps)
        kb = randn(n_pg * ps, Hkv, d)
        vb = randn(n_pg * ps, Hkv, d)
        for h in range(Hkv):
            blocks = planted[b][h].to(device)
            if blocks.numel():
                tok = (blocks[:, None] * cfg.block_size +
                       torch.arange(cfg.block_size, device=device)[None, :]).reshape(-1)
                tok = tok[tok < L]
                kb[tok, h, :] += cfg.shift * u[b, h]
        phys = table[b, :n_pg].to(device).long() if table is not None else torch.tensor([b], device=device)
        k_pool[phys] = kb.view(n_pg, ps, Hkv, d).to(dt)
        v_pool[phys] = vb.view(n_pg, ps, Hkv, d).to(dt)
        del kb, vb

    return {
        "cfg": cfg,
        "layer": layer,
        "q": q,
        "k_pool": k_pool,
        "v_pool": v_pool,
        "k_draft": k_draft,
        "v_draft": v_draft,
        "block_table": table.to(device) if table is not None else None,
        "seq_lens": seq_lens.to(device),
        "draft_mask": masks_to_tensor(masks).to(device),
        "masks": masks,
        "planted": planted,
        "poison_page": poison,
    }


def shrink(cfg: VerifyConfig, T: int, **kw) -> VerifyConfig:
    """A smaller version of a config (same structure, shorter prefix) for fast parity cases."""
    min_len = min(cfg.min_len, T // 4) if cfg.min_len else 0
    return cfg.scaled(T=T, min_len=min_len, **kw)


def algorithmic_bytes(cfg: VerifyConfig, seq_lens: Optional[torch.Tensor] = None) -> Dict[str, int]:
    """Bytes each step of the method must move for one layer (what the roofline is priced on).

    verify_attn: selected K+V, draft K/V, q, out, selected indices and (if paged) the page
                 table entries of the selected blocks.
    score_select: fp32 representatives once, q of draft 0, indices out.
    block_reps:  K once in, fp32 representatives out.
    """
    if seq_lens is None:
        seq_lens = seq_lens_for(cfg)
    e = cfg.elem_bytes
    row = cfg.d * e
    attn = 0
    sel = 0
    reps = 0
    for L in seq_lens.tolist():
        nb = -(-L // cfg.block_size)
        cnt = min(cfg.k_blocks, nb)
        attn += 2 * cfg.Hkv * cnt * cfg.block_size * row          # selected K and V
        attn += cfg.Hkv * cnt * 4                                  # sel_idx
        if cfg.page_size:
            attn += cfg.Hkv * cnt * max(1, cfg.block_size // cfg.page_size) * 4
        sel += cfg.Hkv * nb * cfg.d * 4 + cfg.Hq * row + cfg.Hkv * (cnt + 1) * 4
        reps += L * cfg.Hkv * row + cfg.Hkv * nb * cfg.d * 4
    attn += 2 * cfg.B * cfg.gamma * cfg.Hkv * row                  # draft K and V
    attn += 2 * cfg.B * cfg.gamma * cfg.Hq * row                   # q in, out
    return {"verify_attn": attn, "score_select": sel, "block_reps": reps}
