"""CPU oracle for the sparse verification-attention step of "Accelerate Speculative
Decoding with Sparse Computation in Verification" (Sec. 3.1-3.3).

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, fp64 numpy statement of what
the path computes, used by the tests, the smoke check and the bench's CPU-baseline
leg.  The product (the HIP library and its Python binding) never imports it, and it
imports nothing from the product.  It shares no code, tables or helpers with the
HIP path.

What each function follows:

  block_reps            Sec. 3.1, block partition (Eq. 4) and the block term of Eq. 5:
                        the representative of block (h, j) is the mean of its keys.
  first_query           Sec. 2.2: the first draft token drives retrieval; with grouped
                        query heads the queries sharing a KV head are averaged.
  block_scores          Eq. 5 with the mean taken first (equal by linearity).
  block_scores_literal  Eq. 5 term by term: sum over the block of q0 . k, divided by the
                        block's token count (the reading taken) or by B (as printed).
  near_tie_blocks       which blocks a selection may differ in without being wrong
                        (scores within a relative gap of the weakest block kept for
                        its score; forced first/last blocks excluded).
  select_blocks         Sec. 3.1: top-N scores, first/last blocks never evicted; one
                        set per (batch, KV head) shared by all draft tokens (Sec. 2.2).
  verify_attn           Sec. 3.1/3.3: the draft tokens attend to the selected blocks
                        and, through the draft mask, to each other; one joint softmax.
  dense_attn            the same with every prefix block kept (Sec. 3.2: no eviction).
  budget_blocks         Eq. 6, per KV head, in blocks.
  anchor_of             Eq. 9: nearest preceding anchor layer (an anchor uses itself).
  verify_step           one layer: retrieve on anchors, reuse otherwise, then attend.

Readings taken where the paper is silent are listed in the design notes of the
repository (partial last block divides by its real token count; ties go to the
lowest block index; forced blocks count inside the budget; scores are unscaled;
softmax scale defaults to 1/sqrt(d); a query row with no visible key gets a zero
output and lse = -inf).

Pinned by tests/test_oracle_pins.py against: an independent loop-level brute force,
torch's scaled_dot_product_attention in fp64, closed forms (Eq. 5 linearity, Eq. 6
sparsity), invariants (weights sum to one, page permutation, unselected blocks) and
the sparsity figures of Table 2.  Absolute attention values on the paper's own
workloads are "parity unpinned": the paper prints none.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------- layout

def _f64(a) -> np.ndarray:
    """Exact fp64 view of an input (numpy array or CPU torch tensor, fp32 or bf16)."""
    if isinstance(a, np.ndarray):
        return a.astype(np.float64, copy=False)
    import torch  # inputs may arrive as torch tensors; no torch arithmetic is used
    return a.detach().to("cpu").to(torch.float64).numpy()


def _ints(a) -> np.ndarray:
    if isinstance(a, np.ndarray):
        return a.astype(np.int64)
    return np.asarray(a.detach().to("cpu").numpy() if hasattr(a, "detach") else a, dtype=np.int64)


class PagedCache:
    """Logical view of a (possibly paged) cache pool[page][tok][Hkv][d].

    Token t of sequence b lives in physical page block_table[b][t // page] at slot
    t % page.  A contiguous cache [B][T][Hkv][d] is the special case of one page per
    sequence (block_table None).
    """

    def __init__(self, pool, block_table=None):
        self.pool = pool                      # kept in its own dtype; converted per slice
        self.page = int(pool.shape[1])
        self.Hkv = int(pool.shape[2])
        self.d = int(pool.shape[3])
        self.table = None if block_table is None else _ints(block_table)

    def tokens(self, b: int, t0: int, t1: int) -> np.ndarray:
        """fp64 array [t1-t0][Hkv][d] of logical tokens t0..t1-1 of sequence b."""
        out = np.empty((t1 - t0, self.Hkv, self.d), dtype=np.float64)
        t = t0
        while t < t1:
            p, s = divmod(t, self.page)
            n = min(self.page - s, t1 - t)
            phys = b if self.table is None else int(self.table[b, p])
            out[t - t0:t - t0 + n] = _f64(self.pool[phys, s:s + n])
            t += n
        return out


# --------------------------------------------------------------------------- Eq. 4-5

def n_blocks(L: int, block_size: int) -> int:
    return -(-int(L) // block_size)


def block_reps(k_pool, block_table, seq_lens, block_size: int, nb_max: Optional[int] = None) -> np.ndarray:
    """Mean key of every block: reps[b][h][j][:] (fp64); rows j >= ceil(L_b/Bs) stay zero."""
    cache = PagedCache(k_pool, block_table)
    lens = _ints(seq_lens)
    B = len(lens)
    if nb_max is None:
        nb_max = max(n_blocks(L, block_size) for L in lens)
    reps = np.zeros((B, cache.Hkv, nb_max, cache.d), dtype=np.float64)
    for b in range(B):
        L = int(lens[b])
        for j in range(n_blocks(L, block_size)):
            t0 = j * block_size
            t1 = min(t0 + block_size, L)
            keys = cache.tokens(b, t0, t1)                 # [n_j][Hkv][d]
            reps[b, :, j, :] = keys.sum(axis=0) / (t1 - t0)
    return reps


def first_query(q, Hkv: int) -> np.ndarray:
    """q0bar[b][h][:] = mean over the G query heads of KV head h of the first draft's query."""
    q = _f64(q)
    B, _gamma, Hq, d = q.shape
    G = Hq // Hkv
    return q[:, 0].reshape(B, Hkv, G, d).sum(axis=2) / G


def block_scores(q, reps: np.ndarray) -> np.ndarray:
    """s[b][h][j] = q0bar[b][h] . reps[b][h][j]   (Eq. 5 after exchanging sum and dot)."""
    q0 = first_query(q, reps.shape[1])
    return np.einsum("bhd,bhjd->bhj", q0, _f64(reps))


def block_scores_literal(q, k_pool, block_table, seq_lens, block_size: int, divisor: str = "count") -> np.ndarray:
    """Eq. 5 term by term: the sum over the block's keys of q0bar . k, divided (no cached mean).

    divisor = "count": by the number of tokens the block holds (the reading this build takes for
    a partial last block); divisor = "block_size": by B as Eq. 5 prints it.  The two differ only
    in a sequence's last block when it is partial, by the factor n_j / B.
    """
    if divisor not in ("count", "block_size"):
        raise ValueError("divisor must be 'count' or 'block_size'")
    cache = PagedCache(k_pool, block_table)
    lens = _ints(seq_lens)
    q0 = first_query(q, cache.Hkv)
    nb_max = max(n_blocks(L, block_size) for L in lens)
    s = np.zeros((len(lens), cache.Hkv, nb_max), dtype=np.float64)
    for b, L in enumerate(lens):
        for j in range(n_blocks(L, block_size)):
            t0, t1 = j * block_size, min((j + 1) * block_size, int(L))
            keys = cache.tokens(b, t0, t1)
            for h in range(cache.Hkv):
                dots = keys[:, h, :] @ q0[b, h]
                s[b, h, j] = dots.sum() / ((t1 - t0) if divisor == "count" else block_size)
    return s


# --------------------------------------------------------------------------- top-N

def select_blocks(scores: np.ndarray, seq_lens, block_size: int, k_blocks: int,
                  n_sink: int = 0, n_local: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Shared block set per (b, h).

    The first n_sink and last n_local blocks are always kept and count inside the
    budget; the remaining budget goes to the highest scores, ties to the lowest block
    index.  Returns (sel_idx int32 [B][Hkv][k] ascending, padded with -1;
    sel_cnt int32 [B][Hkv] = min(k, nb_b)).
    """
    if k_blocks < 1 or n_sink < 0 or n_local < 0 or n_sink + n_local > k_blocks:
        raise ValueError("bad budget")
    lens = _ints(seq_lens)
    B, Hkv, _ = scores.shape
    sel_idx = np.full((B, Hkv, k_blocks), -1, dtype=np.int32)
    sel_cnt = np.zeros((B, Hkv), dtype=np.int32)
    for b in range(B):
        nb = n_blocks(lens[b], block_size)
        cnt = min(k_blocks, nb)
        forced = set(range(min(n_sink, nb))) | set(range(max(nb - n_local, 0), nb))
        for h in range(Hkv):
            rest = [j for j in range(nb) if j not in forced]
            rest.sort(key=lambda j: (-float(scores[b, h, j]), j))
            chosen = sorted(forced | set(rest[:max(cnt - len(forced), 0)]))
            chosen = chosen[:cnt] if len(chosen) > cnt else chosen
            sel_idx[b, h, :len(chosen)] = chosen
            sel_cnt[b, h] = len(chosen)
    return sel_idx, sel_cnt


def near_tie_blocks(scores_bh: np.ndarray, nb: int, chosen: Sequence[int], rel_gap: float = 1e-3,
                    n_sink: int = 0, n_local: int = 0) -> List[int]:
    """Blocks of one (b, h) whose score lies within rel_gap of the weakest block kept for its score.

    The first n_sink and last n_local blocks are kept whatever they score (Sec. 3.1), so they
    neither set the threshold nor can they be near-ties: the threshold is the lowest score among
    the chosen blocks outside those two ranges, and only blocks outside them are returned.  A
    selection that differs from the oracle's only inside this set is a near-tie, not an error;
    tests count and report such cases.
    """
    free = lambda j: n_sink <= j < nb - n_local
    kept = [int(c) for c in chosen if c >= 0 and free(int(c))]
    if not kept:
        return []
    s_k = min(float(scores_bh[j]) for j in kept)
    tol = rel_gap * max(abs(s_k), 1e-30)
    return [j for j in range(nb) if free(j) and abs(float(scores_bh[j]) - s_k) <= tol]


# --------------------------------------------------------------------------- attention

def _mask_bits(draft_mask, B: int, gamma: int) -> np.ndarray:
    """bool [B][gamma][gamma]: entry (b, i, t) says draft i may attend draft t."""
    if draft_mask is None:
        m = np.tril(np.ones((gamma, gamma), dtype=bool))
        return np.broadcast_to(m, (B, gamma, gamma)).copy()
    raw = draft_mask
    if hasattr(raw, "detach"):
        raw = raw.detach().to("cpu").numpy()
    raw = np.asarray(raw)
    if raw.dtype != object:
        raw = raw.astype(np.int64).astype(object)
    raw = np.vectorize(lambda x: int(x) & ((1 << 64) - 1), otypes=[object])(raw)
    if raw.ndim == 1:
        raw = np.broadcast_to(raw, (B, gamma))
    out = np.zeros((B, gamma, gamma), dtype=bool)
    for b in range(B):
        for i in range(gamma):
            for t in range(gamma):
                out[b, i, t] = (int(raw[b, i]) >> t) & 1
    return out


def _attend(q, k_cache: PagedCache, v_cache: PagedCache, seq_lens, k_draft, v_draft, draft_mask,
            blocks_of, block_size: int, sm_scale: Optional[float], return_weights: bool):
    q = _f64(q)
    kd = _f64(k_draft)
    vd = _f64(v_draft)
    lens = _ints(seq_lens)
    B, gamma, Hq, d = q.shape
    Hkv = k_cache.Hkv
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(d) if (sm_scale is None or sm_scale <= 0) else float(sm_scale)
    allow = _mask_bits(draft_mask, B, gamma)
    out = np.zeros((B, gamma, Hq, d), dtype=np.float64)
    lse = np.zeros((B, gamma, Hq), dtype=np.float64)
    weights = {} if return_weights else None
    for b in range(B):
        L = int(lens[b])
        for h in range(Hkv):
            toks: List[int] = []
            ks, vs = [], []
            for j in blocks_of(b, h):
                t0, t1 = j * block_size, min((j + 1) * block_size, L)
                ks.append(k_cache.tokens(b, t0, t1)[:, h, :])
                vs.append(v_cache.tokens(b, t0, t1)[:, h, :])
                toks.extend(range(t0, t1))
            kp = np.concatenate(ks, axis=0) if ks else np.zeros((0, d))
            vp = np.concatenate(vs, axis=0) if vs else np.zeros((0, d))
            n_p = kp.shape[0]
            keys = np.concatenate([kp, kd[b, :, h, :]], axis=0)      # prefix tokens, then drafts
            vals = np.concatenate([vp, vd[b, :, h, :]], axis=0)
            for i in range(gamma):
                vis = np.concatenate([np.ones(n_p, dtype=bool), allow[b, i]])
                for g in range(G):
                    j = h * G + g
                    logit = scale * (keys @ q[b, i, j])
                    logit = np.where(vis, logit, -np.inf)
                    if not vis.any():
                        # no key is visible (no kept block and a draft mask without the row's own
                        # bit): the paper defines nothing here; reading: zero output, lse = -inf
                        out[b, i, j] = 0.0
                        lse[b, i, j] = -np.inf
                        if return_weights:
                            weights[(b, i, j)] = (list(toks), np.zeros(len(vis)))
                        continue
                    m = logit.max()
                    p = np.exp(logit - m)
                    z = p.sum()
                    w = p / z
                    out[b, i, j] = w @ vals
                    lse[b, i, j] = m + math.log(z)
                    if return_weights:
                        weights[(b, i, j)] = (list(toks), w)
    if return_weights:
        return out, lse, weights
    return out, lse


def verify_attn(q, k_pool, v_pool, block_table, seq_lens, k_draft, v_draft, draft_mask,
                sel_idx, sel_cnt, block_size: int, sm_scale: Optional[float] = None,
                return_weights: bool = False):
    """Attention of every draft query over (tokens of its KV head's selected blocks) U (visible drafts).

    Returns out fp64 [B][gamma][Hq][d], lse fp64 [B][gamma][Hq] (natural log of the sum of
    exp(scaled logits)) and, on request, the softmax rows as {(b, i, j): (prefix_tokens, weights)}
    where weights lists the prefix tokens first and the gamma drafts last.
    """
    sel_idx = _ints(sel_idx)
    sel_cnt = _ints(sel_cnt)

    def blocks_of(b, h):
        return [int(x) for x in sel_idx[b, h, :int(sel_cnt[b, h])]]

    return _attend(q, PagedCache(k_pool, block_table), PagedCache(v_pool, block_table), seq_lens,
                   k_draft, v_draft, draft_mask, blocks_of, block_size, sm_scale, return_weights)


def dense_attn(q, k_pool, v_pool, block_table, seq_lens, k_draft, v_draft, draft_mask,
               block_size: int, sm_scale: Optional[float] = None, return_weights: bool = False):
    """The same attention with no eviction: every prefix block participates."""
    lens = _ints(seq_lens)

    def blocks_of(b, _h):
        return list(range(n_blocks(lens[b], block_size)))

    return _attend(q, PagedCache(k_pool, block_table), PagedCache(v_pool, block_table), seq_lens,
                   k_draft, v_draft, draft_mask, blocks_of, block_size, sm_scale, return_weights)


# --------------------------------------------------------------------------- Eq. 6, Eq. 9

def budget_blocks(L: int, L0: int, rho: float, block_size: int) -> Tuple[int, bool]:
    """Blocks kept per KV head for a prefix of L tokens; (k, dense).

    L <= L0: no eviction (dense, k = all blocks).  Otherwise Eq. 6 divided by the number of
    KV heads: ((L - L0) * rho + L0) / Bs, rounded up and clamped to [1, nb].
    """
    nb = n_blocks(L, block_size)
    if L <= L0:
        return nb, True
    k = int(math.ceil(((L - L0) * rho + L0) / block_size - 1e-12))
    return max(1, min(k, nb)), False


def anchor_of(layer: int, anchors: Sequence[int]) -> int:
    """Layer whose retrieval result layer `layer` uses: itself if it is an anchor, else the
    nearest preceding anchor (Eq. 9).  Layer 0 must be an anchor."""
    if layer in anchors:
        return layer
    prev = [a for a in anchors if a < layer]
    if not prev:
        raise ValueError("no preceding anchor layer")
    return max(prev)


def verify_step(q, k_pool, v_pool, block_table, seq_lens, k_draft, v_draft, draft_mask,
                reps, block_size: int, k_blocks: int, do_select: bool,
                sel_idx=None, sel_cnt=None, n_sink: int = 0, n_local: int = 0,
                sm_scale: Optional[float] = None):
    """One layer of one verification step.  Anchor layer (do_select): score, select, attend.
    Other layers: attend with the block set handed in (the preceding anchor's)."""
    if do_select:
        s = block_scores(q, reps)
        sel_idx, sel_cnt = select_blocks(s, seq_lens, block_size, k_blocks, n_sink, n_local)
    out, lse = verify_attn(q, k_pool, v_pool, block_table, seq_lens, k_draft, v_draft, draft_mask,
                           sel_idx, sel_cnt, block_size, sm_scale)
    return out, lse, sel_idx, sel_cnt
