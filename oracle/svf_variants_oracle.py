"""CPU oracle for the retrieval variants on either side of the paper's rule.

TEST INFRASTRUCTURE ONLY, like svf_oracle.py: plain numpy / Python loops in fp64 and exact
integers, imported by tests and by the bench's CPU leg, never by the product, and sharing no
code with the HIP path.

What each function follows:

  block_minmax      Sec. 3.1 names Quest as the block-retrieval idea the method starts from;
                    Quest's block summary is the per-channel minimum and maximum of the block's
                    keys (instead of Eq. 5's mean key).
  round_bf16        round-to-nearest-even to the bfloat16 grid (representatives stored in half
                    the bytes); returns fp64 values that lie on that grid.
  head_scores       the first draft token's score per QUERY head: Eq. 5 with that head's query
                    (mean-key summary), or Quest's upper bound  sum_c max(q_c min_c, q_c max_c)
                    (min/max summary).
  group_scores      how the Hq/Hkv query heads that share a KV head are combined: their mean
                    (for the mean-key summary this is Eq. 5 with the mean query, by linearity)
                    or their maximum.
  select_global     Eq. 6 read literally: N_budget counts blocks over all H KV heads of a
                    sequence, so the top-N rule of Sec. 3.1 runs over the (head, block) pairs of
                    the sequence and KV heads keep different numbers of blocks.
  near_tie_pairs    pairs whose score is within a relative gap of the weakest kept pair.

Readings taken where the paper is silent: sink / local blocks are forced per KV head and count
inside the budget; equal scores go to the lower KV head, then to the lower block; a partial last
block summarises the tokens it has; a sequence with fewer pairs than the budget keeps all.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import svf_oracle as O

GROUP_MEAN, GROUP_MAX = 0, 1


def block_minmax(k_pool, block_table, seq_lens, block_size: int,
                 nb_max: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """(mn, mx) fp64 [B][Hkv][nb_max][d]: per-channel minimum / maximum of each block's keys;
    rows of blocks that do not exist are 0."""
    cache = O.PagedCache(k_pool, block_table)
    lens = O._ints(seq_lens)
    B = len(lens)
    Hkv, d = cache.Hkv, cache.d
    if nb_max is None:
        nb_max = max(O.n_blocks(int(L), block_size) for L in lens)
    mn = np.zeros((B, Hkv, nb_max, d))
    mx = np.zeros((B, Hkv, nb_max, d))
    for b in range(B):
        L = int(lens[b])
        for j in range(O.n_blocks(L, block_size)):
            t0, t1 = j * block_size, min((j + 1) * block_size, L)
            keys = cache.tokens(b, t0, t1)                        # [tokens][Hkv][d]
            mn[b, :, j] = keys.min(axis=0)
            mx[b, :, j] = keys.max(axis=0)
    return mn, mx


def round_bf16(a) -> np.ndarray:
    """Nearest bfloat16 (ties to even) of every element, returned in fp64.  bfloat16 keeps the
    sign, the 8 exponent bits and the top 7 mantissa bits of a binary32 number; values are first
    rounded to binary32 (the representatives are computed in binary32 on the device)."""
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lower = bits & np.uint64(0xffff)
    keep = bits >> np.uint64(16)
    up = (lower > 0x8000) | ((lower == 0x8000) & ((keep & np.uint64(1)) == 1))
    keep = keep + up.astype(np.uint64)
    out = (keep << np.uint64(16)).astype(np.uint32).view(np.float32)
    return out.astype(np.float64)


def head_scores(q, reps: Optional[np.ndarray] = None, mn: Optional[np.ndarray] = None,
                mx: Optional[np.ndarray] = None) -> np.ndarray:
    """fp64 [B][Hq][nb]: the first draft token's score of every block per query head.
    Give `reps` (mean keys) for Eq. 5, or `mn` and `mx` for the min/max bound."""
    qf = O._f64(q)[:, 0]                                          # [B][Hq][d]
    B, Hq, d = qf.shape
    src = reps if reps is not None else mn
    Hkv, nb = src.shape[1], src.shape[2]
    G = Hq // Hkv
    s = np.zeros((B, Hq, nb))
    for b in range(B):
        for hq in range(Hq):
            h = hq // G
            if reps is not None:
                s[b, hq] = np.asarray(reps[b, h], dtype=np.float64) @ qf[b, hq]
            else:
                lo = np.asarray(mn[b, h], dtype=np.float64) * qf[b, hq]
                hi = np.asarray(mx[b, h], dtype=np.float64) * qf[b, hq]
                s[b, hq] = np.maximum(lo, hi).sum(axis=-1)
    return s


def group_scores(s_head: np.ndarray, Hkv: int, rule: int) -> np.ndarray:
    """fp64 [B][Hkv][nb]: the scores of the query heads sharing a KV head, averaged or maximised."""
    B, Hq, nb = s_head.shape
    g = s_head.reshape(B, Hkv, Hq // Hkv, nb)
    if rule == GROUP_MEAN:
        return g.mean(axis=2)
    if rule == GROUP_MAX:
        return g.max(axis=2)
    raise ValueError("unknown group rule")


def select_global(scores: np.ndarray, seq_lens, block_size: int, n_total: int, stride: int,
                  n_sink: int = 0, n_local: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Top-N over the (KV head, block) pairs of each sequence.

    scores fp64 [B][Hkv][nb_max].  Per KV head the first n_sink and last n_local blocks are
    always kept and count inside n_total; the rest of n_total goes to the highest scores,
    equal scores to the lower head, then the lower block.  Returns (sel_idx int32
    [B][Hkv][stride] ascending per head, padded with -1; sel_cnt int32 [B][Hkv])."""
    lens = O._ints(seq_lens)
    B, Hkv, _ = scores.shape
    if n_total < 1 or n_sink < 0 or n_local < 0 or (n_sink + n_local) * Hkv > n_total:
        raise ValueError("bad budget")
    sel_idx = np.full((B, Hkv, stride), -1, dtype=np.int32)
    sel_cnt = np.zeros((B, Hkv), dtype=np.int32)
    for b in range(B):
        nb = O.n_blocks(int(lens[b]), block_size)
        keep_n = min(n_total, Hkv * nb)
        forced_j = set(range(min(n_sink, nb))) | set(range(max(nb - n_local, 0), nb))
        forced = [(h, j) for h in range(Hkv) for j in sorted(forced_j)]
        rest = [(h, j) for h in range(Hkv) for j in range(nb) if j not in forced_j]
        rest.sort(key=lambda hj: (-float(scores[b, hj[0], hj[1]]), hj[0], hj[1]))
        chosen = forced + rest[:max(keep_n - len(forced), 0)]
        for h in range(Hkv):
            js = sorted(j for (hh, j) in chosen if hh == h)
            if len(js) > stride:
                raise ValueError("stride too small for this head's share")
            sel_idx[b, h, :len(js)] = js
            sel_cnt[b, h] = len(js)
    return sel_idx, sel_cnt


def near_tie_pairs(scores_b: np.ndarray, nb: int, sel_idx_b, sel_cnt_b, rel_gap: float = 1e-3,
                   n_sink: int = 0, n_local: int = 0) -> List[Tuple[int, int]]:
    """(head, block) pairs of one sequence whose score lies within rel_gap of the weakest pair
    kept for its score (forced sink / local blocks aside); a selection that differs from the
    oracle's only inside this set is a near-tie."""
    Hkv = scores_b.shape[0]
    free = lambda j: n_sink <= j < nb - n_local
    kept = [(h, int(j)) for h in range(Hkv) for j in sel_idx_b[h][:int(sel_cnt_b[h])] if free(int(j))]
    if not kept:
        return []
    s_k = min(float(scores_b[h, j]) for h, j in kept)
    tol = rel_gap * max(abs(s_k), 1e-30)
    return [(h, j) for h in range(Hkv) for j in range(nb) if free(j) and abs(float(scores_b[h, j]) - s_k) <= tol]
