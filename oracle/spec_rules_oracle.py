"""CPU oracle for the two small per-token rules around the sparse verification: the expert
skipping of the sparse mixture of experts (Sec. 3.5, Eq. 15-16) and the acceptance / resampling
of speculative decoding (Sec. 2.1, Eq. 2-3).

TEST INFRASTRUCTURE ONLY: plain numpy / Python loops in fp64, imported by tests and by the bench's
CPU leg, never by the product, and sharing no code with the HIP path.

  skip_ratios      the quantity of Eq. 15 for every skip size i = 1 .. k-1 of every token.
  calibrate_beta   Sec. 3.5: beta_i = median over the calibration tokens of that quantity.
  moe_skip         Eq. 16: per token, the largest i <= m whose quantity lies below beta_i; the i
                   lowest-weight experts are skipped.
  accept_resample  Eq. 2: draft token k is accepted with probability min(1, p_theta / p_phi),
                   tested in order, everything behind the first rejection is dropped; Eq. 3: the
                   rejected position is resampled from norm(max(0, p_theta - p_phi)).

Reading of Eq. 15-16 (printed inconsistently: the weights are sorted ascending and the i lowest,
e_1 .. e_i, are skipped, yet the printed sum runs over the first k - i weights and is compared
with "<"): the quantity is the share of the routing mass that would be skipped,
    r_i = (w_1 + .. + w_i) / (w_1 + .. + w_k)      (ascending order),
small when the i lowest experts hardly matter, and i experts may be skipped when r_i < beta_i,
beta_i the median of r_i over the calibration tokens.  For k = 2 this is the rule the section
generalises (skip the second expert when its weight relative to the first is below the median
of that relation): w_1 / (w_1 + w_2) is an increasing function of w_1 / w_2, and medians commute
with increasing functions.  Equal weights: the expert listed first counts as the lower one.
Random numbers are inputs: u_accept[k] decides position k (accept iff u < alpha), u_resample
picks the resampled token by inversion of the cumulative residual (the first token whose
cumulative mass exceeds u times the total).  A residual that is zero everywhere (the two
distributions coincide, so a rejection needs u = 1) falls back to p_theta.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def skip_ratios(w) -> np.ndarray:
    """fp64 [T][k-1]: r_i for i = 1 .. k-1 (column i-1)."""
    w = np.asarray(w, dtype=np.float64)
    s = np.sort(w, axis=1)                                # ascending
    return np.cumsum(s, axis=1)[:, :-1] / s.sum(axis=1, keepdims=True)


def calibrate_beta(w_cal) -> np.ndarray:
    """fp64 [k-1]: the threshold map {beta_1 .. beta_{k-1}} of one layer."""
    return np.median(skip_ratios(w_cal), axis=0)


def moe_skip(w, beta: Sequence[float], m: int) -> Tuple[np.ndarray, np.ndarray]:
    """(n_skip int32 [T], keep bool [T][k]) by Eq. 16; 1 <= m < k."""
    w = np.asarray(w, dtype=np.float64)
    T, k = w.shape
    if not 1 <= m < k:
        raise ValueError("m out of range")
    r = skip_ratios(w)
    n_skip = np.zeros(T, dtype=np.int32)
    keep = np.ones((T, k), dtype=bool)
    for t in range(T):
        best = 0
        for i in range(1, m + 1):
            if r[t, i - 1] < beta[i - 1]:
                best = i
        order = sorted(range(k), key=lambda j: (w[t, j], j))      # ascending, listed-first is lower
        n_skip[t] = best
        keep[t, order[:best]] = False
    return n_skip, keep


def accept_resample(p_target, p_draft, draft_tokens, u_accept, u_resample) -> Tuple[np.ndarray, np.ndarray, dict]:
    """p_* [B][gamma][V], draft_tokens [B][gamma], u_accept [B][gamma], u_resample [B].
    Returns (n_accepted int32 [B], resampled int32 [B] (-1: nothing rejected), details) where
    details holds, per sequence with a rejection, the cumulative residual and the target mass
    (for bracket checks of another implementation's choice)."""
    pt = np.asarray(p_target, dtype=np.float64)
    pd = np.asarray(p_draft, dtype=np.float64)
    tok = np.asarray(draft_tokens)
    ua = np.asarray(u_accept, dtype=np.float64)
    ur = np.asarray(u_resample, dtype=np.float64)
    B, gamma, V = pt.shape
    n_acc = np.zeros(B, dtype=np.int32)
    res = np.full(B, -1, dtype=np.int32)
    details = {}
    for b in range(B):
        k = 0
        while k < gamma:
            x = int(tok[b, k])
            alpha = min(1.0, pt[b, k, x] / pd[b, k, x]) if pd[b, k, x] > 0 else 1.0      # Eq. 2
            if not ua[b, k] < alpha:
                break
            k += 1
        n_acc[b] = k
        if k < gamma:
            resid = np.maximum(0.0, pt[b, k] - pd[b, k])                                  # Eq. 3
            if resid.sum() == 0.0:
                resid = pt[b, k].copy()
            cdf = np.cumsum(resid)
            target = ur[b] * cdf[-1]
            v = int(np.searchsorted(cdf, target, side="right"))
            res[b] = min(v, V - 1)
            details[b] = {"cdf": cdf, "target": target, "resid": resid}
    return n_acc, res, details
