"""CPU oracle for the retrieval analytics the paper bases its attention design on
(Sec. 2.2 and Fig. 2: how similar are the blocks retrieved by different draft tokens;
Sec. 3.3, Eq. 7-8: which layers retrieve differently from the layer before them).

TEST INFRASTRUCTURE ONLY, like svf_oracle.py: plain numpy / Python sets in fp64 and exact
integers, imported by tests and by the bench's CPU leg, never by the product, and sharing no
code with the HIP path.

What each function follows:

  draft_queries         Sec. 2.2: every draft token retrieves "based on its respective query";
                        with grouped query heads the queries sharing a KV head are averaged,
                        exactly as svf_oracle.first_query does for draft 0.
  per_draft_scores      Eq. 5 for every draft token's query instead of the first one only.
  per_draft_masks       Sec. 3.1 top-N rule applied per draft token: M[b][h][i] in {0,1}^nb.
  pack_masks            the bitset layout the library uses: block j -> bit j % 64 of word j / 64.
  overlap_by_distance   Sec. 2.2 / Fig. 2: |M_i & M_i'| / (number of retrieved blocks) for pairs
                        of draft tokens, averaged per positional distance |pos_i - pos_i'|.
  jaccard_adjacent      Eq. 7: J(M_l, M_{l-1}) = |M_l & M_{l-1}| / |M_l | M_{l-1}| over all
                        candidate blocks of a sample; J of the first layer is 0 by definition.
  topk_anchors          Eq. 8: the K layers with the largest 1 - J.

Readings taken where the paper is silent: the overlap's "total number of blocks" is the number
of blocks each token retrieves (k, or all blocks of a sequence shorter than k blocks);
sequences without any block do not enter the averages; J of two empty masks is 1 (identical
sets); calibration over several samples averages the per-sample J before Eq. 8; equal values
in Eq. 8 go to the lower layer.  Absolute overlap values on the paper's own workloads (Fig. 2:
"exceeding 0.8 in most layers") are "parity unpinned": they need the model and its data.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

from . import svf_oracle as O


def draft_queries(q, Hkv: int) -> np.ndarray:
    """[B][gamma][Hkv][d] fp64: draft i's query averaged over the query heads of each KV head."""
    qf = O._f64(q)
    B, gamma, Hq, d = qf.shape
    G = Hq // Hkv
    return qf.reshape(B, gamma, Hkv, G, d).mean(axis=3)


def per_draft_scores(q, reps: np.ndarray) -> np.ndarray:
    """s[b][i][h][j] = mean-query of draft i (KV head h) . representative j (Eq. 5 per draft)."""
    Hkv = reps.shape[1]
    qm = draft_queries(q, Hkv)                                   # [B][gamma][Hkv][d]
    return np.einsum("bihd,bhjd->bihj", qm, np.asarray(reps, dtype=np.float64))


def per_draft_masks(scores: np.ndarray, seq_lens, block_size: int, k_blocks: int,
                    n_sink: int = 0, n_local: int = 0) -> np.ndarray:
    """bool [B][Hkv][gamma][nb_max]: the top-N rule of Sec. 3.1 for every draft token."""
    B, gamma, Hkv, nb_max = scores.shape
    masks = np.zeros((B, Hkv, gamma, nb_max), dtype=bool)
    for i in range(gamma):
        idx, cnt = O.select_blocks(scores[:, i], seq_lens, block_size, k_blocks, n_sink, n_local)
        for b in range(B):
            for h in range(Hkv):
                masks[b, h, i, idx[b, h, :cnt[b, h]]] = True
    return masks


def masks_from_selection(sel_idx, sel_cnt, nb_max: int) -> np.ndarray:
    """bool [B][Hkv][nb_max] from an index list (what svf_score_select returns)."""
    idx = O._ints(sel_idx)
    cnt = O._ints(sel_cnt)
    B, Hkv, _ = idx.shape
    m = np.zeros((B, Hkv, nb_max), dtype=bool)
    for b in range(B):
        for h in range(Hkv):
            m[b, h, idx[b, h, :cnt[b, h]]] = True
    return m


def pack_masks(masks: np.ndarray) -> np.ndarray:
    """uint64 [..., ceil(nb/64)]: block j is bit j % 64 of word j // 64."""
    nb = masks.shape[-1]
    W = (nb + 63) // 64
    out = np.zeros(masks.shape[:-1] + (W,), dtype=np.uint64)
    for j in range(nb):
        out[..., j // 64] |= masks[..., j].astype(np.uint64) << np.uint64(j % 64)
    return out


def overlap_by_distance(masks: np.ndarray, pos: Sequence[int], seq_lens, block_size: int,
                        k_blocks: int, n_dist: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Overlap of the blocks retrieved by two draft tokens, by positional distance (Fig. 2).

    masks: bool [B][Hkv][gamma][nb]; pos[i]: position (tree depth) of draft i.
    Returns (inter int64 [B][n_dist]: sum over KV heads and pairs i < i' at that distance of
    |M_i & M_i'|; pairs int64 [n_dist]: pairs at that distance; mean fp64 [n_dist]: the average
    over sequences (that have blocks), heads and pairs of |M_i & M_i'| / kept blocks, NaN where
    no pair has that distance).  Distances >= n_dist are not counted.
    """
    B, Hkv, gamma, _ = masks.shape
    lens = O._ints(seq_lens)
    inter = np.zeros((B, n_dist), dtype=np.int64)
    pairs = np.zeros(n_dist, dtype=np.int64)
    for i in range(gamma):
        for i2 in range(i + 1, gamma):
            dist = abs(int(pos[i]) - int(pos[i2]))
            if dist < n_dist:
                pairs[dist] += 1
    for b in range(B):
        for h in range(Hkv):
            sets = [set(np.flatnonzero(masks[b, h, i]).tolist()) for i in range(gamma)]
            for i in range(gamma):
                for i2 in range(i + 1, gamma):
                    dist = abs(int(pos[i]) - int(pos[i2]))
                    if dist < n_dist:
                        inter[b, dist] += len(sets[i] & sets[i2])
    mean = np.full(n_dist, np.nan)
    kept = np.array([min(k_blocks, O.n_blocks(int(L), block_size)) for L in lens], dtype=np.float64)
    live = kept > 0
    for dist in range(n_dist):
        if pairs[dist] > 0 and live.any():
            per_seq = inter[live, dist] / (kept[live] * Hkv * pairs[dist])
            mean[dist] = per_seq.mean()
    return inter, pairs, mean


def jaccard_adjacent(masks_by_layer: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Eq. 7 for one sample.  masks_by_layer: bool [L][...]: layer l's mask over all candidate
    blocks (any trailing shape, e.g. [B][Hkv][nb]).  Returns (inter int64 [L], union int64 [L],
    J fp64 [L]); entry 0 is (0, 0, 0.0): J(M_1, M_0) = 0 by definition."""
    L = masks_by_layer.shape[0]
    inter = np.zeros(L, dtype=np.int64)
    union = np.zeros(L, dtype=np.int64)
    J = np.zeros(L, dtype=np.float64)
    for l in range(1, L):
        a = set(np.flatnonzero(masks_by_layer[l].reshape(-1)).tolist())
        b = set(np.flatnonzero(masks_by_layer[l - 1].reshape(-1)).tolist())
        inter[l] = len(a & b)
        union[l] = len(a | b)
        J[l] = 1.0 if union[l] == 0 else inter[l] / union[l]
    return inter, union, J


def topk_anchors(J: Sequence[float], K: int) -> List[int]:
    """Eq. 8: the K layers with the largest 1 - J(M_l, M_{l-1}); equal values go to the lower
    layer.  Returns the anchor layers in ascending order."""
    L = len(J)
    if not 1 <= K <= L:
        raise ValueError("K out of range")
    order = sorted(range(L), key=lambda l: (-(1.0 - float(J[l])), l))
    return sorted(order[:K])


def anchors_from_samples(J_samples: np.ndarray, K: int) -> List[int]:
    """Calibration over several samples (Sec. 3.3): average the per-sample J, then Eq. 8."""
    return topk_anchors(np.asarray(J_samples, dtype=np.float64).mean(axis=0), K)
