"""Pins of the retrieval-analytics oracle (CPU): brute force from the definitions, closed forms,
special cases that reduce to the main path's oracle.  Sec. 2.2 / Fig. 2 (overlap of the blocks
retrieved by different draft tokens) and Sec. 3.3, Eq. 7-8 (Jaccard similarity of adjacent layers,
anchor layers)."""
import itertools

import numpy as np
import pytest
import torch

import workloads as W
from oracle import svf_analytics_oracle as A
from oracle import svf_oracle as O


def tiny(**kw):
    base = dict(name="tiny", cfg_id=8, dtype="f32", B=2, Hq=4, Hkv=2, d=16, T=96, block_size=8, gamma=5,
                k_blocks=3, page_size=0, planted=2, shift=1.0, min_len=20)
    base.update(kw)
    return W.VerifyConfig(**base)


def layer_and_scores(cfg, layer=0):
    x = W.make_layer(cfg, layer)
    reps = O.block_reps(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
    return x, reps, A.per_draft_scores(x["q"], reps)


def test_draft_zero_is_the_main_path_retrieval():
    """Sec. 2.2: the method retrieves with the first draft token; the per-draft rule at i = 0 must be it."""
    cfg = tiny()
    x, reps, s = layer_and_scores(cfg)
    np.testing.assert_allclose(s[:, 0], O.block_scores(x["q"], reps), rtol=0, atol=1e-12)
    masks = A.per_draft_masks(s, x["seq_lens"], cfg.block_size, cfg.k_blocks)
    idx, cnt = O.select_blocks(O.block_scores(x["q"], reps), x["seq_lens"], cfg.block_size, cfg.k_blocks)
    np.testing.assert_array_equal(masks[:, :, 0], A.masks_from_selection(idx, cnt, cfg.nb_max))


def test_per_draft_masks_against_loops():
    """Eq. 5 and the top-N rule written out with loops, per draft token."""
    cfg = tiny(n_sink=1, n_local=1, k_blocks=4)
    x, reps, s = layer_and_scores(cfg)
    masks = A.per_draft_masks(s, x["seq_lens"], cfg.block_size, cfg.k_blocks, cfg.n_sink, cfg.n_local)
    q = x["q"].double().numpy()
    G = cfg.Hq // cfg.Hkv
    for b in range(cfg.B):
        nb = -(-int(x["seq_lens"][b]) // cfg.block_size)
        for h in range(cfg.Hkv):
            for i in range(cfg.gamma):
                qm = sum(q[b, i, h * G + g] for g in range(G)) / G
                sc = [float(sum(qm[c] * reps[b, h, j, c] for c in range(cfg.d))) for j in range(nb)]
                forced = {0, nb - 1}
                rest = sorted((j for j in range(nb) if j not in forced), key=lambda j: (-sc[j], j))
                want = forced | set(rest[:min(cfg.k_blocks, nb) - len(forced)])
                assert set(np.flatnonzero(masks[b, h, i]).tolist()) == want


def test_pack_masks_layout():
    m = np.zeros((2, 130), dtype=bool)
    m[0, [0, 63, 64, 129]] = True
    m[1, 65] = True
    w = A.pack_masks(m)
    assert w.shape == (2, 3) and w.dtype == np.uint64
    assert w[0].tolist() == [(1 << 0) | (1 << 63), 1 << 0, 1 << 1]
    assert w[1].tolist() == [0, 1 << 1, 0]


def test_overlap_closed_forms():
    """Constructed masks: identical sets overlap 1, disjoint sets 0, half-shared sets 1/2 (Fig. 2's ratio)."""
    B, Hkv, gamma, nb, k = 1, 2, 4, 32, 4
    masks = np.zeros((B, Hkv, gamma, nb), dtype=bool)
    masks[:, :, 0, [0, 1, 2, 3]] = True
    masks[:, :, 1, [0, 1, 2, 3]] = True            # distance 1 from draft 0: identical
    masks[:, :, 2, [2, 3, 4, 5]] = True            # distance 2 from draft 0: half shared
    masks[:, :, 3, [10, 11, 12, 13]] = True        # distance 3 from draft 0: disjoint
    pos = [0, 1, 2, 3]
    inter, pairs, mean = A.overlap_by_distance(masks, pos, [nb * 8], 8, k, 4)
    assert pairs.tolist() == [0, 3, 2, 1]
    # distance 1: pairs (0,1) 4 shared, (1,2) 2, (2,3) 0; distance 2: (0,2) 2, (1,3) 0; distance 3: (0,3) 0
    assert inter[0].tolist() == [0, Hkv * 6, Hkv * 2, 0]
    assert np.isnan(mean[0])
    np.testing.assert_allclose(mean[1:], [6 / (4 * 3), 2 / (4 * 2), 0.0])


def test_overlap_brute_force_and_same_position():
    """A tree has different tokens at the same position (distance 0); compare with a direct count."""
    cfg = tiny(gamma=6, tree_depth=2, k_blocks=4)
    x, reps, s = layer_and_scores(cfg)
    masks = A.per_draft_masks(s, x["seq_lens"], cfg.block_size, cfg.k_blocks)
    parents = W.draft_tree(cfg).tolist()
    pos = [0] * cfg.gamma
    for i, p in enumerate(parents):
        pos[i] = 0 if p < 0 else pos[p] + 1
    assert len(set(pos)) < cfg.gamma                      # some tokens share a position
    n_dist = max(pos) + 1
    inter, pairs, mean = A.overlap_by_distance(masks, pos, x["seq_lens"], cfg.block_size, cfg.k_blocks, n_dist)
    want = np.zeros((cfg.B, n_dist), dtype=np.int64)
    npairs = np.zeros(n_dist, dtype=np.int64)
    for i, i2 in itertools.combinations(range(cfg.gamma), 2):
        npairs[abs(pos[i] - pos[i2])] += 1
        for b in range(cfg.B):
            for h in range(cfg.Hkv):
                want[b, abs(pos[i] - pos[i2])] += int((masks[b, h, i] & masks[b, h, i2]).sum())
    np.testing.assert_array_equal(inter, want)
    np.testing.assert_array_equal(pairs, npairs)
    kept = [min(cfg.k_blocks, -(-int(L) // cfg.block_size)) for L in x["seq_lens"]]
    for dist in range(n_dist):
        ref = np.mean([want[b, dist] / (kept[b] * cfg.Hkv * npairs[dist]) for b in range(cfg.B)])
        assert mean[dist] == pytest.approx(ref, rel=1e-15)
    assert ((mean >= 0) & (mean <= 1)).all()


def test_identical_queries_retrieve_identical_blocks():
    cfg = tiny()
    x = W.make_layer(cfg)
    x["q"][:] = x["q"][:, :1]                             # every draft token asks the same question
    reps = O.block_reps(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
    masks = A.per_draft_masks(A.per_draft_scores(x["q"], reps), x["seq_lens"], cfg.block_size, cfg.k_blocks)
    _, _, mean = A.overlap_by_distance(masks, list(range(cfg.gamma)), x["seq_lens"], cfg.block_size, cfg.k_blocks,
                                       cfg.gamma)
    np.testing.assert_allclose(mean[1:], 1.0)


def test_empty_sequence_is_left_out_of_the_average():
    B, Hkv, gamma, nb, k = 2, 1, 2, 8, 2
    masks = np.zeros((B, Hkv, gamma, nb), dtype=bool)
    masks[0, 0, :, [1, 2]] = True
    _, _, mean = A.overlap_by_distance(masks, [0, 1], [64, 0], 8, k, 2)
    assert mean[1] == 1.0


def test_jaccard_closed_forms():
    """Eq. 7 on sets whose intersection and union are known by construction."""
    nb = 40
    L = 5
    m = np.zeros((L, 2, nb), dtype=bool)
    m[0, :, :6] = True
    m[1, :, :6] = True                                    # same as layer 0: J = 1
    m[2, :, 10:16] = True                                 # disjoint from layer 1: J = 0
    m[3, 0, 12:18] = True                                 # head 0 shares 4 of 8, head 1 shares 0 of 6
    m[4] = False                                          # empty against non-empty: J = 0
    inter, union, J = A.jaccard_adjacent(m)
    assert (inter[0], union[0], J[0]) == (0, 0, 0.0)      # first layer: 0 by definition
    assert (inter[1], union[1], J[1]) == (12, 12, 1.0)
    assert (inter[2], union[2], J[2]) == (0, 24, 0.0)
    assert (inter[3], union[3]) == (4, 8 + 6) and J[3] == pytest.approx(4 / 14)
    assert (inter[4], union[4], J[4]) == (0, 6, 0.0)
    # two empty masks are identical sets
    assert A.jaccard_adjacent(np.zeros((2, 8), dtype=bool))[2][1] == 1.0


def test_jaccard_is_symmetric_and_tied_to_overlap():
    """For two sets of equal size k with overlap ratio o = |A & B| / k, Eq. 7 gives o / (2 - o)."""
    rng = np.random.default_rng(7)
    nb, k = 64, 12
    for _ in range(20):
        a = np.zeros(nb, dtype=bool)
        b = np.zeros(nb, dtype=bool)
        a[rng.choice(nb, k, replace=False)] = True
        b[rng.choice(nb, k, replace=False)] = True
        j_ab = A.jaccard_adjacent(np.stack([a, b]))[2][1]
        j_ba = A.jaccard_adjacent(np.stack([b, a]))[2][1]
        o = (a & b).sum() / k
        assert j_ab == j_ba == pytest.approx(o / (2 - o), rel=1e-15)


def test_topk_anchors():
    """Eq. 8 on a worked example; the first layer (J = 0 by definition) is always an anchor."""
    J = [0.0, 0.9, 0.2, 0.8, 0.1, 0.95]
    assert A.topk_anchors(J, 1) == [0]
    assert A.topk_anchors(J, 3) == [0, 2, 4]
    assert A.topk_anchors(J, 6) == [0, 1, 2, 3, 4, 5]
    # nested: the K anchors are among the K + 1 anchors
    for K in range(1, 6):
        assert set(A.topk_anchors(J, K)) < set(A.topk_anchors(J, K + 1))
    # equal similarities: the lower layer wins
    assert A.topk_anchors([0.0, 0.5, 0.5, 0.5], 2) == [0, 1]
    with pytest.raises(ValueError):
        A.topk_anchors(J, 0)
    # several calibration samples: the mean similarity decides
    Js = np.array([[0.0, 0.1, 0.9, 0.9], [0.0, 0.9, 0.1, 0.9]])
    assert A.anchors_from_samples(Js, 2) in ([0, 1], )   # layers 1 and 2 tie at 0.5: lower layer


def test_anchors_feed_the_reuse_rule():
    """Eq. 8 -> Eq. 9: with the anchors of a calibration run every layer finds a preceding anchor."""
    J = [0.0, 0.9, 0.3, 0.85, 0.8, 0.2, 0.95, 0.9]
    anchors = A.topk_anchors(J, 3)
    assert anchors == [0, 2, 5]
    assert [O.anchor_of(l, anchors) for l in range(8)] == [0, 0, 2, 2, 2, 5, 5, 5]


def test_planted_positions_make_reuse_groups_similar():
    """The workload plants the same blocks in all layers of a reuse group: the first-draft masks of an
    anchor and its follower then coincide, and differ from the next group's (what Sec. 3.3 observes)."""
    cfg = W.shrink(W.CONFIGS[3], 8192)
    masks = []
    for layer in range(4):
        x = W.make_layer(cfg, layer)
        reps = O.block_reps(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
        idx, cnt = O.select_blocks(O.block_scores(x["q"], reps), x["seq_lens"], cfg.block_size, cfg.k_blocks)
        masks.append(A.masks_from_selection(idx, cnt, cfg.nb_max))
    _, _, J = A.jaccard_adjacent(np.stack(masks))
    assert J[1] > J[2] and J[3] > J[2]
    assert A.topk_anchors(J, 2) == [0, 2]
