"""Pins of the retrieval-variants oracle (CPU): brute force from the definitions, the bound that
makes the min/max summary what it is, closed forms, and special cases that reduce to the main
path's oracle (Sec. 3.1, Eq. 5; Sec. 3.2, Eq. 6 read over all KV heads)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import svf_oracle as O
from oracle import svf_variants_oracle as V


def tiny(**kw):
    base = dict(name="tiny", cfg_id=9, dtype="f32", B=2, Hq=6, Hkv=2, d=16, T=100, block_size=8, gamma=3,
                k_blocks=3, page_size=4, planted=2, shift=1.0, min_len=30)
    base.update(kw)
    return W.VerifyConfig(**base)


def test_minmax_against_token_loops():
    cfg = tiny()
    x = W.make_layer(cfg)
    mn, mx = V.block_minmax(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
    pool = x["k_pool"].double().numpy()
    table = x["block_table"].numpy()
    for b in range(cfg.B):
        L = int(x["seq_lens"][b])
        for j in range(cfg.nb_max):
            toks = range(j * cfg.block_size, min((j + 1) * cfg.block_size, L))
            for h in range(cfg.Hkv):
                for c in range(cfg.d):
                    vals = [pool[table[b, t // cfg.page_size], t % cfg.page_size, h, c] for t in toks]
                    assert mn[b, h, j, c] == (min(vals) if vals else 0.0)
                    assert mx[b, h, j, c] == (max(vals) if vals else 0.0)
    reps = O.block_reps(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
    assert (mn <= reps + 1e-15).all() and (reps <= mx + 1e-15).all()


def test_minmax_score_bounds_every_key_of_the_block():
    """What the min/max summary is for: sum_c max(q_c min_c, q_c max_c) >= q . k for every key k of
    the block, and it is attained when all keys of the block are equal."""
    cfg = tiny()
    x = W.make_layer(cfg)
    mn, mx = V.block_minmax(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
    s = V.head_scores(x["q"], mn=mn, mx=mx)
    cache = O.PagedCache(x["k_pool"], x["block_table"])
    q = x["q"].double().numpy()
    G = cfg.G
    slack = []
    for b in range(cfg.B):
        L = int(x["seq_lens"][b])
        for j in range(O.n_blocks(L, cfg.block_size)):
            keys = cache.tokens(b, j * cfg.block_size, min((j + 1) * cfg.block_size, L))
            for hq in range(cfg.Hq):
                dots = keys[:, hq // G] @ q[b, 0, hq]
                assert (dots <= s[b, hq, j] + 1e-12).all()
                slack.append(s[b, hq, j] - dots.max())
    assert max(slack) > 0                                    # a bound, not the maximum itself
    # constant keys: the bound is the dot product
    k1 = x["k_pool"].clone()
    k1[:] = k1[0, 0]
    mn1, mx1 = V.block_minmax(k1, x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
    s1 = V.head_scores(x["q"], mn=mn1, mx=mx1)
    key = k1[0, 0].double().numpy()
    for b in range(cfg.B):
        nb = O.n_blocks(int(x["seq_lens"][b]), cfg.block_size)
        for hq in range(cfg.Hq):
            np.testing.assert_allclose(s1[b, hq, :nb], key[hq // G] @ q[b, 0, hq], rtol=1e-13)


def test_mean_key_scores_reduce_to_the_main_path():
    """Eq. 5 is linear in the query: the mean over the group's heads of the per-head scores is the
    score of the mean query (the main oracle), and the literal per-key form of Eq. 5."""
    cfg = tiny()
    x = W.make_layer(cfg)
    reps = O.block_reps(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
    s_head = V.head_scores(x["q"], reps=reps)
    s = V.group_scores(s_head, cfg.Hkv, V.GROUP_MEAN)
    np.testing.assert_allclose(s, O.block_scores(x["q"], reps), rtol=0, atol=1e-12)
    lit = O.block_scores_literal(x["q"], x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size)
    for b in range(cfg.B):
        nb = O.n_blocks(int(x["seq_lens"][b]), cfg.block_size)
        np.testing.assert_allclose(s[b, :, :nb], lit[b, :, :nb], rtol=0, atol=1e-12)


def test_group_rules():
    rng = np.random.default_rng(3)
    s_head = rng.standard_normal((2, 6, 5))
    mean = V.group_scores(s_head, 2, V.GROUP_MEAN)
    mx = V.group_scores(s_head, 2, V.GROUP_MAX)
    for b in range(2):
        for h in range(2):
            for j in range(5):
                vals = [s_head[b, 3 * h + g, j] for g in range(3)]
                assert mean[b, h, j] == pytest.approx(sum(vals) / 3, rel=1e-15)
                assert mx[b, h, j] == max(vals)
    assert (mx >= mean).all()
    # one query head per KV head: both rules are the identity
    np.testing.assert_array_equal(V.group_scores(s_head, 6, V.GROUP_MAX), s_head)
    np.testing.assert_array_equal(V.group_scores(s_head, 6, V.GROUP_MEAN), s_head)
    with pytest.raises(ValueError):
        V.group_scores(s_head, 2, 7)


def test_round_bf16_against_the_library_conversion():
    rng = np.random.default_rng(11)
    a = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-6, 6, 4000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e-39, 65280.0]])
    a = a.astype(np.float32).astype(np.float64)
    want = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).double().numpy()
    np.testing.assert_array_equal(V.round_bf16(a), want)
    # ties go to the even mantissa: 1 + 2^-8 sits between 1 and 1 + 2^-7
    assert V.round_bf16([1.00390625])[0] == 1.0
    assert V.round_bf16([1.01171875])[0] == 1.015625         # 1 + 3 * 2^-8 -> 1 + 2^-6 (even)
    # already on the grid: unchanged
    g = V.round_bf16(a)
    np.testing.assert_array_equal(V.round_bf16(g), g)


def test_select_global_worked_example():
    """Two heads, four blocks, five pairs kept: by hand."""
    scores = np.array([[[0.9, 0.1, 0.8, 0.3],
                        [0.2, 0.7, 0.3, 0.6]]])
    idx, cnt = V.select_global(scores, [4 * 8], 8, 5, 4)
    # descending: (0,0) .9, (0,2) .8, (1,1) .7, (1,3) .6, then .3 twice: the lower head wins
    assert cnt.tolist() == [[3, 2]]
    assert idx[0, 0].tolist() == [0, 2, 3, -1] and idx[0, 1].tolist() == [1, 3, -1, -1]
    # sink block forced in both heads, counted inside the five
    idx, cnt = V.select_global(scores, [4 * 8], 8, 5, 4, n_sink=1)
    assert idx[0, 0].tolist() == [0, 2, -1, -1] and idx[0, 1].tolist() == [0, 1, 3, -1]
    # local block as well: 4 forced pairs, one free
    idx, cnt = V.select_global(scores, [4 * 8], 8, 5, 4, n_sink=1, n_local=1)
    assert idx[0, 0].tolist() == [0, 2, 3, -1] and idx[0, 1].tolist() == [0, 3, -1, -1]
    with pytest.raises(ValueError):
        V.select_global(scores, [32], 8, 3, 4, n_sink=1, n_local=1)   # forced pairs exceed the budget
    with pytest.raises(ValueError):
        V.select_global(scores, [32], 8, 5, 2)                         # head 0 keeps three: stride 2 too small


def test_select_global_against_sorting_and_the_per_head_rule():
    cfg = tiny(Hq=8, Hkv=4, n_sink=1, n_local=1)
    x = W.make_layer(cfg)
    reps = O.block_reps(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
    s = O.block_scores(x["q"], reps)
    n_total = 14
    idx, cnt = V.select_global(s, x["seq_lens"], cfg.block_size, n_total, cfg.nb_max, 1, 1)
    for b in range(cfg.B):
        nb = O.n_blocks(int(x["seq_lens"][b]), cfg.block_size)
        assert cnt[b].sum() == min(n_total, cfg.Hkv * nb)
        kept = {(h, int(j)) for h in range(cfg.Hkv) for j in idx[b, h, :cnt[b, h]]}
        forced = {(h, j) for h in range(cfg.Hkv) for j in (0, nb - 1)}
        assert forced <= kept
        free_kept = [s[b, h, j] for (h, j) in kept - forced]
        free_out = [s[b, h, j] for h in range(cfg.Hkv) for j in range(nb) if (h, j) not in kept]
        assert min(free_kept) >= max(free_out)               # nothing left out beats anything kept
        for h in range(cfg.Hkv):
            assert (np.diff(idx[b, h, :cnt[b, h]]) > 0).all() and (idx[b, h, cnt[b, h]:] == -1).all()
    # a single KV head: the global rule is the per-head rule
    s1 = s[:, :1]
    ig, cg = V.select_global(s1, x["seq_lens"], cfg.block_size, 5, 5, 1, 1)
    ip, cp = O.select_blocks(s1, x["seq_lens"], cfg.block_size, 5, 1, 1)
    np.testing.assert_array_equal(ig, ip)
    np.testing.assert_array_equal(cg, cp)
    # one head outscoring the others takes what it can hold
    s2 = s.copy()
    s2[:, 2] += 1e3
    ig, cg = V.select_global(s2, x["seq_lens"], cfg.block_size, n_total, cfg.nb_max, 0, 0)
    for b in range(cfg.B):
        nb = O.n_blocks(int(x["seq_lens"][b]), cfg.block_size)
        assert cg[b, 2] == min(nb, n_total)
    # budget beyond the pairs there are: everything is kept
    ig, cg = V.select_global(s, x["seq_lens"], cfg.block_size, 10 ** 6, cfg.nb_max)
    for b in range(cfg.B):
        assert (cg[b] == O.n_blocks(int(x["seq_lens"][b]), cfg.block_size)).all()


def test_near_tie_pairs():
    scores = np.array([[1.0, 0.5, 0.4999, 0.1], [0.5002, 0.2, 0.9, 0.0]])
    idx = np.array([[0, 1, -1, -1], [2, -1, -1, -1]])
    assert V.near_tie_pairs(scores, 4, idx, [2, 1]) == [(0, 1), (0, 2), (1, 0)]
    assert V.near_tie_pairs(scores, 4, idx, [0, 0]) == []
    # forced blocks neither set the threshold nor count as ties
    idx = np.array([[0, 1, 3, -1], [0, 2, 3, -1]])
    assert V.near_tie_pairs(scores, 4, idx, [3, 3], n_sink=1, n_local=1) == [(0, 1), (0, 2)]
