"""Pins of the expert-skipping and accept / resample oracle (CPU): hand-worked cases, the two-expert
rule the section generalises, invariants, and the distribution the acceptance rule must preserve
(Sec. 3.5, Eq. 15-16; Sec. 2.1, Eq. 2-3)."""
import numpy as np
import pytest

from oracle import spec_rules_oracle as R


def test_skip_ratios_by_hand():
    w = np.array([[0.4, 0.1, 0.3, 0.2]])                  # ascending .1 .2 .3 .4
    np.testing.assert_allclose(R.skip_ratios(w), [[0.1, 0.3, 0.6]])
    r = R.skip_ratios(np.random.default_rng(0).random((50, 8)))
    assert (np.diff(r, axis=1) > 0).all() and (r > 0).all() and (r < 1).all()
    # the i lowest of k weights carry at most i / k of the mass
    assert (r <= np.arange(1, 8) / 8 + 1e-15).all()
    # scale-free
    np.testing.assert_allclose(R.skip_ratios(7.5 * w), R.skip_ratios(w))


def test_two_experts_reduce_to_the_ratio_rule():
    """k = 2, m = 1: skip the weaker expert iff w_low / w_high is below the median of that relation."""
    rng = np.random.default_rng(1)
    cal = rng.random((1001, 2)) + 0.01
    beta = R.calibrate_beta(cal)
    rel = cal.min(axis=1) / cal.max(axis=1)
    med = np.median(rel)
    w = rng.random((500, 2)) + 0.01
    n_skip, keep = R.moe_skip(w, beta, 1)
    want = (w.min(axis=1) / w.max(axis=1)) < med
    assert (n_skip == want.astype(np.int32)).all()
    assert (keep.sum(axis=1) == 2 - n_skip).all()
    assert all(keep[t, np.argmax(w[t])] for t in range(500))


def test_median_threshold_splits_the_calibration_set():
    rng = np.random.default_rng(2)
    cal = rng.dirichlet(np.ones(8) * 0.7, size=2001)
    beta = R.calibrate_beta(cal)
    r = R.skip_ratios(cal)
    for i in range(7):
        assert abs((r[:, i] < beta[i]).mean() - 0.5) < 1e-3
    # with m = 1 exactly the tokens below beta_1 skip one expert
    n_skip, _ = R.moe_skip(cal, beta, 1)
    assert (n_skip == (r[:, 0] < beta[0])).all()


def test_moe_skip_worked_example_and_invariants():
    w = np.array([[0.30, 0.02, 0.25, 0.03, 0.40],         # ascending .02 .03 .25 .30 .40 -> r = .02 .05 .30 .60
                  [0.20, 0.20, 0.20, 0.20, 0.20]])        # r = .2 .4 .6 .8
    beta = [0.03, 0.04, 0.35, 0.5]
    n_skip, keep = R.moe_skip(w, beta, 3)
    # token 0: r_1 < beta_1, r_2 >= beta_2, r_3 < beta_3 -> the largest admissible size, 3
    assert n_skip.tolist() == [3, 0]
    assert keep[0].tolist() == [True, False, False, False, True] and keep[1].all()
    n_skip, keep = R.moe_skip(w, beta, 2)
    assert n_skip.tolist() == [1, 0] and keep[0].tolist() == [True, False, True, True, True]
    # equal weights: the expert listed first is the lower one
    n_skip, keep = R.moe_skip(w[1:], [0.5, 0.5, 0.7, 0.9], 2)
    assert n_skip.tolist() == [2] and keep[0].tolist() == [False, False, True, True, True]
    with pytest.raises(ValueError):
        R.moe_skip(w, beta, 5)
    with pytest.raises(ValueError):
        R.moe_skip(w, beta, 0)
    # a larger budget never skips less; skipped experts never outweigh kept ones
    rng = np.random.default_rng(3)
    cal = rng.dirichlet(np.ones(8), size=999)
    beta = R.calibrate_beta(cal)
    prev = np.zeros(999, dtype=np.int32)
    for m in range(1, 8):
        n_skip, keep = R.moe_skip(cal, beta, m)
        assert (n_skip >= prev).all() and (n_skip <= m).all()
        prev = n_skip
        for t in range(0, 999, 37):
            if n_skip[t]:
                assert cal[t][~keep[t]].max() <= cal[t][keep[t]].min()


def test_accept_resample_by_hand():
    # one sequence, three draft positions, four tokens
    pt = np.array([[[0.5, 0.2, 0.2, 0.1], [0.1, 0.6, 0.2, 0.1], [0.25, 0.25, 0.25, 0.25]]])
    pd = np.array([[[0.25, 0.25, 0.25, 0.25], [0.1, 0.2, 0.6, 0.1], [0.7, 0.1, 0.1, 0.1]]])
    tok = np.array([[0, 2, 0]])          # alpha = min(1, 2) = 1; 0.2 / 0.6 = 1/3; 0.25 / 0.7
    n, r, _ = R.accept_resample(pt, pd, tok, [[0.99, 0.30, 0.0]], [0.0])
    assert n.tolist() == [3] and r.tolist() == [-1]                  # 0.30 < 1/3: accepted; 0 < 0.357
    n, r, d = R.accept_resample(pt, pd, tok, [[0.99, 0.34, 0.0]], [0.5])
    assert n.tolist() == [1]                                          # rejected at position 1; the third is dropped
    # residual at position 1: max(0, pt - pd) = [0, 0.4, 0, 0] -> token 1 whatever u is
    assert r.tolist() == [1]
    np.testing.assert_allclose(d[0]["resid"], [0, 0.4, 0, 0], atol=1e-15)
    n, r, _ = R.accept_resample(pt, pd, tok, [[0.99, 0.2, 0.5]], [0.70])
    assert n.tolist() == [2]
    # residual at position 2: [0, .15, .15, .15]; cumulative .15 .30 .45; target .70 * .45 = .315 -> token 3
    assert r.tolist() == [3]
    n, r, _ = R.accept_resample(pt, pd, tok, [[0.99, 0.2, 0.5]], [0.0])
    assert r.tolist() == [1]                                          # the first token with positive residual


def test_acceptance_preserves_the_target_distribution():
    """Eq. 2-3 exist to make the emitted token follow p_theta: the exact law of the first emitted token,
    summed over draft token and outcome, must be p_theta (checked in closed form, no sampling)."""
    rng = np.random.default_rng(5)
    V = 6
    pt = rng.dirichlet(np.ones(V))
    pd = rng.dirichlet(np.ones(V))
    law = np.zeros(V)
    for x in range(V):                                    # the draft proposes x with probability pd[x]
        alpha = min(1.0, pt[x] / pd[x])
        law[x] += pd[x] * alpha
        # on rejection the oracle's residual law, read off through the inverse-CDF rule on a fine grid of u
        us = (np.arange(20000) + 0.5) / 20000
        _, r, _ = R.accept_resample(np.tile(pt, (us.size, 1, 1)), np.tile(pd, (us.size, 1, 1)),
                                    np.full((us.size, 1), x), np.full((us.size, 1), 1.0), us)
        law += pd[x] * (1 - alpha) * np.bincount(r, minlength=V) / us.size
    np.testing.assert_allclose(law, pt, atol=2e-4)


def test_identical_distributions_always_accept_and_zero_residual_falls_back():
    rng = np.random.default_rng(6)
    p = rng.dirichlet(np.ones(10), size=(2, 3))
    tok = rng.integers(0, 10, (2, 3))
    n, r, _ = R.accept_resample(p, p, tok, rng.random((2, 3)) * 0.999, [0.3, 0.6])
    assert n.tolist() == [3, 3] and r.tolist() == [-1, -1]
    n, r, _ = R.accept_resample(p, p, tok, np.ones((2, 3)), [0.0, 0.999999])      # u = 1 rejects even alpha = 1
    assert n.tolist() == [0, 0]
    assert r[0] == 0 and r[1] == 9                                     # sampled from p_theta itself
