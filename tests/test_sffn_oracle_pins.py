"""Pins of the sparse feed-forward oracle (CPU): the library's own linear / activation routines,
identities that follow from Eq. 10-14, closed forms, and the workload recipe against the sparsity
levels the paper reports (Table 3)."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import sffn_oracle as FO
from workloads import ffn as WF

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sffn_sparsity_table3.txt")


def tiny(**kw):
    return WF.FFN_CONFIGS[1].scaled(**kw)


def args_of(w):
    return (w["x"], w["w_gate"], w["w_up"], w["w_down_t"], w["b_gate"], w["b_up"], w["b_down"])


@pytest.mark.parametrize("act", ["silu", "gelu"])
def test_dense_against_the_library_routines(act):
    """Eq. 10-11 with torch's linear and activation in fp64."""
    w = WF.make_ffn(tiny(act=act))
    x, wg, wu, wd, bg, bu, bd = [None if t is None else t.double() for t in args_of(w)]
    fn = F.silu if act == "silu" else F.gelu
    want = F.linear(fn(F.linear(x, wg, bg)) * F.linear(x, wu, bu), wd.t(), bd).numpy()
    got = FO.dense_ffn(*args_of(w), act=act)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(FO.gate(w["x"], w["w_gate"], w["b_gate"], act), fn(F.linear(x, wg, bg)).numpy(),
                               rtol=1e-12, atol=1e-13)


def test_activation_closed_forms():
    z = np.array([0.0, math.log(3.0), -math.log(3.0), 50.0, -50.0])
    np.testing.assert_allclose(FO.activation(z, "silu"),
                               [0.0, 0.75 * math.log(3.0), -0.25 * math.log(3.0), 50.0, 0.0], atol=1e-15)
    # GELU(z) + GELU(-z) = z * (Phi(z) - Phi(-z)) ... simplest identities: GELU(z) - GELU(-z) = z, GELU(0) = 0
    z = np.linspace(-6, 6, 25)
    np.testing.assert_allclose(FO.activation(z, "gelu") - FO.activation(-z, "gelu"), z, atol=1e-14)
    np.testing.assert_allclose(FO.activation(z, "silu") - FO.activation(-z, "silu"), z, atol=1e-14)
    with pytest.raises(ValueError):
        FO.activation(z, "relu6")


def test_worked_example_by_hand():
    """One token, two model dimensions, three hidden channels whose gate values are known in closed form."""
    ln3 = math.log(3.0)
    x = torch.tensor([[1.0, 2.0]])
    w_gate = torch.tensor([[0.0, 0.0], [ln3, 0.0], [-ln3, 0.0]])          # z = 0, ln 3, -ln 3
    w_up = torch.tensor([[5.0, 5.0], [1.0, 1.0], [2.0, -1.0]])            # up = 15, 3, 0 (+ bias)
    b_up = torch.tensor([0.0, 1.0, 4.0])                                  # up = 15, 4, 4
    w_down_t = torch.tensor([[7.0, 7.0], [1.0, -2.0], [10.0, 20.0]])
    b_down = torch.tensor([0.5, -0.5])
    h = [0.0, 0.75 * ln3, -0.25 * ln3]
    y, active, hh = FO.sparse_ffn(x, w_gate, w_up, w_down_t, None, b_up, b_down, "silu", tau=0.5)
    np.testing.assert_allclose(hh[0], h, atol=1e-15)
    assert active.tolist() == [[False, True, False]]                      # |h| = 0, 0.824, 0.275 against 0.5
    np.testing.assert_allclose(y[0], [0.5 + h[1] * 4 * 1.0, -0.5 + h[1] * 4 * -2.0], atol=1e-14)
    y, active, _ = FO.sparse_ffn(x, w_gate, w_up, w_down_t, None, b_up, b_down, "silu", tau=0.2)
    assert active.tolist() == [[False, True, True]]
    np.testing.assert_allclose(y[0], [0.5 + h[1] * 4 + h[2] * 4 * 10, -0.5 - h[1] * 8 + h[2] * 4 * 20], atol=1e-13)
    # the comparison of Eq. 12 is strict
    assert FO.inactive(np.array([[0.5, -0.5, 0.4999]]), 0.5).tolist() == [[False, False, True]]


def test_threshold_zero_is_the_dense_layer_and_infinity_leaves_the_bias():
    w = WF.make_ffn(tiny())
    dense = FO.dense_ffn(*args_of(w))
    y0, a0, _ = FO.sparse_ffn(*args_of(w), tau=0.0)
    assert a0.all()
    np.testing.assert_allclose(y0, dense, rtol=1e-12, atol=1e-13)
    yi, ai, _ = FO.sparse_ffn(*args_of(w), tau=float("inf"))
    assert not ai.any()
    np.testing.assert_allclose(yi, np.broadcast_to(w["b_down"].double().numpy(), yi.shape))


def test_index_form_equals_masked_form_and_the_dropped_terms():
    """Eq. 13-14 gather the channels outside S; multiplying the dense hidden vector by the 0/1 mask is
    the same thing, and the difference to the dense output is exactly the dropped channels' terms,
    each smaller than tau |up_i| |W_down[:, i]|."""
    cfg = tiny(M=5, tau=0.08)
    w = WF.make_ffn(cfg)
    x, wg, wu, wd, bg, bu, bd = [None if t is None else t.double().numpy() for t in args_of(w)]
    y, active, h = FO.sparse_ffn(*args_of(w), tau=cfg.tau)
    assert 0 < active.sum() < active.size
    up = x @ wu.T + bu
    masked = (h * up * active) @ wd + bd
    np.testing.assert_allclose(y, masked, rtol=1e-12, atol=1e-13)
    dense = FO.dense_ffn(*args_of(w))
    for m in range(cfg.M):
        dropped = np.flatnonzero(~active[m])
        terms = (h[m, dropped] * up[m, dropped])[:, None] * wd[dropped]
        np.testing.assert_allclose(dense[m] - y[m], terms.sum(axis=0), rtol=1e-10, atol=1e-13)
        bound = cfg.tau * (np.abs(up[m, dropped])[:, None] * np.abs(wd[dropped])).sum(axis=0)
        assert (np.abs(dense[m] - y[m]) <= bound + 1e-13).all()


def test_given_active_set_overrides_the_threshold():
    w = WF.make_ffn(tiny())
    _, a, _ = FO.sparse_ffn(*args_of(w), tau=0.05)
    flipped = a.copy()
    flipped[0, :10] = ~flipped[0, :10]
    y1, a1, _ = FO.sparse_ffn(*args_of(w), tau=123.0, active=flipped)
    assert (a1 == flipped).all()
    y2, _, _ = FO.sparse_ffn(*args_of(w), tau=0.05)
    assert np.abs(y1[0] - y2[0]).max() > 0 and np.array_equal(y1[1:], y2[1:])   # tokens are independent


def test_workload_reaches_the_sparsity_levels_of_table_3():
    """The synthetic gate scales are fitted to the mean sparsities the paper reports per threshold."""
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    cfg = WF.FFN_CONFIGS[2].scaled(M=16, d_ff=4096, d_model=512)
    w = WF.make_ffn(cfg)
    h = FO.gate(w["x"], w["w_gate"], None, "silu")
    for tau, s_f in rows:
        got = FO.inactive(h, float(tau)).mean()
        assert abs(got - float(s_f)) < 0.04, (tau, got)
    # and the quiet channels are shared by the tokens of a step: far more channels are inactive for all 8
    # tokens than independent draws would leave
    s = FO.inactive(h[:8], 0.05)
    assert s.all(axis=0).mean() > 5 * s.mean() ** 8 and s.all(axis=0).mean() > 0.15
