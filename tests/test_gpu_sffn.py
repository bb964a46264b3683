"""GPU parity of the sparse feed-forward verification (Sec. 3.4, Eq. 10-14), through the C ABI,
against the fp64 oracle on the same seeded inputs.

Bars.  The active set (Eq. 12) is decided on the device's fp32 gate value: it must equal the
oracle's except for channels whose |h| lies within 2e-5 + 1e-5 |h| of tau (counted).  The output
is compared with the oracle evaluated on the set the device used; the bound is derived from the
arithmetic: the per-channel products are rounded to bf16 once (8 significant bits: relative 2^-8)
and so is y, all sums are fp32, hence |y_gpu - y_ref| <= 2^-7 * A with A = sum_i |h_i up_i|
|W_down[n, i]| + |b_down| >= |y|, with 5 % slack for the fp32 sums."""
import numpy as np
import pytest
import torch

import paper_2512_21911_amd as S
from oracle import sffn_oracle as FO
from workloads import ffn as WF

pytestmark = pytest.mark.gpu


WALKS = {"together": S.SVF_FFN_WALK_TOGETHER, "gate_first": S.SVF_FFN_WALK_GATE_FIRST}


def run_gpu(cfg, w, tau=None, walk=S.SVF_FFN_WALK_AUTO):
    tau = cfg.tau if tau is None else tau
    shape = S.make_ffn_shape(M=cfg.M, d_model=cfg.d_model, d_ff=cfg.d_ff, act=cfg.act, tau=tau, walk=walk)
    g = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in w.items()}
    y = torch.full((cfg.M, cfg.d_model), float("nan"), device="cuda", dtype=torch.bfloat16)
    active = torch.full((cfg.d_ff,), -1, device="cuda", dtype=torch.int64)
    ws = S.new_ffn_workspace(shape)
    ws.fill_(0xff)                                        # the workspace needs no initialisation
    S.svf_sparse_ffn(shape, g["x"], g["w_gate"], g["w_up"], g["w_down_t"], y, ws, g["b_gate"], g["b_up"], g["b_down"],
                     active)
    torch.cuda.synchronize()
    bits = active.cpu().numpy().view(np.uint64)
    act = ((bits[None, :] >> np.arange(cfg.M, dtype=np.uint64)[:, None]) & np.uint64(1)).astype(bool)   # [M][d_ff]
    assert (bits >> np.uint64(cfg.M) == 0).all() if cfg.M < 64 else True, "bits of tokens that do not exist"
    return y.double().cpu().numpy(), act


def check(cfg, w, tau=None, tokens=None, walk=S.SVF_FFN_WALK_AUTO):
    tau = cfg.tau if tau is None else tau
    y, act = run_gpu(cfg, w, tau, walk)
    toks = list(range(cfg.M)) if tokens is None else tokens
    sub = dict(w)
    sub["x"] = w["x"][toks]
    args = (sub["x"], w["w_gate"], w["w_up"], w["w_down_t"], w["b_gate"], w["b_up"], w["b_down"])
    _, act_ref, h = FO.sparse_ffn(*args, act=cfg.act, tau=tau)
    flips = act[toks] != act_ref
    near = np.abs(np.abs(h) - tau) <= 2e-5 + 1e-5 * np.abs(h)
    assert (flips <= near).all(), f"{int((flips & ~near).sum())} active bits differ away from the threshold"
    y_ref, _, _ = FO.sparse_ffn(*args, act=cfg.act, tau=tau, active=act[toks])
    wd = w["w_down_t"].double().numpy()
    up = sub["x"].double().numpy() @ w["w_up"].double().numpy().T + (0 if w["b_up"] is None else w["b_up"].double().numpy())
    A = (np.abs(h * up) * act[toks]) @ np.abs(wd) + (0 if w["b_down"] is None else np.abs(w["b_down"].double().numpy()))
    err = np.abs(y[toks] - y_ref)
    assert np.isfinite(y).all()
    worst = float((err / (2.0 ** -7 * 1.05 * A + 1e-6)).max())
    assert worst <= 1.0, f"output error {worst:.2f} x the derived bound"
    print(f"[sffn] {cfg.name} walk={walk} M={cfg.M} tau={tau}: active {act[toks].mean():.3f}, rows read "
          f"{act.any(axis=0).mean():.3f}, flips {int(flips.sum())}, error {worst:.2f} of the bound", flush=True)
    return y, act


@pytest.mark.parametrize("walk", sorted(WALKS))
@pytest.mark.parametrize("act", ["silu", "gelu"])
def test_tiny_with_biases(act, walk):
    cfg = WF.FFN_CONFIGS[1].scaled(act=act)
    check(cfg, WF.make_ffn(cfg), walk=WALKS[walk])


@pytest.mark.parametrize("walk", sorted(WALKS))
@pytest.mark.parametrize("tau", [0.0, 0.01, 0.05, 0.1])
def test_expert_shape_at_the_papers_thresholds(tau, walk):
    cfg = WF.FFN_CONFIGS[2]
    w = WF.make_ffn(cfg)
    y, act = check(cfg, w, tau, walk=WALKS[walk])
    if tau == 0.0:                                        # Eq. 10-11: the dense layer
        assert act.all()
        dense = FO.dense_ffn(w["x"], w["w_gate"], w["w_up"], w["w_down_t"], act=cfg.act)
        assert np.abs(y - dense).max() <= 2e-2 * max(1.0, np.abs(dense).max())


@pytest.mark.parametrize("walk", sorted(WALKS))
@pytest.mark.parametrize("M", [1, 31, 32, 33, 60, 64])
def test_token_counts(M, walk):
    cfg = WF.FFN_CONFIGS[2].scaled(M=M, d_model=512, d_ff=352, bias=True)
    check(cfg, WF.make_ffn(cfg), walk=WALKS[walk])


@pytest.mark.parametrize("M", [5, 40])
@pytest.mark.parametrize("walk", sorted(WALKS))
@pytest.mark.parametrize("d_model,d_ff", [(128, 32), (384, 96), (640, 2080), (1024, 32), (256, 7200)])
def test_ragged_splits(d_model, d_ff, walk, M):
    """Fewer chunks than wavefronts, chunk counts that do not divide by four, one tile, hidden sizes that
    leave wavefronts of the down projection without a step, a hidden size whose tiles of the joint walk
    are cut below 32 channels with a last tile moved back; with 40 tokens the joint walk takes two tiles
    per workgroup (an odd tile count leaves the last workgroup a repeated tile)."""
    cfg = WF.FFN_CONFIGS[1].scaled(M=M, d_model=d_model, d_ff=d_ff)
    check(cfg, WF.make_ffn(cfg), walk=WALKS[walk])


@pytest.mark.parametrize("walk", sorted(WALKS))
def test_everything_inactive_leaves_the_bias(walk):
    cfg = WF.FFN_CONFIGS[1].scaled(M=4, d_model=256, d_ff=128)
    w = WF.make_ffn(cfg)
    y, act = check(cfg, w, tau=1e6, walk=WALKS[walk])
    assert not act.any()
    want = w["b_down"].to(torch.bfloat16).double().numpy()
    assert np.array_equal(y, np.broadcast_to(want, y.shape))


@pytest.mark.parametrize("walk", sorted(WALKS))
def test_dense_8b_full_size(walk):
    """The benchmark's shape; the oracle checks every token."""
    cfg = WF.FFN_CONFIGS[3]
    check(cfg, WF.make_ffn(cfg), walk=WALKS[walk])


@pytest.mark.parametrize("walk", sorted(WALKS))
def test_dense_8b_tree_full_size_sampled_tokens(walk):
    cfg = WF.FFN_CONFIGS[4]
    check(cfg, WF.make_ffn(cfg), tokens=[0, 31, 32, 59], walk=WALKS[walk])


@pytest.mark.parametrize("walk", sorted(WALKS))
def test_same_bits_on_repeated_calls(walk):
    cfg = WF.FFN_CONFIGS[2]
    w = WF.make_ffn(cfg)
    y0, a0 = run_gpu(cfg, w, walk=WALKS[walk])
    for _ in range(3):
        y1, a1 = run_gpu(cfg, w, walk=WALKS[walk])
        assert np.array_equal(y0, y1) and np.array_equal(a0, a1)
