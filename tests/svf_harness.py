"""Shared plumbing of the GPU parity tests: run the HIP path through the C ABI, run the oracle
on the same seeded inputs, compare.  Holds no arithmetic of the method."""
from __future__ import annotations

import numpy as np
import torch

import paper_2512_21911_amd as S
import workloads as W
from oracle import svf_oracle as O

OUT_TOL = {"f32": 1e-4, "bf16": 2e-2}      # max-abs on attention outputs
LSE_TOL = {"f32": 1e-4, "bf16": 1e-3}
REPS_TOL = 1e-5                            # |gpu - oracle| <= REPS_TOL * max(1, |oracle|)
TIE_GAP = 1e-3                             # relative score gap under which a selection mismatch is a near-tie


def shape_for(cfg: W.VerifyConfig, x, **over) -> S.SvfShape:
    kw = dict(B=cfg.B, gamma=cfg.gamma, Hq=cfg.Hq, Hkv=cfg.Hkv, d=cfg.d, dtype=cfg.dtype,
              block_size=cfg.block_size, max_seq_len=cfg.T, k_blocks=cfg.k_blocks, k_pool=x["k_pool"],
              page_size=cfg.page_size,
              max_pages_per_seq=(x["block_table"].shape[1] if x["block_table"] is not None else 0),
              n_sink=cfg.n_sink, n_local=cfg.n_local)
    kw.update(over)
    return S.make_shape(**kw)


def to_gpu(x):
    return {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in x.items()}


class DeviceRun:
    """Device buffers of one layer plus the results of the three calls."""

    def __init__(self, cfg, x_gpu, shape=None, poison=True):
        self.cfg, self.x = cfg, x_gpu
        self.shape = shape if shape is not None else shape_for(cfg, x_gpu)
        dev = "cuda"
        fill = float("nan") if poison else 0.0
        self.reps = torch.full((cfg.B, cfg.Hkv, cfg.nb_max, cfg.d), fill, device=dev, dtype=torch.float32)
        self.scores = torch.full((cfg.B, cfg.Hkv, cfg.nb_max), fill, device=dev, dtype=torch.float32)
        self.sel_idx = torch.full((cfg.B, cfg.Hkv, self.shape.k_blocks), -7, device=dev, dtype=torch.int32)
        self.sel_cnt = torch.full((cfg.B, cfg.Hkv), -7, device=dev, dtype=torch.int32)
        self.out = torch.full((cfg.B, cfg.gamma, cfg.Hq, cfg.d), fill, device=dev, dtype=cfg.torch_dtype)
        self.lse = torch.full((cfg.B, cfg.gamma, cfg.Hq), fill, device=dev, dtype=torch.float32)
        self.ws = S.new_workspace(self.shape)

    def block_reps(self, first_block=0, n_blocks=-1):
        x = self.x
        S.svf_block_reps(self.shape, x["k_pool"], x["block_table"], x["seq_lens"], self.reps, first_block, n_blocks)
        return self

    def score_select(self, with_scores=True):
        x = self.x
        S.svf_score_select(self.shape, x["q"], self.reps, x["seq_lens"], self.sel_idx, self.sel_cnt, self.ws,
                           self.scores if with_scores else None)
        return self

    def verify_attn(self, mask="auto", sel_idx=None, sel_cnt=None):
        x = self.x
        dm = x["draft_mask"] if mask == "auto" else mask
        S.svf_verify_attn(self.shape, x["q"], x["k_pool"], x["v_pool"], x["block_table"], x["seq_lens"],
                          x["k_draft"], x["v_draft"], dm,
                          self.sel_idx if sel_idx is None else sel_idx,
                          self.sel_cnt if sel_cnt is None else sel_cnt, self.out, self.ws, self.lse)
        return self

    def verify_step(self, do_select, mask="auto"):
        x = self.x
        dm = x["draft_mask"] if mask == "auto" else mask
        S.svf_verify_step(self.shape, do_select, x["q"], self.reps, x["k_pool"], x["v_pool"], x["block_table"],
                          x["seq_lens"], x["k_draft"], x["v_draft"], dm, self.sel_idx, self.sel_cnt,
                          self.out, self.ws, self.lse)
        return self

    def sync(self):
        torch.cuda.synchronize()
        return self


def oracle_reps(cfg, x):
    return O.block_reps(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)


def check_reps(cfg, x, reps_gpu, reps_ref=None):
    ref = oracle_reps(cfg, x) if reps_ref is None else reps_ref
    got = reps_gpu.double().cpu().numpy()
    lens = x["seq_lens"].cpu().tolist()
    for b, L in enumerate(lens):
        nb = -(-L // cfg.block_size)
        if nb == 0:
            continue
        err = np.abs(got[b, :, :nb] - ref[b, :, :nb]) / np.maximum(1.0, np.abs(ref[b, :, :nb]))
        assert np.isfinite(got[b, :, :nb]).all(), "non-finite representative"
        assert err.max() <= REPS_TOL, f"reps mismatch b={b}: {err.max():.3e}"
    return ref


def check_selection(cfg, x, scores_ref, idx_gpu, cnt_gpu, n_sink=0, n_local=0, k_blocks=None):
    """Bit-exact block sets, except blocks whose oracle score is within TIE_GAP (relative) of the
    weakest kept score.  Returns (oracle idx, oracle cnt, number of excused near-tie blocks)."""
    k = cfg.k_blocks if k_blocks is None else k_blocks
    idx_ref, cnt_ref = O.select_blocks(scores_ref, x["seq_lens"], cfg.block_size, k, n_sink, n_local)
    idx_g = idx_gpu.cpu().numpy()
    cnt_g = cnt_gpu.cpu().numpy()
    np.testing.assert_array_equal(cnt_g, cnt_ref)
    lens = x["seq_lens"].cpu().tolist()
    near = 0
    for b in range(cfg.B):
        nb = -(-lens[b] // cfg.block_size)
        for h in range(cfg.Hkv):
            c = int(cnt_ref[b, h])
            g = idx_g[b, h, :c]
            assert (np.diff(g) > 0).all(), "selected ids must ascend"
            assert (idx_g[b, h, c:] == -1).all(), "padding must be -1"
            if c == 0:
                continue
            assert g.min() >= 0 and g.max() < nb
            if (g == idx_ref[b, h, :c]).all():
                continue
            ties = set(O.near_tie_blocks(scores_ref[b, h], nb, idx_ref[b, h, :c], TIE_GAP, n_sink, n_local))
            diff = set(g.tolist()) ^ set(idx_ref[b, h, :c].tolist())
            assert diff <= ties, f"selection mismatch at (b={b}, h={h}): {sorted(diff)} not near-ties"
            near += len(diff)
    return idx_ref, cnt_ref, near


def oracle_attn(cfg, x, sel_idx, sel_cnt, mask="auto", sm_scale=None):
    dm = x["draft_mask"] if mask == "auto" else mask
    return O.verify_attn(x["q"], x["k_pool"], x["v_pool"], x["block_table"], x["seq_lens"],
                         x["k_draft"], x["v_draft"], dm, sel_idx, sel_cnt, cfg.block_size, sm_scale)


def check_attn(cfg, out_gpu, lse_gpu, out_ref, lse_ref):
    got = out_gpu.double().cpu().numpy()
    assert np.isfinite(got).all(), "non-finite attention output"
    err = np.abs(got - out_ref).max()
    assert err <= OUT_TOL[cfg.dtype], f"attention output max-abs error {err:.3e}"
    if lse_gpu is not None:
        lerr = np.abs(lse_gpu.double().cpu().numpy() - lse_ref).max()
        assert lerr <= LSE_TOL[cfg.dtype], f"lse max-abs error {lerr:.3e}"
    return err


def full_parity(cfg, layer=0, x=None):
    """reps -> scores/select -> attention on the GPU against the oracle; returns a small report."""
    x = W.make_layer(cfg, layer) if x is None else x
    run = DeviceRun(cfg, to_gpu(x))
    run.block_reps().score_select().verify_attn().sync()
    reps_ref = check_reps(cfg, x, run.reps)
    scores_ref = O.block_scores(x["q"], reps_ref)
    idx_ref, cnt_ref, near = check_selection(cfg, x, scores_ref, run.sel_idx, run.sel_cnt, cfg.n_sink, cfg.n_local)
    # attention is compared on the block set the GPU used (identical to the oracle's unless near-ties occurred)
    out_ref, lse_ref = oracle_attn(cfg, x, run.sel_idx.cpu(), run.sel_cnt.cpu())
    err = check_attn(cfg, run.out, run.lse, out_ref, lse_ref)
    # the fused step (selection + gather list + attention) and both reuse modes give the same bits
    out0, lse0, idx0, cnt0 = run.out.clone(), run.lse.clone(), run.sel_idx.clone(), run.sel_cnt.clone()
    for mode in (S.SVF_STEP_ANCHOR, S.SVF_STEP_REUSE_GATHER, S.SVF_STEP_REUSE):
        run.out.fill_(float("nan"))
        run.lse.fill_(float("nan"))
        if mode == S.SVF_STEP_ANCHOR:
            run.sel_idx.fill_(-7)
            run.sel_cnt.fill_(-7)
        run.verify_step(mode).sync()
        assert torch.equal(run.sel_idx, idx0) and torch.equal(run.sel_cnt, cnt0), f"step mode {mode}: selection"
        assert torch.equal(run.out.view(torch.uint8), out0.view(torch.uint8)), f"step mode {mode}: output bits"
        assert torch.equal(run.lse.view(torch.int32), lse0.view(torch.int32)), f"step mode {mode}: lse bits"
    return {"near_ties": near, "max_abs_err": err, "run": run, "x": x,
            "idx_ref": idx_ref, "cnt_ref": cnt_ref, "scores_ref": scores_ref}
