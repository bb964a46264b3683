"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and rejects bad
arguments before touching the GPU (none of these calls launches anything)."""
import ctypes
import os
import re

import pytest

import paper_2512_21911_amd as S
from oracle import svf_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(svf_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = S.lib()
    names = declared_symbols()
    assert {"svf_block_reps", "svf_score_select", "svf_verify_attn", "svf_verify_step"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def good_shape(**kw):
    base = dict(B=2, gamma=4, Hq=8, Hkv=2, d=128, dtype="bf16", block_size=64, max_seq_len=1024, k_blocks=4,
                page_size=16, max_pages_per_seq=64, kv_strides=(16 * 2 * 128, 2 * 128, 128))
    base.update(kw)
    return S.make_shape(**base)


def test_version_and_strerror():
    assert S.svf_version() >= 100
    for code in range(0, -8, -1):
        assert S.strerror(code) and "unknown" not in S.strerror(code)
    assert "unknown" in S.strerror(-99)


def test_budget_blocks_host_helper():
    assert S.svf_budget_blocks(32768, 4096, 0.1, 64) == O.budget_blocks(32768, 4096, 0.1, 64)
    assert S.svf_budget_blocks(4096, 4096, 0.1, 64) == (64, True)
    assert S.svf_budget_blocks(100000, 1024, 0.1, 16) == O.budget_blocks(100000, 1024, 0.1, 16)
    for bad in [(0, 10, 0.1, 16), (10, -1, 0.1, 16), (10, 5, 0.0, 16), (10, 5, 1.0, 16), (10, 5, 0.1, 0)]:
        with pytest.raises(S.SvfError):
            S.svf_budget_blocks(*bad)


@pytest.mark.parametrize("kw,code", [
    (dict(dtype=7), -3),
    (dict(gamma=0), -2), (dict(gamma=65), -2), (dict(Hq=7), -2), (dict(d=96), -2), (dict(block_size=0), -2),
    (dict(kv_strides=(4096, 100, 128)), -2), (dict(kv_strides=(4096, 256, 64)), -2),
    (dict(page_size=48), -4), (dict(max_pages_per_seq=8), -4),
    (dict(k_blocks=0), -5), (dict(n_sink=3, n_local=2), -5),
])
def test_shape_validation(kw, code):
    sh = good_shape(**kw)
    assert S.svf_workspace_bytes(sh) == 0
    fake = ctypes.c_void_p(0x1000)
    rc = S.lib().svf_block_reps(ctypes.byref(sh), fake, fake, fake, 0, -1, fake, None)
    assert rc == code
    rc = S.lib().svf_verify_attn(ctypes.byref(sh), *([fake] * 13), 1 << 30, None)
    assert rc == code


def test_null_alignment_and_workspace_checks():
    sh = good_shape()
    need = S.svf_workspace_bytes(sh)
    assert need > 0 and need % 256 == 0
    L = S.lib()
    ok, null = ctypes.c_void_p(0x10000), None
    assert L.svf_block_reps(ctypes.byref(sh), null, ok, ok, 0, -1, ok, None) == -1
    assert L.svf_block_reps(ctypes.byref(sh), ok, null, ok, 0, -1, ok, None) == -1          # paged needs a table
    assert L.svf_block_reps(ctypes.byref(sh), ctypes.c_void_p(0x10004), ok, ok, 0, -1, ok, None) == -2
    assert L.svf_block_reps(ctypes.byref(sh), ok, ok, ok, -1, -1, ok, None) == -2
    assert L.svf_block_reps(None, ok, ok, ok, 0, -1, ok, None) == -1
    args = [ok] * 13
    assert L.svf_verify_attn(ctypes.byref(sh), *args, need - 1, None) == -6
    args[12] = null
    assert L.svf_verify_attn(ctypes.byref(sh), *args, need, None) == -6
    args[12] = ctypes.c_void_p(0x10010)
    assert L.svf_verify_attn(ctypes.byref(sh), *args, need, None) == -6                     # misaligned workspace
    args = [ok] * 13
    args[7] = null                                                                           # draft mask may be NULL...
    args[11] = null                                                                          # ...and so may lse
    args[0] = null                                                                           # but q may not
    assert L.svf_verify_attn(ctypes.byref(sh), *args, need, None) == -1
    sargs = [ok] * 14
    sargs[1] = null                                                                          # reps required when selecting
    assert L.svf_verify_step(ctypes.byref(sh), 1, *sargs, need, None) == -1
    assert L.svf_verify_step(ctypes.byref(sh), 3, *([ok] * 14), need, None) == -2           # no such step mode
    assert L.svf_verify_step(ctypes.byref(sh), -1, *([ok] * 14), need, None) == -2
    assert L.svf_workspace_set_wait_polls(ctypes.byref(sh), ok, need, -2, None) == -2      # polls out of range
    assert L.svf_workspace_set_wait_polls(ctypes.byref(sh), ok, need, 4097, None) == -2
    assert L.svf_workspace_set_wait_polls(ctypes.byref(sh), null, need, 8, None) == -6     # no workspace
    assert L.svf_workspace_set_wait_polls(ctypes.byref(sh), ok, need - 256, 8, None) == -6
    assert L.svf_diag_wait_fallbacks(ctypes.byref(sh), null, need, ok, None) == -6          # no workspace
    assert L.svf_diag_wait_fallbacks(ctypes.byref(sh), ok, need - 256, ok, None) == -6
    assert L.svf_diag_wait_fallbacks(ctypes.byref(sh), ok, need, null, None) == -1           # nowhere to put the counts
    assert L.svf_score_select(ctypes.byref(sh), ok, ok, ok, ok, ok, null, ok, need - 256, None) == -6
    assert L.svf_workspace_init(null, 256, None) == -1
    assert L.svf_workspace_init(ctypes.c_void_p(0x10010), 256, None) == -6


def test_contiguous_cache_needs_no_table():
    sh = good_shape(page_size=0, max_pages_per_seq=0, kv_strides=(1024 * 256, 256, 128))
    assert S.svf_workspace_bytes(sh) > 0
    # argument checks pass up to the (undersized) workspace: no table required
    ok = ctypes.c_void_p(0x10000)
    args = [ok] * 13
    args[3] = None
    assert S.lib().svf_verify_attn(ctypes.byref(sh), *args, 0, None) == -6


def test_analytics_entry_points_validate_before_launching():
    sh = good_shape()
    L = S.lib()
    ok, null = ctypes.c_void_p(0x10000), None
    assert S.svf_mask_words(sh) == -(-(sh.max_seq_len // sh.block_size) // 64)
    need = L.svf_analytics_workspace_bytes(ctypes.byref(sh))
    assert need > 0 and need % 256 == 0
    assert L.svf_select_per_draft(ctypes.byref(sh), null, ok, ok, ok, ok, ok, need, None) == -1
    assert L.svf_select_per_draft(ctypes.byref(sh), ok, ok, ok, ok, null, null, 0, None) == -6      # needs scores or ws
    assert L.svf_select_per_draft(ctypes.byref(sh), ok, ok, ok, ok, null, ok, need - 1, None) == -6
    assert L.svf_masks_from_selection(ctypes.byref(sh), ok, null, ok, None) == -1
    assert L.svf_overlap_by_distance(ctypes.byref(sh), ok, ok, 0, ok, None) == -2
    assert L.svf_overlap_by_distance(ctypes.byref(sh), ok, ok, 65, ok, None) == -2
    assert L.svf_overlap_by_distance(ctypes.byref(sh), ok, null, 4, ok, None) == -1
    assert L.svf_jaccard_adjacent(ctypes.byref(sh), ok, 0, ok, None) == -2
    assert L.svf_jaccard_adjacent(ctypes.byref(sh), null, 4, ok, None) == -1


def test_topk_anchors_matches_the_oracle():
    """Eq. 8 runs on the host: compare with the oracle on random similarities, ties included."""
    import numpy as np
    from oracle import svf_analytics_oracle as A
    rng = np.random.default_rng(3)
    for trial in range(50):
        n = int(rng.integers(1, 40))
        J = np.round(rng.random(n), 1 if trial % 2 else 6)     # coarse rounding makes ties
        J[0] = 0.0
        for K in {1, n, int(rng.integers(1, n + 1))}:
            assert S.svf_topk_anchors(J.tolist(), K) == A.topk_anchors(J, K)
    L = S.lib()
    arr = (ctypes.c_double * 3)(0.0, 0.5, 1.5)
    out = (ctypes.c_int32 * 3)()
    assert L.svf_topk_anchors(arr, 3, 2, out) == -2            # a similarity above 1
    arr = (ctypes.c_double * 3)(0.0, float("nan"), 0.5)
    assert L.svf_topk_anchors(arr, 3, 2, out) == -2
    arr = (ctypes.c_double * 3)(0.0, 0.5, 0.5)
    assert L.svf_topk_anchors(arr, 3, 0, out) == -2 and L.svf_topk_anchors(arr, 3, 4, out) == -2
    assert L.svf_topk_anchors(None, 3, 1, out) == -1


def test_retrieval_variants_validate_before_launching():
    sh = good_shape()                                   # nb_max = 16, k_blocks = 4, Hkv = 2
    L = S.lib()
    ok, null = ctypes.c_void_p(0x10000), None
    need = S.svf_workspace_bytes(sh)

    def retrieve(rt, shape=sh, q=ok, ws=ok, ws_bytes=need):
        return L.svf_retrieve(ctypes.byref(shape), ctypes.byref(rt) if rt is not None else None, q, ok, ok, ok, ok,
                              null, ws, ws_bytes, None)

    def summaries(rt, out=ok):
        return L.svf_block_summaries(ctypes.byref(sh), ctypes.byref(rt) if rt is not None else None, ok, ok, ok, 0,
                                     -1, out, None)

    good = S.SvfRetrieval(S.SVF_SUMMARY_MINMAX, S.SVF_BF16, S.SVF_GROUP_MAX, S.SVF_BUDGET_PER_HEAD, 0)
    assert retrieve(None) == -1 and summaries(None) == -1
    assert retrieve(S.SvfRetrieval(2, 0, 0, 0, 0)) == -2 and summaries(S.SvfRetrieval(2, 0, 0, 0, 0)) == -2
    assert retrieve(S.SvfRetrieval(0, 2, 0, 0, 0)) == -3
    assert retrieve(S.SvfRetrieval(0, 0, 2, 0, 0)) == -2
    assert retrieve(S.SvfRetrieval(0, 0, 0, 2, 0)) == -2
    assert retrieve(good, q=null) == -1 and summaries(good, out=null) == -1
    assert retrieve(good, ws=null) == -6 and retrieve(good, ws_bytes=need - 1) == -6
    # global budget: at least one pair, the forced pairs must fit, and sel_idx rows must hold a head's share
    glob = lambda n: S.SvfRetrieval(0, 0, 0, S.SVF_BUDGET_GLOBAL, n)
    assert retrieve(glob(0)) == -5
    assert retrieve(glob(8)) == -5                                        # k_blocks 4 < min(16, 8)
    assert retrieve(glob(4), ws_bytes=0) == -6                            # budget accepted, then the workspace check
    sink = good_shape(n_sink=1, n_local=1, k_blocks=4)
    assert retrieve(glob(3), shape=sink) == -5                            # 2 heads x 2 forced blocks > 3
    assert retrieve(glob(4), shape=sink, ws_bytes=0) == -6


def test_sparse_ffn_validates_before_launching():
    L = S.lib()
    ok, null = ctypes.c_void_p(0x10000), None
    sh = S.make_ffn_shape(M=8, d_model=256, d_ff=64, act="silu", tau=0.05)
    need = S.svf_ffn_workspace_bytes(sh)
    assert need > 0 and need % 256 == 0

    def call(shape=sh, x=ok, y=ok, ws=ok, ws_bytes=need, b=null, active=null):
        return L.svf_sparse_ffn(ctypes.byref(shape), x, ok, ok, ok, b, null, null, y, active, ws, ws_bytes, None)

    for bad in (dict(M=0), dict(M=65), dict(d_model=192), dict(d_model=0), dict(d_ff=48), dict(d_ff=0), dict(act=2), dict(walk=3), dict(walk=-1),
                dict(tau=-0.1), dict(tau=float("nan")), dict(tau=float("inf"))):
        kw = dict(M=8, d_model=256, d_ff=64, act="silu", tau=0.05)
        kw.update(bad)
        assert S.svf_ffn_workspace_bytes(S.make_ffn_shape(**kw)) == 0, bad
        assert call(shape=S.make_ffn_shape(**kw)) == -2, bad
    assert call(x=null) == -1 and call(y=null) == -1
    assert call(x=ctypes.c_void_p(0x10008)) == -2 and call(b=ctypes.c_void_p(0x10004)) == -2
    assert call(active=ctypes.c_void_p(0x10004)) == -2
    assert call(ws=null) == -6 and call(ws=ctypes.c_void_p(0x10010)) == -6 and call(ws_bytes=need - 1) == -6


def test_rules_validate_before_launching():
    L = S.lib()
    ok, null = ctypes.c_void_p(0x10000), None
    assert L.svf_moe_skip(null, 4, 8, 2, ok, ok, ok, None) == -1
    assert L.svf_moe_skip(ok, 0, 8, 2, ok, ok, ok, None) == -2
    assert L.svf_moe_skip(ok, 4, 1, 1, ok, ok, ok, None) == -2 and L.svf_moe_skip(ok, 4, 33, 1, ok, ok, ok, None) == -2
    assert L.svf_moe_skip(ok, 4, 8, 0, ok, ok, ok, None) == -5 and L.svf_moe_skip(ok, 4, 8, 8, ok, ok, ok, None) == -5
    need = L.svf_moe_calibrate_workspace_bytes(1000, 8)
    assert need == -(-7 * 1000 * 4 // 256) * 256 and L.svf_moe_calibrate_workspace_bytes(0, 8) == 0
    assert L.svf_moe_calibrate_workspace_bytes(10, 40) == 0
    assert L.svf_moe_calibrate(ok, 1000, 8, null, ok, need, None) == -1
    assert L.svf_moe_calibrate(ok, 1000, 8, ok, ok, need - 1, None) == -6
    assert L.svf_moe_calibrate(ok, 1000, 8, ok, ctypes.c_void_p(0x10010), need, None) == -6
    args = [ok] * 5
    assert L.svf_accept_resample(*args, 2, 4, 100, ok, null, None) == -1
    assert L.svf_accept_resample(*args, 0, 4, 100, ok, ok, None) == -2
    assert L.svf_accept_resample(*args, 2, 65, 100, ok, ok, None) == -2
    assert L.svf_accept_resample(*args, 2, 4, 0, ok, ok, None) == -2
    assert L.svf_accept_resample(*args, 2, 4, 524289, ok, ok, None) == -2

