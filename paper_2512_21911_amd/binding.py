"""ctypes binding of libsvf: argument marshalling only.

Every function here has the name of the C entry point it calls (include/svf.h) and does no
arithmetic of its own.  Tensors are torch CUDA tensors used purely as device memory; work is
enqueued on torch's current stream.  A missing library is an error: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from .build import LIB_PATH

SVF_F32, SVF_BF16 = 0, 1

ERR_NAMES = {0: "SVF_OK", -1: "SVF_ERR_NULL", -2: "SVF_ERR_SHAPE", -3: "SVF_ERR_DTYPE", -4: "SVF_ERR_PAGING",
             -5: "SVF_ERR_BUDGET", -6: "SVF_ERR_WORKSPACE", -7: "SVF_ERR_HIP"}


class SvfShape(ctypes.Structure):
    """Mirror of svf_shape_t."""
    _fields_ = [
        ("B", ctypes.c_int32), ("gamma", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("d", ctypes.c_int32), ("dtype", ctypes.c_int32), ("block_size", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("max_pages_per_seq", ctypes.c_int32), ("max_seq_len", ctypes.c_int32),
        ("kv_stride_page", ctypes.c_int64), ("kv_stride_tok", ctypes.c_int64), ("kv_stride_head", ctypes.c_int64),
        ("k_blocks", ctypes.c_int32), ("n_sink", ctypes.c_int32), ("n_local", ctypes.c_int32),
        ("mask_per_batch", ctypes.c_int32), ("sm_scale", ctypes.c_float),
    ]


class SvfRetrieval(ctypes.Structure):
    """Mirror of svf_retrieval_t."""
    _fields_ = [("summary", ctypes.c_int32), ("summary_dtype", ctypes.c_int32), ("group_rule", ctypes.c_int32),
                ("budget_rule", ctypes.c_int32), ("n_total", ctypes.c_int32)]


SVF_SUMMARY_MEAN, SVF_SUMMARY_MINMAX = 0, 1
SVF_GROUP_MEAN, SVF_GROUP_MAX = 0, 1
SVF_BUDGET_PER_HEAD, SVF_BUDGET_GLOBAL = 0, 1


class SvfFfnShape(ctypes.Structure):
    """Mirror of svf_ffn_shape_t (include/svf_ffn.h)."""
    _fields_ = [("M", ctypes.c_int32), ("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("act", ctypes.c_int32),
                ("tau", ctypes.c_float), ("walk", ctypes.c_int32)]


SVF_ACT_SILU, SVF_ACT_GELU = 0, 1
SVF_FFN_WALK_AUTO, SVF_FFN_WALK_GATE_FIRST, SVF_FFN_WALK_TOGETHER = 0, 1, 2


class SvfError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {ERR_NAMES.get(code, code)} ({strerror(code)})")


_lib = None

EXPORTS = ["svf_version", "svf_strerror", "svf_budget_blocks", "svf_workspace_bytes", "svf_workspace_init",
           "svf_block_reps", "svf_score_select", "svf_verify_attn", "svf_verify_step", "svf_workspace_set_wait_polls",
           "svf_static_workspace_bytes", "svf_verify_attn_static_ws", "svf_diag_workspace_bytes", "svf_diag_verify_attn", "svf_diag_wait_fallbacks",
           "svf_mask_words", "svf_analytics_workspace_bytes", "svf_select_per_draft", "svf_masks_from_selection",
           "svf_overlap_by_distance", "svf_jaccard_adjacent", "svf_topk_anchors",
           "svf_block_summaries", "svf_retrieve", "svf_ffn_workspace_bytes", "svf_sparse_ffn",
           "svf_moe_skip", "svf_moe_calibrate_workspace_bytes", "svf_moe_calibrate", "svf_accept_resample"]


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (python -m paper_2512_21911_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                               "or `python -m paper_2512_21911_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        shp = ctypes.POINTER(SvfShape)
        L.svf_version.restype = ctypes.c_int
        L.svf_static_workspace_bytes.restype = ctypes.c_size_t
        L.svf_static_workspace_bytes.argtypes = []
        L.svf_verify_attn_static_ws.restype = ctypes.c_int
        L.svf_verify_attn_static_ws.argtypes = [shp] + [vp] * 13
        L.svf_diag_workspace_bytes.restype = ctypes.c_size_t
        L.svf_diag_workspace_bytes.argtypes = [shp, ctypes.c_int]
        L.svf_diag_wait_fallbacks.restype = ctypes.c_int
        L.svf_diag_wait_fallbacks.argtypes = [shp, vp, ctypes.c_size_t, vp, vp]
        L.svf_diag_verify_attn.restype = ctypes.c_int
        L.svf_diag_verify_attn.argtypes = [shp, ctypes.c_int] + [vp] * 13 + [ctypes.c_size_t, vp]
        L.svf_workspace_set_wait_polls.restype = ctypes.c_int
        L.svf_workspace_set_wait_polls.argtypes = [shp, vp, ctypes.c_size_t, ctypes.c_int, vp]
        L.svf_mask_words.restype = i32
        L.svf_mask_words.argtypes = [shp]
        L.svf_analytics_workspace_bytes.restype = ctypes.c_size_t
        L.svf_analytics_workspace_bytes.argtypes = [shp]
        L.svf_select_per_draft.restype = ctypes.c_int
        L.svf_select_per_draft.argtypes = [shp] + [vp] * 6 + [ctypes.c_size_t, vp]
        L.svf_masks_from_selection.restype = ctypes.c_int
        L.svf_masks_from_selection.argtypes = [shp] + [vp] * 4
        L.svf_overlap_by_distance.restype = ctypes.c_int
        L.svf_overlap_by_distance.argtypes = [shp, vp, vp, i32, vp, vp]
        L.svf_jaccard_adjacent.restype = ctypes.c_int
        L.svf_jaccard_adjacent.argtypes = [shp, vp, i32, vp, vp]
        L.svf_topk_anchors.restype = ctypes.c_int
        L.svf_topk_anchors.argtypes = [ctypes.POINTER(ctypes.c_double), i32, i32, ctypes.POINTER(i32)]
        rtp = ctypes.POINTER(SvfRetrieval)
        L.svf_block_summaries.restype = ctypes.c_int
        L.svf_block_summaries.argtypes = [shp, rtp, vp, vp, vp, i32, i32, vp, vp]
        L.svf_retrieve.restype = ctypes.c_int
        L.svf_retrieve.argtypes = [shp, rtp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        fsp = ctypes.POINTER(SvfFfnShape)
        L.svf_ffn_workspace_bytes.restype = ctypes.c_size_t
        L.svf_ffn_workspace_bytes.argtypes = [fsp]
        L.svf_sparse_ffn.restype = ctypes.c_int
        L.svf_sparse_ffn.argtypes = [fsp] + [vp] * 10 + [ctypes.c_size_t, vp]
        L.svf_moe_skip.restype = ctypes.c_int
        L.svf_moe_skip.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp]
        L.svf_moe_calibrate_workspace_bytes.restype = ctypes.c_size_t
        L.svf_moe_calibrate_workspace_bytes.argtypes = [i32, i32]
        L.svf_moe_calibrate.restype = ctypes.c_int
        L.svf_moe_calibrate.argtypes = [vp, i32, i32, vp, vp, ctypes.c_size_t, vp]
        L.svf_accept_resample.restype = ctypes.c_int
        L.svf_accept_resample.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp]
        L.svf_version.argtypes = []
        L.svf_strerror.restype = ctypes.c_char_p
        L.svf_strerror.argtypes = [ctypes.c_int]
        L.svf_budget_blocks.restype = i32
        L.svf_budget_blocks.argtypes = [i64, i64, ctypes.c_double, i32, ctypes.POINTER(i32)]
        L.svf_workspace_bytes.restype = ctypes.c_size_t
        L.svf_workspace_bytes.argtypes = [shp]
        L.svf_workspace_init.restype = ctypes.c_int
        L.svf_workspace_init.argtypes = [vp, ctypes.c_size_t, vp]
        L.svf_block_reps.restype = ctypes.c_int
        L.svf_block_reps.argtypes = [shp, vp, vp, vp, i32, i32, vp, vp]
        L.svf_score_select.restype = ctypes.c_int
        L.svf_score_select.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.svf_verify_attn.restype = ctypes.c_int
        L.svf_verify_attn.argtypes = [shp] + [vp] * 13 + [ctypes.c_size_t, vp]
        L.svf_verify_step.restype = ctypes.c_int
        L.svf_verify_step.argtypes = [shp, ctypes.c_int] + [vp] * 14 + [ctypes.c_size_t, vp]
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str):
    if rc != 0:
        raise SvfError(rc, where)


def svf_version() -> int:
    return lib().svf_version()


def strerror(code: int) -> str:
    return lib().svf_strerror(code).decode()


def svf_budget_blocks(L: int, L0: int, rho: float, block_size: int):
    dense = ctypes.c_int32(0)
    k = lib().svf_budget_blocks(L, L0, rho, block_size, ctypes.byref(dense))
    if k < 0:
        raise SvfError(k, "svf_budget_blocks")
    return k, bool(dense.value)


def make_shape(*, B, gamma, Hq, Hkv, d, dtype, block_size, max_seq_len, k_blocks, k_pool: Optional[torch.Tensor] = None,
               page_size=0, max_pages_per_seq=0, n_sink=0, n_local=0, mask_per_batch=0, sm_scale=0.0,
               kv_strides=None) -> SvfShape:
    """Fill an svf_shape_t.  Strides come from `kv_strides` = (page, token, head) in elements, or
    from a pool tensor laid out [page][slot][Hkv][d]."""
    if kv_strides is None:
        kv_strides = (k_pool.stride(0), k_pool.stride(1), k_pool.stride(2))
    code = {torch.float32: SVF_F32, torch.bfloat16: SVF_BF16, "f32": SVF_F32, "bf16": SVF_BF16}.get(dtype, dtype)
    return SvfShape(B, gamma, Hq, Hkv, d, code, block_size, page_size, max_pages_per_seq, max_seq_len,
                    kv_strides[0], kv_strides[1], kv_strides[2], k_blocks, n_sink, n_local, mask_per_batch, sm_scale)


def svf_workspace_bytes(shape: SvfShape) -> int:
    return lib().svf_workspace_bytes(ctypes.byref(shape))


def svf_workspace_init(ws: torch.Tensor):
    _check(lib().svf_workspace_init(_ptr(ws), ws.numel() * ws.element_size(), _stream()), "svf_workspace_init")


def new_workspace(shape: SvfShape, device="cuda") -> torch.Tensor:
    """Allocate (through torch) and clear a workspace for `shape`."""
    n = svf_workspace_bytes(shape)
    if n == 0:
        raise SvfError(-2, "svf_workspace_bytes")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    svf_workspace_init(ws)
    return ws


def svf_block_reps(shape, K, block_table, seq_lens, reps, first_block=0, n_blocks=-1):
    _check(lib().svf_block_reps(ctypes.byref(shape), _ptr(K), _ptr(block_table), _ptr(seq_lens),
                                first_block, n_blocks, _ptr(reps), _stream()), "svf_block_reps")


def svf_score_select(shape, q, reps, seq_lens, sel_idx, sel_cnt, ws, scores=None):
    _check(lib().svf_score_select(ctypes.byref(shape), _ptr(q), _ptr(reps), _ptr(seq_lens), _ptr(sel_idx),
                                  _ptr(sel_cnt), _ptr(scores), _ptr(ws), ws.numel(), _stream()),
           "svf_score_select")


def svf_verify_attn(shape, q, K, V, block_table, seq_lens, k_draft, v_draft, draft_mask, sel_idx, sel_cnt,
                    out, ws, lse=None):
    _check(lib().svf_verify_attn(ctypes.byref(shape), _ptr(q), _ptr(K), _ptr(V), _ptr(block_table),
                                 _ptr(seq_lens), _ptr(k_draft), _ptr(v_draft), _ptr(draft_mask),
                                 _ptr(sel_idx), _ptr(sel_cnt), _ptr(out), _ptr(lse), _ptr(ws), ws.numel(),
                                 _stream()), "svf_verify_attn")


def svf_verify_attn_static_ws(shape, q, K, V, block_table, seq_lens, k_draft, v_draft, draft_mask, sel_idx, sel_cnt,
                              out, lse=None):
    _check(lib().svf_verify_attn_static_ws(ctypes.byref(shape), _ptr(q), _ptr(K), _ptr(V), _ptr(block_table),
                                           _ptr(seq_lens), _ptr(k_draft), _ptr(v_draft), _ptr(draft_mask),
                                           _ptr(sel_idx), _ptr(sel_cnt), _ptr(out), _ptr(lse), _stream()),
           "svf_verify_attn_static_ws")


SVF_KERNEL_AUTO, SVF_KERNEL_VECTOR_ALU = 0, 1


def new_diag_workspace(shape, kernel, device="cuda") -> torch.Tensor:
    n = int(lib().svf_diag_workspace_bytes(ctypes.byref(shape), int(kernel)))
    if n == 0:
        raise SvfError(-2, "svf_diag_workspace_bytes")
    return torch.zeros(n, dtype=torch.uint8, device=device)


def svf_diag_wait_fallbacks(shape, ws):
    """(exchange fallbacks, merge fallbacks) counted in `ws` since it was last cleared; synchronises."""
    counts = torch.zeros(2, dtype=torch.int64, device=ws.device)
    _check(lib().svf_diag_wait_fallbacks(ctypes.byref(shape), _ptr(ws), ws.numel(), _ptr(counts), _stream()),
           "svf_diag_wait_fallbacks")
    return tuple(int(v) for v in counts.cpu())


def svf_diag_verify_attn(shape, kernel, q, K, V, block_table, seq_lens, k_draft, v_draft, draft_mask, sel_idx, sel_cnt,
                         out, ws, lse=None):
    _check(lib().svf_diag_verify_attn(ctypes.byref(shape), int(kernel), _ptr(q), _ptr(K), _ptr(V), _ptr(block_table),
                                      _ptr(seq_lens), _ptr(k_draft), _ptr(v_draft), _ptr(draft_mask), _ptr(sel_idx),
                                      _ptr(sel_cnt), _ptr(out), _ptr(lse), _ptr(ws), ws.numel(), _stream()),
           "svf_diag_verify_attn")


def svf_static_workspace_bytes() -> int:
    return int(lib().svf_static_workspace_bytes())


SVF_STEP_REUSE, SVF_STEP_ANCHOR, SVF_STEP_REUSE_GATHER = 0, 1, 2


def svf_workspace_set_wait_polls(shape, ws, polls):
    _check(lib().svf_workspace_set_wait_polls(ctypes.byref(shape), _ptr(ws), ws.numel(), int(polls), _stream()),
           "svf_workspace_set_wait_polls")


def svf_verify_step(shape, mode, q, reps, K, V, block_table, seq_lens, k_draft, v_draft, draft_mask,
                    sel_idx, sel_cnt, out, ws, lse=None):
    _check(lib().svf_verify_step(ctypes.byref(shape), int(mode), _ptr(q), _ptr(reps), _ptr(K), _ptr(V),
                                 _ptr(block_table), _ptr(seq_lens), _ptr(k_draft), _ptr(v_draft),
                                 _ptr(draft_mask), _ptr(sel_idx), _ptr(sel_cnt), _ptr(out), _ptr(lse),
                                 _ptr(ws), ws.numel(), _stream()), "svf_verify_step")


# ---- retrieval analytics (argument marshalling only) ------------------------------------------

def svf_mask_words(shape) -> int:
    return int(lib().svf_mask_words(ctypes.byref(shape)))


def new_analytics_workspace(shape, device="cuda"):
    import torch
    n = int(lib().svf_analytics_workspace_bytes(ctypes.byref(shape)))
    if n == 0:
        raise SvfError("svf_analytics_workspace_bytes: invalid shape")
    return torch.empty(n, dtype=torch.uint8, device=device)


def svf_select_per_draft(shape, q, reps, seq_lens, masks, ws=None, scores=None):
    _check(lib().svf_select_per_draft(ctypes.byref(shape), _ptr(q), _ptr(reps), _ptr(seq_lens), _ptr(masks),
                                      _ptr(scores), _ptr(ws), ws.numel() if ws is not None else 0, _stream()),
           "svf_select_per_draft")


def svf_masks_from_selection(shape, sel_idx, sel_cnt, masks):
    _check(lib().svf_masks_from_selection(ctypes.byref(shape), _ptr(sel_idx), _ptr(sel_cnt), _ptr(masks), _stream()),
           "svf_masks_from_selection")


def svf_overlap_by_distance(shape, masks, pos, n_dist, inter):
    _check(lib().svf_overlap_by_distance(ctypes.byref(shape), _ptr(masks), _ptr(pos), int(n_dist), _ptr(inter),
                                         _stream()), "svf_overlap_by_distance")


def svf_jaccard_adjacent(shape, masks_by_layer, n_layers, inter_union):
    _check(lib().svf_jaccard_adjacent(ctypes.byref(shape), _ptr(masks_by_layer), int(n_layers), _ptr(inter_union),
                                      _stream()), "svf_jaccard_adjacent")


def svf_topk_anchors(J, K):
    """Eq. 8 on the host: J is a sequence of per-layer similarities; returns the K anchor layers."""
    n = len(J)
    arr = (ctypes.c_double * n)(*[float(v) for v in J])
    out = (ctypes.c_int32 * max(int(K), 1))()
    _check(lib().svf_topk_anchors(arr, n, int(K), out), "svf_topk_anchors")
    return [int(out[i]) for i in range(int(K))]


# ---- retrieval variants (argument marshalling only) -------------------------------------------

def svf_block_summaries(shape, retrieval, K, block_table, seq_lens, summaries, first_block=0, n_blocks=-1):
    _check(lib().svf_block_summaries(ctypes.byref(shape), ctypes.byref(retrieval), _ptr(K), _ptr(block_table),
                                     _ptr(seq_lens), first_block, n_blocks, _ptr(summaries), _stream()),
           "svf_block_summaries")


def svf_retrieve(shape, retrieval, q, summaries, seq_lens, sel_idx, sel_cnt, ws, scores=None):
    _check(lib().svf_retrieve(ctypes.byref(shape), ctypes.byref(retrieval), _ptr(q), _ptr(summaries),
                              _ptr(seq_lens), _ptr(sel_idx), _ptr(sel_cnt), _ptr(scores), _ptr(ws), ws.numel(),
                              _stream()), "svf_retrieve")


# ---- sparse feed-forward verification (argument marshalling only) ------------------------------

def make_ffn_shape(*, M, d_model, d_ff, act="silu", tau=0.0, walk=SVF_FFN_WALK_AUTO) -> SvfFfnShape:
    code = {"silu": SVF_ACT_SILU, "gelu": SVF_ACT_GELU}.get(act, act)
    return SvfFfnShape(M, d_model, d_ff, code, tau, walk)


def svf_ffn_workspace_bytes(shape: SvfFfnShape) -> int:
    return int(lib().svf_ffn_workspace_bytes(ctypes.byref(shape)))


def new_ffn_workspace(shape: SvfFfnShape, device="cuda") -> torch.Tensor:
    n = svf_ffn_workspace_bytes(shape)
    if n == 0:
        raise SvfError(-2, "svf_ffn_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def svf_sparse_ffn(shape, x, w_gate, w_up, w_down_t, y, ws, b_gate=None, b_up=None, b_down=None, active=None):
    _check(lib().svf_sparse_ffn(ctypes.byref(shape), _ptr(x), _ptr(w_gate), _ptr(w_up), _ptr(w_down_t), _ptr(b_gate),
                                _ptr(b_up), _ptr(b_down), _ptr(y), _ptr(active), _ptr(ws), ws.numel(), _stream()),
           "svf_sparse_ffn")


# ---- expert skipping, acceptance / resampling (argument marshalling only) -----------------------

def svf_moe_skip(w, m, beta, n_skip, keep_mask):
    T, k = w.shape
    _check(lib().svf_moe_skip(_ptr(w), T, k, int(m), _ptr(beta), _ptr(n_skip), _ptr(keep_mask), _stream()), "svf_moe_skip")


def svf_moe_calibrate(w_cal, beta, ws=None):
    T, k = w_cal.shape
    if ws is None:
        ws = torch.empty(int(lib().svf_moe_calibrate_workspace_bytes(T, k)), dtype=torch.uint8, device=w_cal.device)
    _check(lib().svf_moe_calibrate(_ptr(w_cal), T, k, _ptr(beta), _ptr(ws), ws.numel(), _stream()), "svf_moe_calibrate")


def svf_accept_resample(p_target, p_draft, draft_tokens, u_accept, u_resample, n_accepted, resampled):
    B, gamma, V = p_target.shape
    _check(lib().svf_accept_resample(_ptr(p_target), _ptr(p_draft), _ptr(draft_tokens), _ptr(u_accept), _ptr(u_resample),
                                     B, gamma, V, _ptr(n_accepted), _ptr(resampled), _stream()), "svf_accept_resample")

