"""Thin ctypes binding of libasyncspade.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI (include/asyncspade.h);
torch is used for device memory and streams.  There is no CPU fallback: if the library is
missing or a call fails this module raises.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libasyncspade.so")
_lib = None

AS_AGG_MAX, AS_AGG_SUM, AS_AGG_SOFTMAX_SUM = 0, 1, 2
AS_PRED_PER_WINDOW, AS_PRED_SINGLE_SOLVE = 0, 1
EXPORTS = ["as_workspace_bytes", "as_workspace_bytes_attn", "as_create", "as_destroy", "as_status_str", "as_predict_query", "as_score_keys",
           "as_topk_select", "as_score_topk", "as_sparse_decode_attn", "as_select_step", "as_select_step_static",
           "as_workspace_bytes_pack",
           "as_select_step_pack", "as_kv_append", "as_window_push", "as_gather_kv", "as_overlap_ratio",
           "as_dense_decode_attn"]
# development / measurement entry points (include/asyncspade_debug.h)
DEBUG_EXPORTS = ["as_debug_select_plan", "as_debug_rows_plan", "as_debug_workspace_gaps", "as_debug_set_select_mode",
                 "as_debug_set_attn_splits", "as_debug_set_timeline", "as_debug_set_predict_mode", "as_debug_set_merge_mode", "as_debug_attn_workspace_bytes", "as_debug_stream_read_paged",
                 "as_debug_stream_read_flat", "as_debug_stream_read_flat_sink_words"]
AS_MAX_PACK = 16
AS_STATIC_SCRATCH_BYTES = 48 << 20


class AsParams(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("page_size", C.c_int32), ("window", C.c_int32), ("budget", C.c_int32),
                ("max_pages_per_seq", C.c_int32), ("ridge_eps", C.c_float), ("softmax_beta", C.c_float),
                ("sm_scale", C.c_float), ("agg", C.c_int32), ("predictor", C.c_int32)]


class AsKvView(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("block_table", C.c_void_p),
                ("ctx_lens", C.c_void_p), ("num_pages", C.c_int64)]


class AsLayerIo(C.Structure):
    _fields_ = [("kv", AsKvView), ("q_win", C.c_void_p), ("q_cur", C.c_void_p), ("sel_idx", C.c_void_p),
                ("sel_cnt", C.c_void_p)]


class AsError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().as_status_str(code).decode() if _lib is not None else str(code)
        super().__init__(f"{where}: {msg} (status {code})")


def lib():
    """Loads the built library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2510_07486_amd.build` first")
        L = C.CDLL(LIB_PATH)
        L.as_workspace_bytes.restype = C.c_size_t
        L.as_workspace_bytes.argtypes = [C.POINTER(AsParams)]
        L.as_workspace_bytes_attn.restype = C.c_size_t
        L.as_workspace_bytes_attn.argtypes = [C.POINTER(AsParams)]
        L.as_create.restype = C.c_int
        L.as_create.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_size_t]
        L.as_destroy.restype = C.c_int
        L.as_destroy.argtypes = [C.c_void_p]
        L.as_status_str.restype = C.c_char_p
        L.as_status_str.argtypes = [C.c_int]
        vp = C.c_void_p
        PP, KP = C.POINTER(AsParams), C.POINTER(AsKvView)
        L.as_predict_query.restype = C.c_int
        L.as_predict_query.argtypes = [vp, PP, vp, vp, vp, vp]
        L.as_score_keys.restype = C.c_int
        L.as_score_keys.argtypes = [vp, PP, KP, vp, vp, C.c_int64, vp]
        L.as_topk_select.restype = C.c_int
        L.as_topk_select.argtypes = [vp, PP, vp, C.c_int64, vp, vp, vp, vp]
        L.as_sparse_decode_attn.restype = C.c_int
        L.as_sparse_decode_attn.argtypes = [vp, PP, KP, vp, vp, vp, vp, vp, vp, vp]
        L.as_dense_decode_attn.restype = C.c_int
        L.as_dense_decode_attn.argtypes = [vp, PP, KP, vp, vp, vp, vp]
        L.as_score_topk.restype = C.c_int
        L.as_score_topk.argtypes = [vp, PP, KP, vp, vp, vp, vp]
        L.as_select_step.restype = C.c_int
        L.as_select_step.argtypes = [vp, PP, KP, vp, vp, vp, vp, vp]
        L.as_select_step_static.restype = C.c_int
        L.as_select_step_static.argtypes = [PP, KP, vp, vp, vp, vp, vp]
        L.as_workspace_bytes_pack.restype = C.c_size_t
        L.as_workspace_bytes_pack.argtypes = [PP, C.c_int32]
        L.as_select_step_pack.restype = C.c_int
        L.as_select_step_pack.argtypes = [vp, PP, C.POINTER(AsLayerIo), C.c_int32, vp]
        L.as_kv_append.restype = C.c_int
        L.as_kv_append.argtypes = [vp, PP, vp, vp, vp, vp, C.c_int64, vp, vp, vp]
        L.as_window_push.restype = C.c_int
        L.as_window_push.argtypes = [vp, PP, vp, vp, vp, vp]
        L.as_gather_kv.restype = C.c_int
        L.as_gather_kv.argtypes = [vp, PP, KP, vp, vp, vp, vp, vp, vp, vp]
        L.as_overlap_ratio.restype = C.c_int
        L.as_overlap_ratio.argtypes = [vp, PP, vp, vp, vp, vp, vp, vp, vp]
        L.as_debug_select_plan.restype = C.c_int
        L.as_debug_select_plan.argtypes = [PP, C.c_int32, C.POINTER(C.c_int32)]
        L.as_debug_rows_plan.restype = C.c_int
        L.as_debug_rows_plan.argtypes = [PP, C.c_int32, C.POINTER(C.c_int32)]
        L.as_debug_workspace_gaps.restype = C.c_int
        L.as_debug_workspace_gaps.argtypes = [vp, PP, C.c_int32, C.POINTER(C.c_int32)]
        L.as_debug_set_select_mode.restype = C.c_int
        L.as_debug_set_select_mode.argtypes = [vp, C.c_int32]
        L.as_debug_set_attn_splits.restype = C.c_int
        L.as_debug_set_attn_splits.argtypes = [vp, C.c_int32]
        L.as_debug_set_merge_mode.restype = C.c_int
        L.as_debug_set_merge_mode.argtypes = [vp, C.c_int32]
        L.as_debug_set_predict_mode.restype = C.c_int
        L.as_debug_set_predict_mode.argtypes = [vp, C.c_int32]
        L.as_debug_set_timeline.restype = C.c_int
        L.as_debug_set_timeline.argtypes = [vp, vp, C.c_int32]
        L.as_debug_attn_workspace_bytes.restype = C.c_size_t
        L.as_debug_attn_workspace_bytes.argtypes = [PP, C.c_int32]
        L.as_debug_stream_read_paged.restype = C.c_int
        L.as_debug_stream_read_paged.argtypes = [vp, PP, KP, vp, C.c_int64, C.c_int32, vp]
        L.as_debug_stream_read_flat.restype = C.c_int
        L.as_debug_stream_read_flat.argtypes = [vp, vp, C.c_size_t, vp, vp]
        L.as_debug_stream_read_flat_sink_words.restype = C.c_size_t
        L.as_debug_stream_read_flat_sink_words.argtypes = []
        _lib = L
    return _lib


def make_params(batch, n_q_heads, n_kv_heads, window, budget, max_pages_per_seq, ridge_eps=1e-2, softmax_beta=1.0,
                sm_scale=None, agg=AS_AGG_MAX, head_dim=128, page_size=16, predictor=AS_PRED_PER_WINDOW) -> AsParams:
    if sm_scale is None:
        sm_scale = 1.0 / math.sqrt(head_dim)
    return AsParams(batch, n_q_heads, n_kv_heads, head_dim, page_size, window, budget, max_pages_per_seq,
                    ridge_eps, softmax_beta, sm_scale, agg, predictor)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors crossing the C ABI must be contiguous"
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def kv_view(k_pool, v_pool, block_table, ctx_lens) -> AsKvView:
    assert k_pool.dtype == torch.bfloat16 and block_table.dtype == torch.int32 and ctx_lens.dtype == torch.int32
    kv = AsKvView(_ptr(k_pool), _ptr(v_pool), _ptr(block_table), _ptr(ctx_lens), k_pool.shape[0])
    # the view holds raw device pointers: keep the tensors alive as long as the view is
    kv._keep_alive = (k_pool, v_pool, block_table, ctx_lens)
    return kv


def _check(code: int, where: str):
    if code != 0:
        raise AsError(code, where)


def as_workspace_bytes(p: AsParams) -> int:
    return int(lib().as_workspace_bytes(C.byref(p)))


def rows_plan(p: AsParams, n_layers: int = 1):
    """(serves the shape, preferred to the fused kernels, pages per workgroup, workgroups per row) of the one-launch
    selection over score rows."""
    out = (C.c_int32 * 4)()
    _check(lib().as_debug_rows_plan(C.byref(p), n_layers, out), "as_debug_rows_plan")
    return tuple(out)


def select_plan(p: AsParams, n_layers: int = 1):
    """(share length, shares per row, candidates per share) the fused selection would use."""
    out = (C.c_int32 * 3)()
    _check(lib().as_debug_select_plan(C.byref(p), n_layers, out), "as_debug_select_plan")
    return tuple(out)


def as_workspace_bytes_pack(p: AsParams, n_layers: int) -> int:
    return int(lib().as_workspace_bytes_pack(C.byref(p), n_layers))


def as_workspace_bytes_attn(p: AsParams) -> int:
    """Leading part of the workspace that the attention calls need (a ctx that only attends)."""
    return int(lib().as_workspace_bytes_attn(C.byref(p)))


class Context:
    """Owns one as_ctx (device workspace).  One per concurrently used stream."""

    def __init__(self, p: AsParams, device: int = 0, workspace_bytes: Optional[int] = None, pack: int = 1):
        self.handle = C.c_void_p()
        nbytes = workspace_bytes
        if nbytes is None:      # large enough for the single-layer calls and for packs of `pack` layers
            nbytes = max(as_workspace_bytes(p), as_workspace_bytes_pack(p, pack) if pack > 1 else 0)
        _check(lib().as_create(C.byref(self.handle), device, nbytes), "as_create")
        self.workspace_bytes = nbytes

    def close(self):
        if self.handle:
            _check(lib().as_destroy(self.handle), "as_destroy")
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def damaged_workspace_gap(self, p: AsParams, n_layers: int = 1) -> int:
        """-1 if no kernel has written outside its region of the workspace (layout of (p, n_layers)), else the index
        of the first damaged gap.  Synchronises; only meaningful if the context has used this one layout."""
        bad = C.c_int32(0)
        _check(lib().as_debug_workspace_gaps(self.handle, C.byref(p), n_layers, C.byref(bad)), "as_debug_workspace_gaps")
        return bad.value

    def set_select_mode(self, m: int):
        """0 = route chosen from the share plan (default), 1 = the two stand-alone kernels through HBM scores, 2 = the fused
        kernels, 3 = through HBM scores in one launch where the shape allows."""
        _check(lib().as_debug_set_select_mode(self.handle, m), "as_debug_set_select_mode")

    def set_attn_splits(self, n: int):
        """Forces the attention split count of this ctx (0 = the library's rule); the workspace must have been sized
        with attn_workspace_bytes_forced for the largest count used."""
        _check(lib().as_debug_set_attn_splits(self.handle, n), "as_debug_set_attn_splits")


    def set_merge_mode(self, m: int):
        """0 = multi-share rows are merged inside the selection kernel where possible (default), 1 = by a second launch."""
        _check(lib().as_debug_set_merge_mode(self.handle, m), "as_debug_set_merge_mode")

    def set_predict_mode(self, m: int):
        """0 = the predictor is a launch of its own (default), 1 = in the prologue of the fused selection kernel where possible."""
        _check(lib().as_debug_set_predict_mode(self.handle, m), "as_debug_set_predict_mode")

    def set_timeline(self, buf: Optional[torch.Tensor]):
        """buf: int64 device tensor [capacity, 2] that receives (entry, exit) wall-clock marks (100 MHz) of every
        workgroup of the fused selection and attention kernels launched through this ctx; None switches it off."""
        self._timeline = buf
        _check(lib().as_debug_set_timeline(self.handle, _ptr(buf), 0 if buf is None else buf.shape[0]),
               "as_debug_set_timeline")


def attn_workspace_bytes_forced(p: AsParams, splits: int) -> int:
    return int(lib().as_debug_attn_workspace_bytes(C.byref(p), splits))


def stream_read_paged(ctx: Context, p: AsParams, kv: AsKvView, sink, words_per_token: bool, stream=None):
    """Calibration kernel: the scoring kernels' paged walk over K with no arithmetic; sink fp32 [B][Hkv][stride]."""
    _check(lib().as_debug_stream_read_paged(ctx.handle, C.byref(p), C.byref(kv), _ptr(sink), sink.shape[2],
                                            1 if words_per_token else 0, _stream(stream)), "as_debug_stream_read_paged")


def stream_read_flat(ctx: Context, buf, sink=None, stream=None):
    """Calibration kernel: plain front-to-back 128-bit read of the tensor `buf` (no page table)."""
    if sink is None:
        sink = torch.empty((lib().as_debug_stream_read_flat_sink_words(),), dtype=torch.int32, device=buf.device)
    nbytes = buf.numel() * buf.element_size()
    _check(lib().as_debug_stream_read_flat(ctx.handle, _ptr(buf), nbytes - nbytes % 16, _ptr(sink), _stream(stream)),
           "as_debug_stream_read_flat")
    return sink


def as_predict_query(ctx: Context, p: AsParams, q_win, q_cur, q_hat=None, stream=None):
    if q_hat is None:
        q_hat = torch.empty((p.batch, p.n_q_heads, p.head_dim), dtype=torch.float32, device=q_win.device)
    _check(lib().as_predict_query(ctx.handle, C.byref(p), _ptr(q_win), _ptr(q_cur), _ptr(q_hat), _stream(stream)),
           "as_predict_query")
    return q_hat


def as_score_keys(ctx: Context, p: AsParams, kv: AsKvView, q_hat, scores=None, stream=None, fill=None):
    if scores is None:
        stride = p.max_pages_per_seq * p.page_size
        scores = torch.empty((p.batch, p.n_kv_heads, stride), dtype=torch.float32, device=q_hat.device)
        if fill is not None:
            scores.fill_(fill)
    _check(lib().as_score_keys(ctx.handle, C.byref(p), C.byref(kv), _ptr(q_hat), _ptr(scores), scores.shape[2],
                               _stream(stream)), "as_score_keys")
    return scores


def as_topk_select(ctx: Context, p: AsParams, scores, ctx_lens, sel_idx=None, sel_cnt=None, stream=None):
    if sel_idx is None:
        sel_idx = torch.empty((p.batch, p.n_kv_heads, p.budget), dtype=torch.int32, device=scores.device)
    if sel_cnt is None:
        sel_cnt = torch.empty((p.batch, p.n_kv_heads), dtype=torch.int32, device=scores.device)
    _check(lib().as_topk_select(ctx.handle, C.byref(p), _ptr(scores), scores.shape[2], _ptr(ctx_lens), _ptr(sel_idx),
                                _ptr(sel_cnt), _stream(stream)), "as_topk_select")
    return sel_idx, sel_cnt


def as_sparse_decode_attn(ctx: Context, p: AsParams, kv: AsKvView, q, sel_idx, sel_cnt, sel_ctx_lens=None, out=None,
                          lse=None, stream=None, want_lse=True):
    if out is None:
        out = torch.empty((p.batch, p.n_q_heads, p.head_dim), dtype=torch.bfloat16, device=q.device)
    if lse is None and want_lse:
        lse = torch.empty((p.batch, p.n_q_heads), dtype=torch.float32, device=q.device)
    _check(lib().as_sparse_decode_attn(ctx.handle, C.byref(p), C.byref(kv), _ptr(q), _ptr(sel_idx), _ptr(sel_cnt),
                                       _ptr(sel_ctx_lens), _ptr(out), _ptr(lse), _stream(stream)),
           "as_sparse_decode_attn")
    return out, lse


def as_dense_decode_attn(ctx: Context, p: AsParams, kv: AsKvView, q, out=None, lse=None, stream=None, want_lse=True):
    if out is None:
        out = torch.empty((p.batch, p.n_q_heads, p.head_dim), dtype=torch.bfloat16, device=q.device)
    if lse is None and want_lse:
        lse = torch.empty((p.batch, p.n_q_heads), dtype=torch.float32, device=q.device)
    _check(lib().as_dense_decode_attn(ctx.handle, C.byref(p), C.byref(kv), _ptr(q), _ptr(out), _ptr(lse),
                                      _stream(stream)), "as_dense_decode_attn")
    return out, lse


def as_score_topk(ctx: Context, p: AsParams, kv: AsKvView, q_hat, sel_idx=None, sel_cnt=None, stream=None):
    if sel_idx is None:
        sel_idx = torch.empty((p.batch, p.n_kv_heads, p.budget), dtype=torch.int32, device=q_hat.device)
    if sel_cnt is None:
        sel_cnt = torch.empty((p.batch, p.n_kv_heads), dtype=torch.int32, device=q_hat.device)
    _check(lib().as_score_topk(ctx.handle, C.byref(p), C.byref(kv), _ptr(q_hat), _ptr(sel_idx), _ptr(sel_cnt),
                               _stream(stream)), "as_score_topk")
    return sel_idx, sel_cnt


def as_select_step(ctx: Context, p: AsParams, kv: AsKvView, q_win, q_cur, sel_idx=None, sel_cnt=None, stream=None):
    if sel_idx is None:
        sel_idx = torch.empty((p.batch, p.n_kv_heads, p.budget), dtype=torch.int32, device=q_win.device)
    if sel_cnt is None:
        sel_cnt = torch.empty((p.batch, p.n_kv_heads), dtype=torch.int32, device=q_win.device)
    _check(lib().as_select_step(ctx.handle, C.byref(p), C.byref(kv), _ptr(q_win), _ptr(q_cur), _ptr(sel_idx),
                                _ptr(sel_cnt), _stream(stream)), "as_select_step")
    return sel_idx, sel_cnt


def as_select_step_static(p: AsParams, kv: AsKvView, q_win, q_cur, sel_idx, sel_cnt, stream=None):
    """as_select_step without a ctx and without any allocation: scratch lives in the library's static device array.
    Outputs are the caller's (no tensor is created here)."""
    _check(lib().as_select_step_static(C.byref(p), C.byref(kv), _ptr(q_win), _ptr(q_cur), _ptr(sel_idx), _ptr(sel_cnt),
                                       _stream(stream)), "as_select_step_static")
    return sel_idx, sel_cnt


def layer_io(kv: AsKvView, q_win, q_cur, sel_idx, sel_cnt) -> AsLayerIo:
    io = AsLayerIo(kv, _ptr(q_win), _ptr(q_cur), _ptr(sel_idx), _ptr(sel_cnt))
    io._keep_alive = (kv, q_win, q_cur, sel_idx, sel_cnt)
    return io


def as_select_step_pack(ctx: Context, p: AsParams, layers, stream=None):
    """layers: sequence of AsLayerIo (see layer_io) or a prepared ctypes array of them."""
    if not isinstance(layers, C.Array):
        layers = (AsLayerIo * len(layers))(*layers)
    _check(lib().as_select_step_pack(ctx.handle, C.byref(p), layers, len(layers), _stream(stream)),
           "as_select_step_pack")


def as_kv_append(ctx: Context, p: AsParams, k_pool, v_pool, block_table, ctx_lens, k_new, v_new, stream=None):
    """In place on k_pool, v_pool and ctx_lens."""
    _check(lib().as_kv_append(ctx.handle, C.byref(p), _ptr(k_pool), _ptr(v_pool), _ptr(block_table), _ptr(ctx_lens),
                              k_pool.shape[0], _ptr(k_new), _ptr(v_new), _stream(stream)), "as_kv_append")


def as_window_push(ctx: Context, p: AsParams, q_win, q_cur, q_new, stream=None):
    """In place on q_win and q_cur."""
    _check(lib().as_window_push(ctx.handle, C.byref(p), _ptr(q_win), _ptr(q_cur), _ptr(q_new), _stream(stream)),
           "as_window_push")


def compact_pages(p: AsParams) -> int:
    return (p.budget + p.page_size - 1) // p.page_size


def as_gather_kv(ctx: Context, p: AsParams, kv: AsKvView, sel_idx, sel_cnt, k_out=None, v_out=None, out_table=None,
                 out_lens=None, stream=None):
    Cp = compact_pages(p)
    dev = sel_idx.device
    shape = (p.batch * Cp, p.n_kv_heads, p.page_size, p.head_dim)
    if k_out is None:
        k_out = torch.empty(shape, dtype=torch.bfloat16, device=dev)
    if v_out is None:
        v_out = torch.empty(shape, dtype=torch.bfloat16, device=dev)
    if out_table is None:
        out_table = torch.empty((p.batch, Cp), dtype=torch.int32, device=dev)
    if out_lens is None:
        out_lens = torch.empty((p.batch,), dtype=torch.int32, device=dev)
    _check(lib().as_gather_kv(ctx.handle, C.byref(p), C.byref(kv), _ptr(sel_idx), _ptr(sel_cnt), _ptr(k_out),
                              _ptr(v_out), _ptr(out_table), _ptr(out_lens), _stream(stream)), "as_gather_kv")
    return k_out, v_out, out_table, out_lens


def as_overlap_ratio(ctx: Context, p: AsParams, idx_a, cnt_a, idx_b, cnt_b, inter=None, ratio=None, stream=None):
    if inter is None:
        inter = torch.empty((p.batch, p.n_kv_heads), dtype=torch.int32, device=idx_a.device)
    if ratio is None:
        ratio = torch.empty((p.batch, p.n_kv_heads), dtype=torch.float32, device=idx_a.device)
    _check(lib().as_overlap_ratio(ctx.handle, C.byref(p), _ptr(idx_a), _ptr(cnt_a), _ptr(idx_b), _ptr(cnt_b),
                                  _ptr(inter), _ptr(ratio), _stream(stream)), "as_overlap_ratio")
    return inter, ratio
