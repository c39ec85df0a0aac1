"""ctypes binding of the C oracle: argument marshalling only (host tensors)."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "asyncspade_oracle.c")
_LIB = os.path.join(_HERE, "libasyncspade_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64 scalar loops, OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.aso_predict_query.restype = C.c_int
        _lib.aso_predict_query_single_solve.restype = C.c_int
        _lib.aso_score_keys.restype = C.c_int
        _lib.aso_score_keys_softmax_sum.restype = C.c_int
        _lib.aso_topk_select.restype = C.c_int
        _lib.aso_sparse_decode_attn.restype = C.c_int
        _lib.aso_ridge_weights.restype = C.c_int
        _lib.aso_set_threads.restype = C.c_int
        for fn in ("aso_overlap_ratio", "aso_kv_append", "aso_window_push", "aso_gather_kv"):
            getattr(_lib, fn).restype = C.c_int
        _lib.aso_f64_to_bf16.restype = C.c_uint16
        _lib.aso_f64_to_bf16.argtypes = [C.c_double]
    return _lib


def _p(t: torch.Tensor):
    assert t.device.type == "cpu" and t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def set_threads(n: int) -> int:
    return _load().aso_set_threads(C.c_int(n))


def f64_to_bf16(x: float) -> int:
    return int(_load().aso_f64_to_bf16(float(x)))


def ridge_weights(R: np.ndarray, T: np.ndarray, eps: float) -> np.ndarray:
    """R [k, D] newest predecessor first, T [D]; returns omega [k] (fp64)."""
    R = np.ascontiguousarray(R, dtype=np.float64)
    T = np.ascontiguousarray(T, dtype=np.float64)
    k, D = R.shape
    om = np.zeros(k, dtype=np.float64)
    rc = _load().aso_ridge_weights(C.c_int(k), C.c_int(D), R.ctypes.data_as(C.c_void_p),
                                   T.ctypes.data_as(C.c_void_p), C.c_double(eps),
                                   om.ctypes.data_as(C.c_void_p))
    if rc != 0:
        raise RuntimeError(f"aso_ridge_weights rc={rc}")
    return om


def predict_query(q_win: torch.Tensor, q_cur: torch.Tensor, eps: float, beta: float = 1.0,
                  return_weights: bool = False, single_solve: bool = False):
    B, Hq, W, D = q_win.shape
    q_win = q_win.contiguous(); q_cur = q_cur.contiguous()
    assert q_win.dtype == torch.bfloat16 and q_cur.dtype == torch.bfloat16
    q_hat = torch.empty((B, Hq, D), dtype=torch.float32)
    wts = torch.zeros((B, Hq, W, W), dtype=torch.float64) if return_weights else None
    fn = _load().aso_predict_query_single_solve if single_solve else _load().aso_predict_query
    rc = fn(C.c_int(B), C.c_int(Hq), C.c_int(W), C.c_int(D), _p(q_win), _p(q_cur),
                                   C.c_double(eps), C.c_double(beta), _p(q_hat),
                                   _p(wts) if wts is not None else None)
    if rc != 0:
        raise RuntimeError(f"aso_predict_query rc={rc}")
    return (q_hat, wts) if return_weights else q_hat


def score_keys(k_pool, block_table, ctx_lens, q_hat, n_kv_heads: int, agg: int = 0, stride: int | None = None,
               fill: float = float("nan"), sm_scale: float | None = None):
    """agg: 0 max, 1 sum of the group's raw logits; 2 sum of the group's softmax probabilities (needs sm_scale)."""
    num_pages, Hkv, P, D = k_pool.shape
    assert Hkv == n_kv_heads
    B, Hq, _ = q_hat.shape
    max_pages = block_table.shape[1]
    if stride is None:
        stride = max_pages * P
    scores = torch.full((B, Hkv, stride), fill, dtype=torch.float32)
    if agg == 2:
        assert sm_scale is not None
        rc = _load().aso_score_keys_softmax_sum(
            C.c_int(B), C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int(P), _p(k_pool.contiguous()),
            _p(block_table.contiguous()), C.c_int(max_pages), _p(ctx_lens.contiguous()), _p(q_hat.contiguous()),
            C.c_double(sm_scale), _p(scores), C.c_int64(stride))
        if rc != 0:
            raise RuntimeError(f"aso_score_keys_softmax_sum rc={rc}")
        return scores
    rc = _load().aso_score_keys(C.c_int(B), C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int(P), _p(k_pool.contiguous()),
                                _p(block_table.contiguous()), C.c_int(max_pages), _p(ctx_lens.contiguous()),
                                _p(q_hat.contiguous()), C.c_int(agg), _p(scores), C.c_int64(stride))
    if rc != 0:
        raise RuntimeError(f"aso_score_keys rc={rc}")
    return scores


def topk_select(scores, ctx_lens, budget: int):
    B, Hkv, stride = scores.shape
    sel_idx = torch.empty((B, Hkv, budget), dtype=torch.int32)
    sel_cnt = torch.empty((B, Hkv), dtype=torch.int32)
    rc = _load().aso_topk_select(C.c_int(B), C.c_int(Hkv), C.c_int(budget), _p(scores.contiguous()),
                                 C.c_int64(stride), _p(ctx_lens.contiguous()), _p(sel_idx), _p(sel_cnt))
    if rc != 0:
        raise RuntimeError(f"aso_topk_select rc={rc}")
    return sel_idx, sel_cnt


def sparse_decode_attn(k_pool, v_pool, block_table, ctx_lens, q, sel_idx, sel_cnt, sm_scale: float,
                       sel_ctx_lens=None):
    num_pages, Hkv, P, D = k_pool.shape
    B, Hq, _ = q.shape
    Cb = sel_idx.shape[2]
    out = torch.empty((B, Hq, D), dtype=torch.bfloat16)
    lse = torch.empty((B, Hq), dtype=torch.float32)
    rc = _load().aso_sparse_decode_attn(
        C.c_int(B), C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int(P), C.c_int(Cb), _p(k_pool.contiguous()),
        _p(v_pool.contiguous()), _p(block_table.contiguous()), C.c_int(block_table.shape[1]),
        _p(ctx_lens.contiguous()), _p(q.contiguous()), _p(sel_idx.contiguous()), _p(sel_cnt.contiguous()),
        _p(sel_ctx_lens.contiguous()) if sel_ctx_lens is not None else None, C.c_double(sm_scale), _p(out), _p(lse))
    if rc != 0:
        raise RuntimeError(f"aso_sparse_decode_attn rc={rc}")
    return out, lse


def select_step(k_pool, block_table, ctx_lens, q_win, q_cur, budget: int, eps: float, beta: float = 1.0,
                agg: int = 0, single_solve: bool = False, sm_scale: float | None = None):
    """predict -> score -> top-k, the three oracle stages chained."""
    q_hat = predict_query(q_win, q_cur, eps, beta, single_solve=single_solve)
    scores = score_keys(k_pool, block_table, ctx_lens, q_hat, k_pool.shape[1], agg, sm_scale=sm_scale)
    sel_idx, sel_cnt = topk_select(scores, ctx_lens, budget)
    return q_hat, scores, sel_idx, sel_cnt


def overlap_ratio(idx_a, cnt_a, idx_b, cnt_b):
    """Eq. 1 per (b, kv head): returns (|S_a & S_b| int32 [B,Hkv], ratio fp32 [B,Hkv])."""
    B, Hkv, Cb = idx_a.shape
    inter = torch.empty((B, Hkv), dtype=torch.int32)
    ratio = torch.empty((B, Hkv), dtype=torch.float32)
    rc = _load().aso_overlap_ratio(C.c_int(B), C.c_int(Hkv), C.c_int(Cb), _p(idx_a.contiguous()),
                                   _p(cnt_a.contiguous()), _p(idx_b.contiguous()), _p(cnt_b.contiguous()),
                                   _p(inter), _p(ratio))
    if rc != 0:
        raise RuntimeError(f"aso_overlap_ratio rc={rc}")
    return inter, ratio


def kv_append(k_pool, v_pool, block_table, ctx_lens, k_new, v_new):
    """In place on k_pool, v_pool and ctx_lens (host tensors)."""
    num_pages, Hkv, P, D = k_pool.shape
    B = ctx_lens.shape[0]
    rc = _load().aso_kv_append(C.c_int(B), C.c_int(Hkv), C.c_int(D), C.c_int(P), _p(k_pool), _p(v_pool),
                               _p(block_table.contiguous()), C.c_int(block_table.shape[1]), _p(ctx_lens),
                               _p(k_new.contiguous()), _p(v_new.contiguous()))
    if rc != 0:
        raise RuntimeError(f"aso_kv_append rc={rc}")


def window_push(q_win, q_cur, q_new):
    """In place on q_win and q_cur (host tensors)."""
    B, Hq, W, D = q_win.shape
    rc = _load().aso_window_push(C.c_int(B), C.c_int(Hq), C.c_int(W), C.c_int(D), _p(q_win), _p(q_cur),
                                 _p(q_new.contiguous()))
    if rc != 0:
        raise RuntimeError(f"aso_window_push rc={rc}")


def gather_kv(k_pool, v_pool, block_table, sel_idx, sel_cnt, fill: float = 0.0):
    """Returns (k_out, v_out [B*Cp,Hkv,P,D] bf16 pre-filled with `fill`, out_table [B,Cp], out_lens [B])."""
    num_pages, Hkv, P, D = k_pool.shape
    B, _, Cb = sel_idx.shape
    Cp = (Cb + P - 1) // P
    k_out = torch.full((B * Cp, Hkv, P, D), fill, dtype=torch.bfloat16)
    v_out = torch.full((B * Cp, Hkv, P, D), fill, dtype=torch.bfloat16)
    table = torch.empty((B, Cp), dtype=torch.int32)
    lens = torch.empty((B,), dtype=torch.int32)
    rc = _load().aso_gather_kv(C.c_int(B), C.c_int(Hkv), C.c_int(D), C.c_int(P), C.c_int(Cb), _p(k_pool.contiguous()),
                               _p(v_pool.contiguous()), _p(block_table.contiguous()), C.c_int(block_table.shape[1]),
                               _p(sel_idx.contiguous()), _p(sel_cnt.contiguous()), _p(k_out), _p(v_out), _p(table),
                               _p(lens))
    if rc != 0:
        raise RuntimeError(f"aso_gather_kv rc={rc}")
    return k_out, v_out, table, lens
