"""The oracle against hand-worked examples stored under tests/golden/ (derived by hand from the paper's equations,
each with its citation and derivation; the paper itself prints no numeric example).  CPU only."""
import json
import math
import os

import numpy as np
import torch

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
GOLD = json.load(open(os.path.join(HERE, "golden", "hand_worked_examples.json")))


def _bf(x):
    return torch.tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)


def _pad(vec, D=128):
    out = np.zeros(D, dtype=np.float32)
    out[: len(vec)] = vec
    return out


def test_predictor_hand_example():
    g = GOLD["predictor_w2_orthogonal"]
    qw = _bf([[_pad(r) for r in g["window_oldest_first"]]])[None]       # [1, 1, W, D]
    qc = _bf([_pad(g["q_cur"])])[None]
    qh, w = oracle.predict_query(qw, qc, g["eps"], g["beta"], return_weights=True)
    assert qh[0, 0, :2].tolist() == g["q_hat"] and (qh[0, 0, 2:] == 0).all()
    assert w[0, 0, 0, :1].tolist() == g["weights_k1"] and w[0, 0, 1, :2].tolist() == g["weights_k2"]
    qs = oracle.predict_query(qw, qc, g["eps"], g["beta"], single_solve=True)
    assert qs[0, 0, :2].tolist() == GOLD["predictor_w2_orthogonal_single_solve"]["q_hat"]


def test_select_and_attend_hand_example():
    g = GOLD["select_and_attend_four_tokens"]
    k = torch.zeros((1, 1, 16, 128), dtype=torch.bfloat16)
    v = torch.zeros((1, 1, 16, 128), dtype=torch.bfloat16)
    for n, (kk, vv) in enumerate(zip(g["keys_dim0_dim1"], g["values_dim0"])):
        k[0, 0, n, :2] = _bf(kk)
        v[0, 0, n, 0] = vv
    bt = torch.zeros((1, 1), dtype=torch.int32)
    lens = torch.tensor([4], dtype=torch.int32)
    q_hat = torch.tensor(_pad(g["q_hat_dim0_dim1"]))[None, None]
    sc = oracle.score_keys(k, bt, lens, q_hat, 1)
    assert sc[0, 0, :4].tolist() == g["scores"]
    idx2, cnt2 = oracle.topk_select(sc, lens, 2)
    assert idx2[0, 0].tolist() == g["selected_budget2"] and cnt2.item() == 2
    idx1, _ = oracle.topk_select(sc, lens, 1)
    assert idx1[0, 0].tolist() == g["selected_budget1"]
    q = _bf([_pad(g["real_query_dim0_dim1"])])[None]
    out, lse = oracle.sparse_decode_attn(k, v, bt, lens, q, idx2, cnt2, g["sm_scale"])
    assert out[0, 0, 0].item() == g["attention_out_dim0"] and (out[0, 0, 1:] == 0).all()
    assert math.isclose(lse.item(), g["lse"], rel_tol=1e-6)


def test_overlap_hand_example():
    g = GOLD["overlap_ratio"]
    a = torch.tensor([[g["set_a"]]], dtype=torch.int32)
    b = torch.tensor([[g["set_b"]]], dtype=torch.int32)
    n = torch.tensor([[len(g["set_a"])]], dtype=torch.int32)
    inter, ratio = oracle.overlap_ratio(a, n, b, n)
    assert inter.item() == g["intersection"] and ratio.item() == g["ratio"]


import pytest  # noqa: E402


@pytest.mark.gpu
def test_hip_path_reproduces_the_hand_examples():
    from paper_2510_07486_amd import api
    g = GOLD["predictor_w2_orthogonal"]
    qw = _bf([[_pad(r) for r in g["window_oldest_first"]]])[None].cuda()
    qc = _bf([_pad(g["q_cur"])])[None].cuda()
    for mode in (api.AS_PRED_PER_WINDOW, api.AS_PRED_SINGLE_SOLVE):
        p = api.make_params(1, 1, 1, 2, 2, 1, ridge_eps=g["eps"], softmax_beta=g["beta"], sm_scale=1.0, predictor=mode)
        ctx = api.Context(p)
        q_hat = api.as_predict_query(ctx, p, qw, qc)
        assert q_hat[0, 0, :2].tolist() == g["q_hat"] and (q_hat[0, 0, 2:] == 0).all()
    s = GOLD["select_and_attend_four_tokens"]
    k = torch.zeros((1, 1, 16, 128), dtype=torch.bfloat16)
    v = torch.zeros((1, 1, 16, 128), dtype=torch.bfloat16)
    for n, (kk, vv) in enumerate(zip(s["keys_dim0_dim1"], s["values_dim0"])):
        k[0, 0, n, :2] = _bf(kk)
        v[0, 0, n, 0] = vv
    kv = api.kv_view(k.cuda(), v.cuda(), torch.zeros((1, 1), dtype=torch.int32).cuda(),
                     torch.tensor([4], dtype=torch.int32).cuda())
    q_hat = torch.tensor(_pad(s["q_hat_dim0_dim1"]))[None, None].cuda()
    for budget, want in ((2, s["selected_budget2"]), (1, s["selected_budget1"])):
        p = api.make_params(1, 1, 1, 2, budget, 1, sm_scale=s["sm_scale"])
        ctx = api.Context(p)
        idx, cnt = api.as_score_topk(ctx, p, kv, q_hat)
        assert idx[0, 0].tolist() == want and cnt.item() == budget
        if budget == 2:
            q = _bf([_pad(s["real_query_dim0_dim1"])])[None].cuda()
            out, lse = api.as_sparse_decode_attn(ctx, p, kv, q, idx, cnt)
            assert out[0, 0, 0].item() == s["attention_out_dim0"] and (out[0, 0, 1:] == 0).all()
            assert math.isclose(lse.item(), s["lse"], rel_tol=1e-6)
    o = GOLD["overlap_ratio"]
    p = api.make_params(1, 1, 1, 1, 4, 1)
    ctx = api.Context(p)
    n = torch.tensor([[4]], dtype=torch.int32).cuda()
    inter, ratio = api.as_overlap_ratio(ctx, p, torch.tensor([[o["set_a"]]], dtype=torch.int32).cuda(), n,
                                        torch.tensor([[o["set_b"]]], dtype=torch.int32).cuda(), n)
    assert inter.item() == o["intersection"] and ratio.item() == o["ratio"]
