"""Pins for the oracle's sparse decode attention (Sec. 4.1; Appendix B's 4*q*h*C term)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2510_07486_amd import workloads as wl
from helpers import gather_keys

SCALE = 1.0 / math.sqrt(128)


def small(**kw):
    base = wl.Workload("t", 2, 8, 2, 4, 16, 90, ctx_min=40, page_table="scatter", pool_slack=1.3, seed=11)
    return wl.make_inputs(wl.scaled(base, **kw))


def all_tokens(inp, C):
    B, H = inp.w.batch, inp.w.n_kv_heads
    idx = torch.full((B, H, C), -1, dtype=torch.int32)
    cnt = torch.zeros((B, H), dtype=torch.int32)
    for b in range(B):
        n = int(inp.ctx_lens[b])
        idx[b, :, :n] = torch.arange(n, dtype=torch.int32)
        cnt[b] = n
    return idx, cnt


def dense_sdpa(inp, b):
    """torch's CPU scaled_dot_product_attention in fp64 over the whole context of sequence b."""
    n = int(inp.ctx_lens[b])
    G = inp.w.group
    outs, lses = [], []
    for h in range(inp.w.n_q_heads):
        K = torch.from_numpy(gather_keys(inp.k_pool, inp.block_table, b, h // G, n))
        V = torch.from_numpy(gather_keys(inp.v_pool, inp.block_table, b, h // G, n))
        q = inp.q_real[b, h].double()[None]
        outs.append(F.scaled_dot_product_attention(q[None], K[None], V[None], scale=SCALE)[0, 0])
        lses.append(torch.logsumexp((K @ q[0]) * SCALE, 0))
    return torch.stack(outs), torch.stack(lses)


def test_budget_covering_context_equals_dense_attention():
    inp = small()
    idx, cnt = all_tokens(inp, 128)
    out, lse = oracle.sparse_decode_attn(inp.k_pool, inp.v_pool, inp.block_table, inp.ctx_lens, inp.q_real,
                                         idx, cnt, SCALE)
    for b in range(inp.w.batch):
        ref, ref_lse = dense_sdpa(inp, b)
        assert torch.equal(out[b], ref.to(torch.bfloat16))          # same value, one rounding to bf16
        np.testing.assert_allclose(lse[b].numpy(), ref_lse.numpy(), rtol=1e-6)


def test_topk_with_budget_above_context_gives_dense_attention():
    inp = small()
    q_hat = oracle.predict_query(inp.q_win, inp.q_cur, 1e-2)
    s = oracle.score_keys(inp.k_pool, inp.block_table, inp.ctx_lens, q_hat, 2)
    idx, cnt = oracle.topk_select(s, inp.ctx_lens, 128)
    out, _ = oracle.sparse_decode_attn(inp.k_pool, inp.v_pool, inp.block_table, inp.ctx_lens, inp.q_real,
                                       idx, cnt, SCALE)
    for b in range(inp.w.batch):
        assert torch.equal(out[b], dense_sdpa(inp, b)[0].to(torch.bfloat16))


def test_dense_tail_completes_a_prefix_selection():
    # select everything below a cut, attend the rest as the dense tail: again dense attention
    inp = small()
    cut = torch.tensor([25, 33], dtype=torch.int32)
    idx = torch.full((2, 2, 64), -1, dtype=torch.int32)
    cnt = torch.zeros((2, 2), dtype=torch.int32)
    for b in range(2):
        idx[b, :, :cut[b]] = torch.arange(int(cut[b]), dtype=torch.int32)
        cnt[b] = cut[b]
    out, lse = oracle.sparse_decode_attn(inp.k_pool, inp.v_pool, inp.block_table, inp.ctx_lens, inp.q_real,
                                         idx, cnt, SCALE, sel_ctx_lens=cut)
    for b in range(2):
        ref, ref_lse = dense_sdpa(inp, b)
        assert torch.equal(out[b], ref.to(torch.bfloat16))
        np.testing.assert_allclose(lse[b].numpy(), ref_lse.numpy(), rtol=1e-6)


def test_single_token_returns_its_value_row():
    inp = small()
    idx = torch.full((2, 2, 4), -1, dtype=torch.int32)
    idx[:, :, 0] = torch.tensor([[7, 30], [0, 39]], dtype=torch.int32)
    cnt = torch.ones((2, 2), dtype=torch.int32)
    out, lse = oracle.sparse_decode_attn(inp.k_pool, inp.v_pool, inp.block_table, inp.ctx_lens, inp.q_real,
                                         idx, cnt, SCALE)
    for b in range(2):
        for h in range(8):
            j = h // 4
            n = int(idx[b, j, 0])
            V = gather_keys(inp.v_pool, inp.block_table, b, j, n + 1)[n]
            K = gather_keys(inp.k_pool, inp.block_table, b, j, n + 1)[n]
            assert np.array_equal(out[b, h].double().numpy(), V)
            assert abs(float(lse[b, h]) - SCALE * float(K @ inp.q_real[b, h].double().numpy())) < 1e-5


def test_constant_values_and_index_order_invariance():
    inp = small()
    g = torch.Generator().manual_seed(0)
    idx = torch.full((2, 2, 16), -1, dtype=torch.int32)
    for b in range(2):
        for j in range(2):
            idx[b, j, :12] = torch.randperm(40, generator=g)[:12].sort().values.to(torch.int32)
    cnt = torch.full((2, 2), 12, dtype=torch.int32)
    a, la = oracle.sparse_decode_attn(inp.k_pool, inp.v_pool, inp.block_table, inp.ctx_lens, inp.q_real, idx, cnt, SCALE)
    idx2 = idx.clone()
    idx2[:, :, :12] = idx[:, :, :12].flip(-1)
    b_, lb = oracle.sparse_decode_attn(inp.k_pool, inp.v_pool, inp.block_table, inp.ctx_lens, inp.q_real, idx2, cnt, SCALE)
    assert torch.equal(a, b_)
    np.testing.assert_allclose(la.numpy(), lb.numpy(), rtol=1e-6)
    v_const = torch.full_like(inp.v_pool, 0.75)
    c, _ = oracle.sparse_decode_attn(inp.k_pool, v_const, inp.block_table, inp.ctx_lens, inp.q_real, idx, cnt, SCALE)
    assert (c.float() == 0.75).all()


def test_empty_selection():
    inp = small()
    idx = torch.full((2, 2, 4), -1, dtype=torch.int32)
    cnt = torch.zeros((2, 2), dtype=torch.int32)
    out, lse = oracle.sparse_decode_attn(inp.k_pool, inp.v_pool, inp.block_table, inp.ctx_lens, inp.q_real, idx, cnt, SCALE)
    assert (out.float() == 0).all() and torch.isinf(lse).all() and (lse < 0).all()


def test_bf16_rounding_helper_is_single_round_to_nearest_even():
    t = torch.tensor([1.0, 1.00390625, 1.01171875, -3.3, 1e-40, 65504.0, 0.1], dtype=torch.float64)
    for x in t.tolist():
        exp = torch.tensor(x, dtype=torch.float64).to(torch.bfloat16).view(torch.int16).item() & 0xFFFF
        assert oracle.f64_to_bf16(x) == exp, x
    # a value that double rounding through fp32 would get wrong: just above a bf16 tie
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert oracle.f64_to_bf16(x) == 0x3F81
