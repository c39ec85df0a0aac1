"""Pins for the oracle's scoring (Alg. 1 step 7, Sec. 4.3 shapes) and top-k (Sec. 4.3 item 2)."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2510_07486_amd import workloads as wl
from helpers import gather_keys


def small(**kw):
    base = wl.Workload("t", 2, 8, 2, 4, 16, 100, ctx_min=37, page_table="scatter", pool_slack=1.5, seed=3)
    return wl.make_inputs(wl.scaled(base, **kw))


def test_mha_scoring_is_a_gemv():
    # one query head per KV head: s = K q (library routine)
    inp = small(n_q_heads=2, n_kv_heads=2)
    q_hat = torch.randn((2, 2, 128), generator=torch.Generator().manual_seed(0))
    s = oracle.score_keys(inp.k_pool, inp.block_table, inp.ctx_lens, q_hat, 2)
    for b in range(2):
        n = int(inp.ctx_lens[b])
        for j in range(2):
            K = gather_keys(inp.k_pool, inp.block_table, b, j, n)
            ref = (K @ q_hat[b, j].double().numpy()).astype(np.float32)
            np.testing.assert_array_equal(s[b, j, :n].numpy(), ref + np.float32(0))
            assert torch.isnan(s[b, j, n:]).all()        # entries past the context stay untouched


@pytest.mark.parametrize("agg", [0, 1])
def test_gqa_group_aggregation(agg):
    inp = small()
    G = inp.w.group
    q_hat = torch.randn((2, 8, 128), generator=torch.Generator().manual_seed(1))
    s = oracle.score_keys(inp.k_pool, inp.block_table, inp.ctx_lens, q_hat, 2, agg)
    for b in range(2):
        n = int(inp.ctx_lens[b])
        for j in range(2):
            K = gather_keys(inp.k_pool, inp.block_table, b, j, n)
            per_head = K @ q_hat[b, j * G:(j + 1) * G].double().numpy().T     # [n, G]
            ref = per_head.max(axis=1) if agg == 0 else per_head.sum(axis=1)
            np.testing.assert_allclose(s[b, j, :n].numpy(), ref, rtol=2e-7, atol=1e-6)


def test_identical_queries_in_group_reduce_to_one_head():
    inp = small()
    q1 = torch.randn((2, 2, 1, 128), generator=torch.Generator().manual_seed(2))
    q_rep = q1.expand(2, 2, 4, 128).reshape(2, 8, 128).contiguous()
    a = oracle.score_keys(inp.k_pool, inp.block_table, inp.ctx_lens, q_rep, 2, 0, fill=0.0)
    b = oracle.score_keys(inp.k_pool, inp.block_table, inp.ctx_lens, q1.reshape(2, 2, 128).contiguous(), 2, 0, fill=0.0)
    assert torch.equal(a, b)


def test_page_permutation_invariance():
    # paging is storage only: moving pages around (with the table) changes nothing
    inp = small()
    q_hat = torch.randn((2, 8, 128), generator=torch.Generator().manual_seed(3))
    a = oracle.score_keys(inp.k_pool, inp.block_table, inp.ctx_lens, q_hat, 2, fill=0.0)
    perm = torch.randperm(inp.num_pages, generator=torch.Generator().manual_seed(4))
    inv = torch.empty_like(perm); inv[perm] = torch.arange(inp.num_pages)
    k2 = inp.k_pool[perm].contiguous()                 # new page p holds old page perm[p]
    bt2 = inv[inp.block_table.long()].to(torch.int32)
    b = oracle.score_keys(k2, bt2, inp.ctx_lens, q_hat, 2, fill=0.0)
    assert torch.equal(a, b)


def test_negative_zero_is_canonicalised():
    inp = small(batch=1, ctx=16, ctx_min=None, page_table="identity")
    inp.k_pool.zero_()
    q_hat = -torch.ones((1, 8, 128))
    s = oracle.score_keys(inp.k_pool, inp.block_table, inp.ctx_lens, q_hat, 2)
    bits = s[0, 0, :16].view(torch.int32)
    assert (bits == 0).all()


# ------------------------------------------------------------------ top-k

def brute_topk(s, C):
    order = np.argsort(-s.astype(np.float64), kind="stable")       # score desc, index asc among equals
    return np.sort(order[: min(C, len(s))])


def run_topk(rows, C, lens=None):
    s = torch.tensor(np.asarray(rows, dtype=np.float32))[None]      # [1, H, N]
    n = s.shape[2]
    lens = torch.tensor([n if lens is None else lens], dtype=torch.int32)
    idx, cnt = oracle.topk_select(s, lens, C)
    return idx[0].numpy(), cnt[0].numpy()


def test_topk_exhaustive_small_with_ties():
    # every score pattern over {0,1,2}^5 and every budget: equals a stable full sort
    for pat in itertools.product([0.0, 1.0, 2.0], repeat=5):
        for C in range(1, 7):
            idx, cnt = run_topk([pat], C)
            exp = brute_topk(np.array(pat, dtype=np.float32), C)
            assert cnt[0] == len(exp)
            assert list(idx[0, :cnt[0]]) == list(exp), (pat, C)
            assert np.all(idx[0, cnt[0]:] == -1)


def test_topk_random_rows_match_argsort():
    rng = np.random.default_rng(0)
    for N, C in [(1, 1), (17, 4), (64, 64), (64, 100), (1000, 37), (4096, 256)]:
        rows = rng.standard_normal((3, N)).astype(np.float32)
        rows[1] = np.round(rows[1] * 2) / 2                    # many exact ties
        idx, cnt = run_topk(rows, C)
        for r in range(3):
            exp = brute_topk(rows[r], C)
            assert cnt[r] == len(exp) and np.array_equal(idx[r, :cnt[r]], exp)


def test_topk_ties_take_lowest_index():
    idx, cnt = run_topk([[1.0, 5.0, 1.0, 1.0, 0.0, 1.0]], 3)
    assert list(idx[0]) == [0, 1, 2]
    idx, cnt = run_topk([[-0.0, 0.0, -0.0, 0.0]], 2)            # signed zeros compare equal
    assert list(idx[0]) == [0, 1]


def test_topk_respects_context_length_and_nan():
    idx, cnt = run_topk([[1.0, 9.0, 3.0, 99.0, 99.0]], 2, lens=3)
    assert cnt[0] == 2 and list(idx[0]) == [1, 2]
    idx, cnt = run_topk([[float("nan"), -np.inf, 1.0]], 2)       # NaN ranks below -inf
    assert list(idx[0]) == [1, 2]
    idx, cnt = run_topk([[0.5, 0.25]], 4, lens=0)
    assert cnt[0] == 0 and np.all(idx[0] == -1)


def test_selection_invariant_under_positive_scaling_of_query():
    inp = small()
    q_hat = torch.randn((2, 8, 128), generator=torch.Generator().manual_seed(5))
    a = oracle.score_keys(inp.k_pool, inp.block_table, inp.ctx_lens, q_hat, 2)
    b = oracle.score_keys(inp.k_pool, inp.block_table, inp.ctx_lens, 4.0 * q_hat, 2)
    ia, ca = oracle.topk_select(a, inp.ctx_lens, 16)
    ib, cb = oracle.topk_select(b, inp.ctx_lens, 16)
    assert torch.equal(ia, ib) and torch.equal(ca, cb)
