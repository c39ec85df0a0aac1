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


# ---- softmax-normalised group aggregation (agg = 2) ----
def _softmax_case(G, Hkv=2, B=2, ctx=300, scale=0.3, seed=0):
    w = wl.Workload("sm", B, G * Hkv, Hkv, 4, 16, ctx, ctx_min=50, page_table="scatter", pool_slack=1.3, seed=seed)
    cpu = wl.make_inputs(w)
    q_hat = torch.randn((B, G * Hkv, 128), generator=torch.Generator().manual_seed(seed + 1)) * 0.5
    sc = oracle.score_keys(cpu.k_pool, cpu.block_table, cpu.ctx_lens, q_hat, Hkv, 2, fill=-7.0, sm_scale=scale)
    return cpu, q_hat, sc


def test_softmax_sum_matches_numpy_and_sums_to_group_size():
    G, Hkv, scale = 4, 2, 0.3
    cpu, q_hat, sc = _softmax_case(G, Hkv, scale=scale)
    for b in range(2):
        n = int(cpu.ctx_lens[b])
        for j in range(Hkv):
            K = gather_keys(cpu.k_pool, cpu.block_table, b, j, n)                     # [n, 128] fp64
            ref = np.zeros(n)
            for g in range(G):
                l = scale * (K @ q_hat[b, j * G + g].double().numpy())
                e = np.exp(l - l.max())
                ref += e / e.sum()
            np.testing.assert_allclose(sc[b, j, :n].numpy(), ref.astype(np.float32), rtol=2e-6, atol=1e-30)
            assert abs(float(sc[b, j, :n].double().sum()) - G) < 1e-4                 # every head's mass is 1
            assert (sc[b, j, n:] == -7.0).all()                                       # nothing written past the context


def test_softmax_sum_with_one_head_ranks_like_the_raw_logits():
    # G = 1: exp is monotone, so the order of the scores (hence any top-k) is that of the raw logits
    cpu, q_hat, sc = _softmax_case(1, Hkv=3, scale=0.7, seed=5)
    raw = oracle.score_keys(cpu.k_pool, cpu.block_table, cpu.ctx_lens, q_hat, 3, 0)
    for b in range(2):
        n = int(cpu.ctx_lens[b])
        for j in range(3):
            a = np.argsort(-sc[b, j, :n].double().numpy(), kind="stable")
            r = np.argsort(-raw[b, j, :n].double().numpy(), kind="stable")
            assert np.array_equal(a[:40], r[:40])


def test_softmax_sum_is_scale_free_across_heads():
    # multiplying one head's query by a constant changes that head's distribution only; with raw-logit max or sum
    # aggregation the largest head dominates, here a head 100 x smaller in norm still contributes its full unit of mass
    cpu, q_hat, sc = _softmax_case(2, Hkv=1, B=1, ctx=200, scale=1.0, seed=9)
    q2 = q_hat.clone()
    q2[:, 1] *= 0.01
    sc2 = oracle.score_keys(cpu.k_pool, cpu.block_table, cpu.ctx_lens, q2, 1, 2, sm_scale=1.0)
    n = int(cpu.ctx_lens[0])
    assert abs(float(sc2[0, 0, :n].double().sum()) - 2.0) < 1e-4
    # head 1 became almost uniform: its contribution is close to 1/n for every token
    K = gather_keys(cpu.k_pool, cpu.block_table, 0, 0, n)
    l0 = K @ q_hat[0, 0].double().numpy()
    p0 = np.exp(l0 - l0.max()); p0 /= p0.sum()
    np.testing.assert_allclose(sc2[0, 0, :n].double().numpy() - p0, 1.0 / n, rtol=0.35)
