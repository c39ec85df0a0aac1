"""GPU parity of the cache-side calls (overlap ratio, KV append, window push, KV re-organisation)
against the oracle, bit for bit, and a multi-step decode loop that uses them the way the method
does: append -> attend over last step's selection plus the new token -> push -> select."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_07486_amd import api
from paper_2510_07486_amd import workloads as wl
from gpu_common import SCALE, f32, params_for, to_dev
from helpers import compare_selection

pytestmark = pytest.mark.gpu
OUT_TOL = 2e-2


def note(*a):
    print(*a, flush=True)


def random_sets(rng, B, H, C, N, lo):
    idx = torch.full((B, H, C), -1, dtype=torch.int32)
    cnt = torch.zeros((B, H), dtype=torch.int32)
    for b in range(B):
        for j in range(H):
            c = int(rng.integers(lo, C + 1))
            idx[b, j, :c] = torch.tensor(np.sort(rng.choice(N, size=c, replace=False)), dtype=torch.int32)
            cnt[b, j] = c
    return idx, cnt


@pytest.mark.parametrize("C,N", [(1, 5), (64, 100), (2048, 5000), (4096, 4096)])
def test_overlap_ratio_bit_exact(C, N):
    note("overlap", C, N)
    rng = np.random.default_rng(C)
    ia, ca = random_sets(rng, 3, 4, C, N, 0)
    ib, cb = random_sets(rng, 3, 4, C, N, 0)
    ib[0, 0], cb[0, 0] = ia[0, 0], ca[0, 0]                    # identical sets: ratio 1
    ca[1, 1] = 0                                               # one side empty
    ca[2, 2] = cb[2, 2] = 0                                    # both empty
    ref_i, ref_r = oracle.overlap_ratio(ia, ca, ib, cb)
    p = api.make_params(3, 4, 4, 1, C, 1)
    ctx = api.Context(p)
    got_i, got_r = api.as_overlap_ratio(ctx, p, ia.cuda(), ca.cuda(), ib.cuda(), cb.cuda())
    assert torch.equal(got_i.cpu(), ref_i)
    assert torch.equal(got_r.cpu(), ref_r)
    if ca[0, 0] > 0:
        assert got_r[0, 0].item() == 1.0


def test_overlap_of_predicted_and_real_query_selections():
    """Eq. 1 between the selection made from the predicted query and the one the real next query
    would have made, on the AR(1) workload: both sides computed by the GPU path and by the oracle."""
    w = wl.scaled(wl.CONFIGS["c2"], ctx=4096, budget=512)
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    p = params_for(cpu)
    ctx = api.Context(p)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    a_idx, a_cnt = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    b_idx, b_cnt = api.as_score_topk(ctx, p, kv, dev.q_real.float().contiguous())
    inter, ratio = api.as_overlap_ratio(ctx, p, a_idx, a_cnt, b_idx, b_cnt)
    ref_i, ref_r = oracle.overlap_ratio(a_idx.cpu(), a_cnt.cpu(), b_idx.cpu(), b_cnt.cpu())
    assert torch.equal(inter.cpu(), ref_i) and torch.equal(ratio.cpu(), ref_r)
    note("  overlap ratio S(q_hat) vs S(q_real), mean over KV heads:", ratio.mean().item())
    assert ratio.mean().item() > 0.5            # rho = 0.95: the prediction keeps most of the real selection


def test_kv_append_and_window_push_bit_exact():
    w = wl.Workload("ap", 5, 16, 4, 9, 16, 160, page_table="permute", seed=8)
    cpu = wl.make_inputs(w)
    cpu.ctx_lens[:] = torch.tensor([0, 15, 16, 77, 160], dtype=torch.int32)     # last one has no room
    dev = to_dev(cpu)
    p = params_for(cpu)
    ctx = api.Context(p)
    g = torch.Generator().manual_seed(4)
    for step in range(3):
        k_new = torch.randn((5, 4, 128), generator=g).to(torch.bfloat16)
        v_new = torch.randn((5, 4, 128), generator=g).to(torch.bfloat16)
        q_new = torch.randn((5, 16, 128), generator=g).to(torch.bfloat16)
        oracle.kv_append(cpu.k_pool, cpu.v_pool, cpu.block_table, cpu.ctx_lens, k_new, v_new)
        oracle.window_push(cpu.q_win, cpu.q_cur, q_new)
        api.as_kv_append(ctx, p, dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens, k_new.cuda(), v_new.cuda())
        api.as_window_push(ctx, p, dev.q_win, dev.q_cur, q_new.cuda())
        assert torch.equal(dev.ctx_lens.cpu(), cpu.ctx_lens)
        assert torch.equal(dev.k_pool.cpu(), cpu.k_pool) and torch.equal(dev.v_pool.cpu(), cpu.v_pool)
        assert torch.equal(dev.q_win.cpu(), cpu.q_win) and torch.equal(dev.q_cur.cpu(), cpu.q_cur)
    assert cpu.ctx_lens.tolist() == [3, 18, 19, 80, 160]


@pytest.mark.parametrize("W", [1, 2, 8, 10, 64])
def test_window_push_window_sizes(W):
    g = torch.Generator().manual_seed(W)
    q_win = torch.randn((2, 6, W, 128), generator=g).to(torch.bfloat16)
    q_cur = torch.randn((2, 6, 128), generator=g).to(torch.bfloat16)
    q_new = torch.randn((2, 6, 128), generator=g).to(torch.bfloat16)
    dw, dc = q_win.cuda(), q_cur.cuda()
    p = api.make_params(2, 6, 2, W, 16, 4)
    ctx = api.Context(p)
    api.as_window_push(ctx, p, dw, dc, q_new.cuda())
    oracle.window_push(q_win, q_cur, q_new)
    assert torch.equal(dw.cpu(), q_win) and torch.equal(dc.cpu(), q_cur)


@pytest.mark.parametrize("kw", [
    dict(batch=3, n_q_heads=8, n_kv_heads=2, ctx=300, ctx_min=20, budget=40),
    dict(batch=4, n_q_heads=32, n_kv_heads=8, ctx=5000, ctx_min=100, budget=1000),   # budget not a page multiple
    dict(batch=2, n_q_heads=16, n_kv_heads=2, ctx=700, ctx_min=600, budget=2048),    # budget above every context
])
def test_gather_kv_bit_exact_and_dense_attention_over_the_compact_pool(kw):
    note("gather", kw)
    w = wl.Workload("ga", window=4, page_table="scatter", pool_slack=1.2, seed=5, **kw)
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    C = w.budget
    q_hat = oracle.predict_query(cpu.q_win, cpu.q_cur, f32(1e-2))
    sc = oracle.score_keys(cpu.k_pool, cpu.block_table, cpu.ctx_lens, q_hat, w.n_kv_heads)
    idx, cnt = oracle.topk_select(sc, cpu.ctx_lens, C)
    rk, rv, rt, rl = oracle.gather_kv(cpu.k_pool, cpu.v_pool, cpu.block_table, idx, cnt, fill=-3.0)
    p = params_for(cpu)
    ctx = api.Context(p)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    k_out = torch.full(rk.shape, -3.0, dtype=torch.bfloat16, device="cuda")
    v_out = torch.full(rv.shape, -3.0, dtype=torch.bfloat16, device="cuda")
    _, _, table, lens = api.as_gather_kv(ctx, p, kv, idx.cuda(), cnt.cuda(), k_out, v_out)
    assert torch.equal(table.cpu(), rt) and torch.equal(lens.cpu(), rl)
    assert torch.equal(k_out.cpu(), rk) and torch.equal(v_out.cpu(), rv)
    # dense attention over the compact view against the oracle's sparse attention over the original cache
    ref, ref_lse = oracle.sparse_decode_attn(cpu.k_pool, cpu.v_pool, cpu.block_table, cpu.ctx_lens, cpu.q_real, idx, cnt,
                                             f32(SCALE))
    Cp = api.compact_pages(p)
    pc = api.make_params(w.batch, w.n_q_heads, w.n_kv_heads, w.window, 16, Cp, sm_scale=f32(SCALE))
    ctx_c = api.Context(pc)
    kvc = api.kv_view(k_out, v_out, table, lens)
    out, lse = api.as_dense_decode_attn(ctx_c, pc, kvc, dev.q_real)
    err = (out.cpu().float() - ref.float()).abs().max().item()
    note("  dense-over-compact max abs err", err)
    assert err <= OUT_TOL
    assert (lse.cpu() - ref_lse).abs().max().item() <= 1e-3


@pytest.mark.parametrize("kw", [
    dict(batch=3, n_q_heads=8, n_kv_heads=2, ctx=2000, ctx_min=1),
    dict(batch=1, n_q_heads=32, n_kv_heads=8, ctx=16384),                            # workload c2 shape, full context
    dict(batch=5, n_q_heads=64, n_kv_heads=8, ctx=700, ctx_min=300),                 # group of 8
    dict(batch=2, n_q_heads=40, n_kv_heads=1, ctx=1500, ctx_min=700),                # MQA, three head blocks
])
def test_dense_decode_attn_matches_oracle(kw):
    """Full attention over the whole cache (the baseline of Appendix B) = the oracle's attention with an
    empty selection and the dense tail starting at token 0."""
    note("dense", kw)
    w = wl.Workload("da", window=4, budget=64, page_table="scatter", pool_slack=1.2, seed=23, **kw)
    cpu = wl.make_inputs(w)
    if w.batch > 1:
        cpu.ctx_lens[0] = 0                                    # an empty sequence: out = 0, lse = -inf
    dev = to_dev(cpu)
    B, Hkv = w.batch, w.n_kv_heads
    ref, ref_lse = oracle.sparse_decode_attn(cpu.k_pool, cpu.v_pool, cpu.block_table, cpu.ctx_lens, cpu.q_real,
                                             torch.full((B, Hkv, 1), -1, dtype=torch.int32),
                                             torch.zeros((B, Hkv), dtype=torch.int32), f32(SCALE),
                                             torch.zeros((B,), dtype=torch.int32))
    p = params_for(cpu)
    ctx = api.Context(p, workspace_bytes=api.as_workspace_bytes_attn(p))     # a ctx that only attends
    out, lse = api.as_dense_decode_attn(ctx, p, api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens),
                                        dev.q_real)
    torch.cuda.synchronize()
    err = (out.cpu().float() - ref.float()).abs().max().item()
    note("  dense attn max abs err", err)
    assert err <= OUT_TOL
    fin = torch.isfinite(ref_lse)
    assert torch.equal(torch.isfinite(lse.cpu()), fin)
    assert (lse.cpu()[fin] - ref_lse[fin]).abs().max().item() <= 1e-3
    assert (out.cpu()[~fin].float() == 0).all()


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (16, 2), (6, 2)])
@pytest.mark.parametrize("splits", [0, 1, 3])
def test_sparse_attention_with_tail_under_forced_split_counts(Hq, Hkv, splits):
    """Selection + own-token tail, under the library's split rule and under forced split counts (the per-ctx
    development knob): the result does not depend on how the token list is cut."""
    w = wl.Workload("va", 3, Hq, Hkv, 4, 300, 2000, ctx_min=100, page_table="scatter", pool_slack=1.2, seed=Hq)
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    q_hat = oracle.predict_query(cpu.q_win, cpu.q_cur, f32(1e-2))
    sc = oracle.score_keys(cpu.k_pool, cpu.block_table, cpu.ctx_lens, q_hat, Hkv)
    lens_sel = torch.clamp(cpu.ctx_lens - 1, min=0)
    idx, cnt = oracle.topk_select(sc, lens_sel, 300)
    ref, ref_lse = oracle.sparse_decode_attn(cpu.k_pool, cpu.v_pool, cpu.block_table, cpu.ctx_lens, cpu.q_real, idx, cnt,
                                             f32(SCALE), lens_sel)
    p = params_for(cpu)
    ctx = api.Context(p, workspace_bytes=max(api.as_workspace_bytes_attn(p), api.attn_workspace_bytes_forced(p, splits)))
    ctx.set_attn_splits(splits)
    out, lse = api.as_sparse_decode_attn(ctx, p, api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens),
                                         dev.q_real, idx.cuda(), cnt.cuda(), lens_sel.cuda())
    torch.cuda.synchronize()
    assert (out.cpu().float() - ref.float()).abs().max().item() <= OUT_TOL
    assert (lse.cpu() - ref_lse).abs().max().item() <= 1e-3
    if splits == 3:     # a forced count beyond what the workspace was sized for is refused, not overrun
        small = api.Context(p, workspace_bytes=api.as_workspace_bytes_attn(p))
        small.set_attn_splits(2)       # 300 tokens allow at most ceil(300 / 128) = 3 splits; the rule gives fewer rows
        need = api.attn_workspace_bytes_forced(p, 2)
        if need > small.workspace_bytes:
            with pytest.raises(api.AsError) as e:
                api.as_sparse_decode_attn(small, p, api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens),
                                          dev.q_real, idx.cuda(), cnt.cuda(), lens_sel.cuda())
            assert e.value.code == 3


def test_decode_loop_append_attend_push_select():
    """Five decode steps on both sides.  Step t+1 attends over the selection made at step t plus the
    token appended since (the dense tail), then the window slides and the next selection is made."""
    w = wl.Workload("loop", 3, 8, 2, 8, 96, 640, page_table="permute", seed=14)
    cpu = wl.make_inputs(w)
    cpu.ctx_lens[:] = torch.tensor([600, 333, 50], dtype=torch.int32)           # room to grow in the mapped pages
    dev = to_dev(cpu)
    p = params_for(cpu)
    ctx = api.Context(p)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    g = torch.Generator().manual_seed(2)
    eps = f32(1e-2)
    # selection for the first step, from the initial window
    sel_lens = cpu.ctx_lens.clone()
    _, sc, ridx, rcnt = oracle.select_step(cpu.k_pool, cpu.block_table, cpu.ctx_lens, cpu.q_win, cpu.q_cur, w.budget, eps)
    gidx, gcnt = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    swaps = compare_selection(gidx, gcnt, ridx, rcnt, sc, cpu.ctx_lens, w.budget)
    for step in range(5):
        k_new = torch.randn((3, 2, 128), generator=g).to(torch.bfloat16)
        v_new = torch.randn((3, 2, 128), generator=g).to(torch.bfloat16)
        q_new = (0.9 * cpu.q_cur.float() + 0.1 * torch.randn((3, 8, 128), generator=g)).to(torch.bfloat16)
        oracle.kv_append(cpu.k_pool, cpu.v_pool, cpu.block_table, cpu.ctx_lens, k_new, v_new)
        api.as_kv_append(ctx, p, dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens, k_new.cuda(), v_new.cuda())
        # attention of this step: last step's selection + the token that arrived after it
        out, lse = api.as_sparse_decode_attn(ctx, p, kv, q_new.cuda(), gidx, gcnt, sel_lens.cuda())
        ref, ref_lse = oracle.sparse_decode_attn(cpu.k_pool, cpu.v_pool, cpu.block_table, cpu.ctx_lens, q_new,
                                                 gidx.cpu(), gcnt.cpu(), f32(SCALE), sel_lens)
        err = (out.cpu().float() - ref.float()).abs().max().item()
        assert err <= OUT_TOL, (step, err)
        assert (lse.cpu() - ref_lse).abs().max().item() <= 1e-3
        # slide the window and select for the next step
        oracle.window_push(cpu.q_win, cpu.q_cur, q_new)
        api.as_window_push(ctx, p, dev.q_win, dev.q_cur, q_new.cuda())
        sel_lens = cpu.ctx_lens.clone()
        _, sc, ridx, rcnt = oracle.select_step(cpu.k_pool, cpu.block_table, cpu.ctx_lens, cpu.q_win, cpu.q_cur, w.budget,
                                               eps)
        gidx, gcnt = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
        swaps += compare_selection(gidx, gcnt, ridx, rcnt, sc, cpu.ctx_lens, w.budget)
        assert torch.equal(dev.ctx_lens.cpu(), cpu.ctx_lens)
    note("  decode loop: tie swaps over 6 selections:", swaps)
    assert torch.equal(dev.k_pool.cpu(), cpu.k_pool) and torch.equal(dev.q_win.cpu(), cpu.q_win)


def test_plain_c_caller_of_the_abi():
    """abi_demo (C99, gcc, HIP runtime for allocations) runs predict -> selection -> attention on a hand-checkable
    case through the C ABI and verifies the results itself."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(api.LIB_PATH), "abi_demo")
    assert os.path.exists(exe), "run the build first"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    note(" ", r.stdout.strip().replace("\n", " | "))
    assert r.returncode == 0 and "abi_demo: OK" in r.stdout, r.stderr
