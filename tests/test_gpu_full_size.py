"""Parity at the benchmark workloads' full sizes, in the launch configuration bench.py times: one layer of c3 / c4 / c5 is
generated on the device, the HIP path runs on the whole batch (selection on its own stream, attention on another,
event hand-off), the layer is copied to the host and EVERY (sequence, KV head) row is checked against the oracle:
selection sets with the tie band (swaps counted), q_hat and attention outputs within 2e-2, lse within 1e-3."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_07486_amd import api
from paper_2510_07486_amd import workloads as wl
from gpu_common import SCALE, f32
from helpers import compare_selection

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,budget", [("c3", 2048), ("c4", 4096), ("c5", 1024), ("c5", 4096)])
def test_full_size_every_row_against_the_oracle(name, budget):
    print("full-size", name, budget, flush=True)
    w = wl.scaled(wl.CONFIGS[name], budget=budget, layers=1)
    inp = wl.make_inputs(w, "cuda")
    eps = f32(1e-2)
    p = api.make_params(w.batch, w.n_q_heads, w.n_kv_heads, w.window, w.budget, inp.max_pages, ridge_eps=eps,
                        sm_scale=f32(SCALE))
    ctx = api.Context(p)
    kv = api.kv_view(inp.k_pool, inp.v_pool, inp.block_table, inp.ctx_lens)
    s_sel, s_att = torch.cuda.Stream(), torch.cuda.Stream()
    sel_idx = torch.empty((w.batch, w.n_kv_heads, w.budget), dtype=torch.int32, device="cuda")
    sel_cnt = torch.empty((w.batch, w.n_kv_heads), dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    api.as_select_step(ctx, p, kv, inp.q_win, inp.q_cur, sel_idx, sel_cnt, stream=s_sel)     # selection stream
    ev = torch.cuda.Event(); ev.record(s_sel)
    s_att.wait_event(ev)
    out, lse = api.as_sparse_decode_attn(ctx, p, kv, inp.q_real, sel_idx, sel_cnt, stream=s_att)
    q_hat = api.as_predict_query(ctx, p, inp.q_win, inp.q_cur, stream=s_att)
    torch.cuda.synchronize()
    print("  HIP path done; copying the layer to the host", flush=True)
    k_cpu, v_cpu = inp.k_pool.cpu(), inp.v_pool.cpu()
    bt, lens = inp.block_table.cpu(), inp.ctx_lens.cpu()
    rq, rs, ridx, rcnt = oracle.select_step(k_cpu, bt, lens, inp.q_win.cpu(), inp.q_cur.cpu(), w.budget, eps)
    print("  oracle selection done", flush=True)
    assert (q_hat.cpu() - rq).abs().max().item() <= 2e-2
    swaps = compare_selection(sel_idx, sel_cnt, ridx, rcnt, rs, lens, w.budget)      # every (sequence, KV head) row
    ref, ref_lse = oracle.sparse_decode_attn(k_cpu, v_cpu, bt, lens, inp.q_real.cpu(), sel_idx.cpu(), sel_cnt.cpu(),
                                             f32(SCALE))
    err = (out.cpu().float() - ref.float()).abs().max().item()
    lse_err = (lse.cpu() - ref_lse).abs().max().item()
    print(f"  {name} budget {budget}: {w.batch * w.n_kv_heads} rows compared, tie swaps {swaps}, "
          f"attention max abs err {err:.3e}, lse err {lse_err:.2e}", flush=True)
    assert err <= 2e-2
    assert lse_err <= 1e-3
    assert ctx.damaged_workspace_gap(p) == -1      # no kernel outgrew its region of the workspace at full size


def test_million_token_context_and_largest_budget():
    """One sequence of 1,000,003 tokens (ragged last page; rows cut into dozens of shares, candidates merged from
    global memory) with budget 4096, then the largest supported budget (65536) on 70,001 tokens; the whole row is
    checked against the oracle."""
    for n_tok, budget, seed in ((1_000_003, 4096, 41), (70_001, 65536, 42)):
        print("long-context", n_tok, budget, flush=True)
        w = wl.Workload("long", 1, 8, 2, 16, budget, n_tok, page_table="permute", n_outlier=4, seed=seed)
        cpu = wl.make_inputs(w)
        dev = wl.Inputs(w, cpu.k_pool.cuda(), cpu.v_pool.cuda(), cpu.block_table.cuda(), cpu.ctx_lens.cuda(),
                        cpu.q_win.cuda(), cpu.q_cur.cuda(), cpu.q_real.cuda())
        eps = f32(1e-2)
        p = api.make_params(1, 8, 2, 16, budget, cpu.max_pages, ridge_eps=eps, sm_scale=f32(SCALE))
        ctx = api.Context(p)
        kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
        gidx, gcnt = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
        out, lse = api.as_sparse_decode_attn(ctx, p, kv, dev.q_real, gidx, gcnt)
        torch.cuda.synchronize()
        rq, rs, ridx, rcnt = oracle.select_step(cpu.k_pool, cpu.block_table, cpu.ctx_lens, cpu.q_win, cpu.q_cur, budget,
                                                eps)
        swaps = compare_selection(gidx, gcnt, ridx, rcnt, rs, cpu.ctx_lens, budget)
        ref, ref_lse = oracle.sparse_decode_attn(cpu.k_pool, cpu.v_pool, cpu.block_table, cpu.ctx_lens, cpu.q_real,
                                                 gidx.cpu(), gcnt.cpu(), f32(SCALE))
        err = (out.cpu().float() - ref.float()).abs().max().item()
        print(f"  plan {api.select_plan(p)}, tie swaps {swaps}, attention max abs err {err:.3e}", flush=True)
        assert err <= 2e-2
        assert (lse.cpu() - ref_lse).abs().max().item() <= 1e-3
        assert ctx.damaged_workspace_gap(p) == -1


def test_block_table_too_wide_for_a_share_plan_runs_the_stages():
    """A budget above the pruning limit needs buffer-sized shares; a block table of 2^25 tokens per sequence would
    need more of them than the merge kernel indexes.  The single-layer calls then score into the workspace and run
    the stand-alone top-k; packs are refused.  The cached context is short, only the table is wide."""
    budget, n_tok, max_pages = 5000, 50_001, (1 << 25) // 16
    w = wl.Workload("wide", 1, 8, 2, 8, budget, n_tok, page_table="permute", seed=77)
    cpu = wl.make_inputs(w)
    bt = torch.zeros((1, max_pages), dtype=torch.int32)
    bt[:, :cpu.max_pages] = cpu.block_table
    eps = f32(1e-2)
    p = api.make_params(1, 8, 2, 8, budget, max_pages, ridge_eps=eps, sm_scale=f32(SCALE))
    assert api.select_plan(p, 1)[1] > 1024
    ctx = api.Context(p)
    kv = api.kv_view(cpu.k_pool.cuda(), cpu.v_pool.cuda(), bt.cuda(), cpu.ctx_lens.cuda())
    print("wide-table", n_tok, budget, "workspace MiB", api.as_workspace_bytes(p) >> 20, flush=True)
    gidx, gcnt = api.as_select_step(ctx, p, kv, cpu.q_win.cuda(), cpu.q_cur.cuda())
    torch.cuda.synchronize()
    rq, rs, ridx, rcnt = oracle.select_step(cpu.k_pool, cpu.block_table, cpu.ctx_lens, cpu.q_win, cpu.q_cur, budget, eps)
    swaps = compare_selection(gidx, gcnt, ridx, rcnt, rs, cpu.ctx_lens, budget)
    print(f"  tie swaps {swaps}", flush=True)
    assert ctx.damaged_workspace_gap(p) == -1
    with pytest.raises(api.AsError) as e:
        api.as_select_step_pack(api.Context(api.make_params(1, 8, 2, 8, 64, 16), pack=2), p,
                                [api.layer_io(kv, cpu.q_win.cuda(), cpu.q_cur.cuda(), gidx, gcnt)] * 2)
    assert e.value.code == 2


def test_full_size_packed_selection_two_layers():
    """Workload c3 at full size, two layers in one as_select_step_pack call (512 rows of 32768 tokens in one
    grid): every row equals the single-layer call bit for bit, and one sampled sequence per layer equals the oracle."""
    w = wl.scaled(wl.CONFIGS["c3"], layers=1)
    eps = f32(1e-2)
    layers = [wl.make_inputs(w, "cuda", layer=l) for l in range(2)]
    p = api.make_params(w.batch, w.n_q_heads, w.n_kv_heads, w.window, w.budget, layers[0].max_pages, ridge_eps=eps,
                        sm_scale=f32(SCALE))
    ctx = api.Context(p, pack=2)
    kvs = [api.kv_view(x.k_pool, x.v_pool, x.block_table, x.ctx_lens) for x in layers]
    sel = [(torch.empty((w.batch, w.n_kv_heads, w.budget), dtype=torch.int32, device="cuda"),
            torch.empty((w.batch, w.n_kv_heads), dtype=torch.int32, device="cuda")) for _ in layers]
    api.as_select_step_pack(ctx, p, [api.layer_io(kvs[l], layers[l].q_win, layers[l].q_cur, sel[l][0], sel[l][1])
                                     for l in range(2)])
    torch.cuda.synchronize()
    for l, b in ((0, 9), (1, 26)):
        one_idx, one_cnt = api.as_select_step(ctx, p, kvs[l], layers[l].q_win, layers[l].q_cur)
        assert torch.equal(one_idx, sel[l][0]) and torch.equal(one_cnt, sel[l][1])
        one = wl.extract_sequence(layers[l], b)
        rq, rs, ridx, rcnt = oracle.select_step(one.k_pool, one.block_table, one.ctx_lens, one.q_win, one.q_cur,
                                                w.budget, eps)
        swaps = compare_selection(sel[l][0][b:b + 1], sel[l][1][b:b + 1], ridx, rcnt, rs, one.ctx_lens, w.budget)
        print(f"  layer {l} sequence {b}: tie swaps {swaps}", flush=True)


def test_largest_batch_the_grids_allow():
    """65535 sequences (the limit the header states), one KV head, one page each, lengths 0..16: every grid dimension that
    carries the batch is at its maximum; the batch is also beyond the size up to which the selection kernel sorts
    sequences by length.  Whole result against the oracle."""
    B, C = 65535, 3
    g = torch.Generator().manual_seed(5)
    k = torch.randn((B, 1, 16, 128), generator=g).to(torch.bfloat16)
    v = torch.randn((B, 1, 16, 128), generator=g).to(torch.bfloat16)
    bt = torch.randperm(B, generator=g).to(torch.int32).view(B, 1)
    lens = torch.randint(0, 17, (B,), generator=g, dtype=torch.int32)
    q_win = torch.randn((B, 1, 2, 128), generator=g).to(torch.bfloat16)
    q_cur = torch.randn((B, 1, 128), generator=g).to(torch.bfloat16)
    q_real = torch.randn((B, 1, 128), generator=g).to(torch.bfloat16)
    eps = f32(1e-2)
    p = api.make_params(B, 1, 1, 2, C, 1, ridge_eps=eps, sm_scale=f32(SCALE))
    ctx = api.Context(p)
    kv = api.kv_view(k.cuda(), v.cuda(), bt.cuda(), lens.cuda())
    print("largest batch", B, "workspace MiB", api.as_workspace_bytes(p) >> 20, flush=True)
    gidx, gcnt = api.as_select_step(ctx, p, kv, q_win.cuda(), q_cur.cuda())
    out, lse = api.as_sparse_decode_attn(ctx, p, kv, q_real.cuda(), gidx, gcnt)
    dense, _ = api.as_dense_decode_attn(ctx, p, kv, q_real.cuda())
    torch.cuda.synchronize()
    rq, rs, ridx, rcnt = oracle.select_step(k, bt, lens, q_win, q_cur, C, eps)
    swaps = compare_selection(gidx, gcnt, ridx, rcnt, rs, lens, C)
    ref, ref_lse = oracle.sparse_decode_attn(k, v, bt, lens, q_real, gidx.cpu(), gcnt.cpu(), f32(SCALE))
    assert (out.cpu().float() - ref.float()).abs().max().item() <= 2e-2
    full_idx = torch.arange(16, dtype=torch.int32).view(1, 1, 16).expand(B, 1, 16).contiguous()
    ref_d, _ = oracle.sparse_decode_attn(k, v, bt, lens, q_real, full_idx, lens.view(B, 1).contiguous(), f32(SCALE))
    assert (dense.cpu().float() - ref_d.float()).abs().max().item() <= 2e-2
    fin = torch.isfinite(ref_lse)
    assert torch.equal(torch.isfinite(lse.cpu()), fin) and (lse.cpu()[fin] - ref_lse[fin]).abs().max().item() <= 1e-3
    # the other entry points at the same batch: stand-alone stages, KV re-organisation, overlap ratio, state updates
    q_hat = api.as_predict_query(ctx, p, q_win.cuda(), q_cur.cuda())
    sc = api.as_score_keys(ctx, p, kv, q_hat)
    sidx, scnt = api.as_topk_select(ctx, p, sc, lens.cuda())
    assert torch.equal(sidx, gidx) and torch.equal(scnt, gcnt)
    k_out, v_out, tab, ln = api.as_gather_kv(ctx, p, kv, gidx, gcnt)
    rk, rv, rtab, rln = oracle.gather_kv(k, v, bt, gidx.cpu(), gcnt.cpu())
    assert torch.equal(tab.cpu(), rtab) and torch.equal(ln.cpu(), rln)
    for b in (0, 1, 30000, B - 1):
        n = int(rln[b])
        assert torch.equal(k_out[b, 0, :n].cpu(), rk[b, 0, :n]) and torch.equal(v_out[b, 0, :n].cpu(), rv[b, 0, :n])
    inter, ratio = api.as_overlap_ratio(ctx, p, gidx, gcnt, sidx, scnt)
    assert torch.equal(inter, gcnt)
    lens_dev = lens.cuda()
    kd, vd = k.cuda(), v.cuda()
    api.as_kv_append(ctx, p, kd, vd, bt.cuda(), lens_dev, q_real.cuda(), q_real.cuda())
    full = lens == 16
    assert torch.equal(lens_dev.cpu(), torch.where(full, lens, lens + 1))
    qw_dev, qc_dev = q_win.cuda(), q_cur.cuda()
    api.as_window_push(ctx, p, qw_dev, qc_dev, q_real.cuda())
    assert torch.equal(qc_dev.cpu(), q_real) and torch.equal(qw_dev[:, :, 1].cpu(), q_cur)
    assert ctx.damaged_workspace_gap(p) == -1
    print(f"  tie swaps {swaps}", flush=True)
