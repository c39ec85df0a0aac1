"""Few-row shapes: scoring and the per-row top-k in one launch (the workgroup that completes a row's arrival count
selects it) against the two stand-alone kernels, one after the other (per-ctx development mode).  Same scores, so the
selections must agree bit for bit, on every repetition (the arrival counters return to zero); and both against the
oracle.  Cases: the two few-row workloads, rows shorter than the budget, empty sequences (their workgroups arrive
too), a ragged batch, the longest rows the register top-k holds (32768 tokens), groups of 16 heads (two operand
sets), sum aggregation, a block table wider than every sequence, a budget of 1."""
import pytest
import torch

import oracle
from paper_2510_07486_amd import api
from paper_2510_07486_amd import workloads as wl
from gpu_common import f32, params_for, to_dev
from helpers import compare_selection

pytestmark = pytest.mark.gpu

CASES = [
    # batch, Hq, Hkv, W, budget, ctx, ctx_min, agg
    (1, 8, 2, 8, 256, 4096, None, 0),        # workload c1
    (1, 32, 8, 16, 2048, 16384, None, 0),    # workload c2
    (1, 32, 8, 16, 2048, 32768, None, 0),    # the longest rows of the register top-k: 32 keys per thread
    (2, 8, 2, 8, 600, 500, 100, 0),          # rows shorter than the budget: everything is kept
    (4, 8, 2, 4, 64, 3000, 0, 1),            # sum aggregation; sequences of length 0
    (3, 32, 2, 8, 100, 5000, 1, 0),          # groups of 16 heads: two operand sets; ragged down to one token
    (2, 4, 4, 8, 1, 1000, 300, 0),           # budget 1 (MHA)
    (2, 16, 4, 8, 333, 7000, 2500, 0),       # odd page counts: the last iteration of a wavefront has one page
]


@pytest.mark.parametrize("case", CASES)
def test_one_launch_equals_the_two_stand_alone_kernels(case):
    B, Hq, Hkv, W, C, ctx_len, ctx_min, agg = case
    print("select rows", case, flush=True)
    w = wl.Workload("sr", B, Hq, Hkv, W, C, ctx_len, ctx_min=ctx_min, page_table="scatter", pool_slack=1.3, seed=C + B)
    cpu = wl.make_inputs(w)
    if ctx_min == 0:
        cpu.ctx_lens[0] = 0
        cpu.ctx_lens[B - 1] = 0
    dev = to_dev(cpu)
    p = params_for(cpu, agg=agg)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    ctx = api.Context(p)
    ctx.set_select_mode(1)                                    # the two stand-alone kernels
    ri, rc = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    torch.cuda.synchronize()
    ctx.set_select_mode(0)
    share, shares, cand = api.select_plan(p, 1)
    for rep in range(5):
        gi, gc = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
        torch.cuda.synchronize()
        assert torch.equal(gi, ri) and torch.equal(gc, rc), rep
    q_hat = api.as_predict_query(ctx, p, dev.q_win, dev.q_cur)
    gi2, gc2 = api.as_score_topk(ctx, p, kv, q_hat)
    torch.cuda.synchronize()
    assert torch.equal(gi2, ri) and torch.equal(gc2, rc)
    assert ctx.damaged_workspace_gap(p) == -1
    rq, rs, oidx, ocnt = oracle.select_step(cpu.k_pool, cpu.block_table, cpu.ctx_lens, cpu.q_win, cpu.q_cur, C, f32(1e-2),
                                            agg=agg, sm_scale=p.sm_scale)
    swaps = compare_selection(ri, rc, oidx, ocnt, rs, cpu.ctx_lens, C)
    print(f"  plan {(share, shares, cand)}, tie swaps vs oracle {swaps}", flush=True)


def test_one_launch_form_under_the_static_entry_and_a_wide_block_table():
    """The entry point that allocates nothing takes the same route with the static array's counters; the block table
    is four times wider than the longest sequence, so most workgroups of a row have no pages and only arrive."""
    B, Hq, Hkv, W, C = 2, 8, 2, 8, 128
    w = wl.Workload("srs", B, Hq, Hkv, W, C, 2000, ctx_min=700, page_table="scatter", pool_slack=1.3, seed=5)
    cpu = wl.make_inputs(w)
    wide = torch.zeros((B, cpu.block_table.shape[1] * 4), dtype=torch.int32)
    wide[:, :cpu.block_table.shape[1]] = cpu.block_table
    cpu.block_table = wide
    dev = to_dev(cpu)
    p = params_for(cpu)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    ctx = api.Context(p)
    ctx.set_select_mode(1)
    ri, rc = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    torch.cuda.synchronize()
    for rep in range(3):
        gi = torch.empty_like(ri)
        gc = torch.empty_like(rc)
        api.as_select_step_static(p, kv, dev.q_win, dev.q_cur, gi, gc)
        torch.cuda.synchronize()
        assert torch.equal(gi, ri) and torch.equal(gc, rc), rep


def test_two_hundred_launches_back_to_back_leave_the_counters_at_zero():
    """No synchronisation between the launches: each one finds the arrival counters as the previous one left them
    (zero), and every result equals the two-launch reference."""
    B, Hq, Hkv, W, C = 2, 8, 2, 8, 200
    w = wl.Workload("srr", B, Hq, Hkv, W, C, 6000, ctx_min=1500, page_table="scatter", pool_slack=1.3, seed=11)
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    p = params_for(cpu)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    ctx = api.Context(p)
    ctx.set_select_mode(1)
    ri, rc = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    torch.cuda.synchronize()
    ctx.set_select_mode(0)
    outs = [(torch.empty_like(ri), torch.empty_like(rc)) for _ in range(200)]
    for gi, gc in outs:
        api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur, gi, gc)
    torch.cuda.synchronize()
    for n, (gi, gc) in enumerate(outs):
        assert torch.equal(gi, ri) and torch.equal(gc, rc), n


@pytest.mark.parametrize("shape", [
    (1, 8, 2, 8, 256, 4096, None, 12),      # workload c1, twelve layers per launch
    (1, 32, 8, 16, 2048, 16384, None, 4),   # workload c2, four layers per launch
    (3, 32, 2, 8, 100, 5000, 1, 3),         # groups of 16 heads, ragged, three layers
    (2, 8, 2, 4, 64, 3000, 0, 5),           # empty sequences in every layer
])
def test_packed_one_launch_equals_the_packed_fused_kernels(shape):
    """as_select_step_pack over few rows: the rows of all layers of the pack share one grid and one set of arrival
    counters; same selections as the fused kernels over the same pack (development route 2), layer by layer, and as
    single-layer calls."""
    B, Hq, Hkv, W, C, ctx_len, ctx_min, n_layers = shape
    print("select rows pack", shape, flush=True)
    w = wl.Workload("srp", B, Hq, Hkv, W, C, ctx_len, ctx_min=ctx_min, page_table="scatter", pool_slack=1.3, seed=C + n_layers)
    cpus = [wl.make_inputs(w, layer=l) for l in range(n_layers)]
    if ctx_min == 0:
        for c in cpus:
            c.ctx_lens[0] = 0
    devs = [to_dev(c) for c in cpus]
    p = params_for(cpus[0])
    kvs = [api.kv_view(d.k_pool, d.v_pool, d.block_table, d.ctx_lens) for d in devs]

    def run(ctx):
        sel = [(torch.empty((B, Hkv, C), dtype=torch.int32, device="cuda"),
                torch.empty((B, Hkv), dtype=torch.int32, device="cuda")) for _ in range(n_layers)]
        api.as_select_step_pack(ctx, p, [api.layer_io(kvs[l], devs[l].q_win, devs[l].q_cur, sel[l][0], sel[l][1])
                                         for l in range(n_layers)])
        torch.cuda.synchronize()
        return sel

    ctx_fused = api.Context(p, pack=n_layers)
    ctx_fused.set_select_mode(2)
    ref = run(ctx_fused)
    ctx = api.Context(p, pack=n_layers)
    for rep in range(3):
        got = run(ctx)
        for l in range(n_layers):
            assert torch.equal(got[l][0], ref[l][0]) and torch.equal(got[l][1], ref[l][1]), (rep, l)
    assert ctx.damaged_workspace_gap(p, n_layers) == -1
    assert ctx_fused.damaged_workspace_gap(p, n_layers) == -1
    single = api.Context(p)
    for l in range(n_layers):
        si, sc = api.as_select_step(single, p, kvs[l], devs[l].q_win, devs[l].q_cur)
        assert torch.equal(si, ref[l][0]) and torch.equal(sc, ref[l][1]), l
