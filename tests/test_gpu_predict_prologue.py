"""The predictor inside the prologue of the fused selection kernel (a per-ctx development mode; the default is a
launch of its own): same selections, bit for bit, as the two-launch form, for windows of 1..16 queries, groups of
1..16 heads, rows with one and with several shares, packed launches, both predictor variants and both softmax
signs; and against the oracle."""
import pytest
import torch

import oracle
from paper_2510_07486_amd import api
from paper_2510_07486_amd import workloads as wl
from gpu_common import f32, params_for, to_dev
from helpers import compare_selection

pytestmark = pytest.mark.gpu

CASES = [
    # batch, Hq, Hkv, W, budget, ctx, ctx_min, predictor, beta, agg
    (40, 32, 8, 16, 256, 6000, 100, 0, 1.0, 0),     # one share per row
    (2, 32, 8, 16, 512, 20000, 9000, 0, 1.0, 0),    # several shares per row: every share predicts for itself
    (3, 16, 1, 5, 128, 9000, 4000, 1, 1.0, 0),      # group of 16 (two operand sets), single-solve weights
    (4, 12, 12, 1, 64, 5000, 2000, 0, -1.0, 0),     # MHA, window of one query, the other softmax sign
    (6, 24, 4, 11, 300, 7000, 1, 1, -1.0, 1),       # sum aggregation, ragged down to one token
    (2, 48, 2, 8, 100, 3000, 500, 0, 1.0, 1),       # sum aggregation over groups of 24 heads: more than the prologue holds, so the
                                                    # predictor stays a launch of its own whatever the mode says
]


@pytest.mark.parametrize("case", CASES)
def test_predictor_in_the_selection_prologue_equals_the_two_launch_form(case):
    B, Hq, Hkv, W, C, ctx_len, ctx_min, pred, beta, agg = case
    print("prologue", case, flush=True)
    w = wl.Workload("pp", B, Hq, Hkv, W, C, ctx_len, ctx_min=ctx_min, page_table="scatter", pool_slack=1.2,
                    rho_range=(0.8, 0.99), seed=W * 100 + Hq)
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    p = params_for(cpu, beta=beta, agg=agg)
    p.predictor = pred
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    ctx, ctx_pack = api.Context(p), api.Context(p, pack=2)     # one workspace layout per ctx
    ctx.set_select_mode(2)                    # the fused kernels, whatever the share plan says
    ref = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    ctx.set_predict_mode(1)
    got = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    torch.cuda.synchronize()
    assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1])
    # the same through a packed launch of two layers (the second with the window rolled by one head)
    qw2, qc2 = dev.q_win.roll(1, dims=1).contiguous(), dev.q_cur.roll(1, dims=1).contiguous()
    outs = []
    for mode in (0, 1):
        ctx_pack.set_predict_mode(mode)
        sel = [(torch.empty_like(ref[0]), torch.empty_like(ref[1])) for _ in range(2)]
        api.as_select_step_pack(ctx_pack, p, [api.layer_io(kv, dev.q_win, dev.q_cur, *sel[0]),
                                         api.layer_io(kv, qw2, qc2, *sel[1])])
        torch.cuda.synchronize()
        outs.append(sel)
    for l in range(2):
        assert torch.equal(outs[0][l][0], outs[1][l][0]) and torch.equal(outs[0][l][1], outs[1][l][1])
    assert torch.equal(outs[1][0][0], ref[0])
    rq, rs, ridx, rcnt = oracle.select_step(cpu.k_pool, cpu.block_table, cpu.ctx_lens, cpu.q_win, cpu.q_cur, C, f32(1e-2),
                                            beta=beta, agg=agg, single_solve=bool(pred))
    swaps = compare_selection(got[0], got[1], ridx, rcnt, rs, cpu.ctx_lens, C)
    print(f"  tie swaps vs oracle {swaps}", flush=True)
    assert ctx.damaged_workspace_gap(p) == -1 and ctx_pack.damaged_workspace_gap(p, 2) == -1
