"""Rows that the fused selection cuts into several shares: merged inside the selection kernel by the last workgroup
of the row to arrive (the default) or by a second launch (per-ctx development mode).  Both must give the same
selections, bit for bit, on every launch: 1024- and 512-thread shapes, max / softmax-sum aggregation, packs, ragged
batches with empty sequences (empty shares arrive too), many shares per row; and the arrival counters must be back at
zero after every launch (a second launch on the same ctx works)."""
import pytest
import torch

import oracle
from paper_2510_07486_amd import api
from paper_2510_07486_amd import workloads as wl
from gpu_common import f32, params_for, to_dev
from helpers import compare_selection

pytestmark = pytest.mark.gpu

CASES = [
    # batch, Hq, Hkv, W, budget, ctx, ctx_min, agg, pack
    (2, 32, 8, 16, 512, 20000, 9000, 0, 1),      # a few shares per row, 1024-thread workgroups
    (1, 8, 2, 8, 256, 4096, None, 0, 1),         # workload c1: 13 short shares per row
    (3, 24, 1, 8, 80, 30000, 1, 0, 1),           # group of 24 heads: the 512-thread shape (its buffer holds 4096 candidates); ragged
    (3, 24, 1, 8, 300, 30000, 1, 0, 1),          # ... and a row with more candidates than that buffer: the merge launch either way
    (2, 16, 4, 8, 256, 12000, 3000, 2, 1),       # softmax-normalised aggregation: two passes, merge after the second
    (2, 8, 2, 8, 200, 9000, 2000, 0, 3),         # a pack of three layers: counters are indexed over the pack's rows
    (5, 8, 2, 4, 128, 6000, 0, 1, 1),            # sum aggregation; sequences of length 0: every share of theirs is empty
]


@pytest.mark.parametrize("case", CASES)
def test_merge_inside_the_selection_kernel_equals_the_merge_launch(case):
    B, Hq, Hkv, W, C, ctx_len, ctx_min, agg, pack = case
    print("merge modes", case, flush=True)
    w = wl.Workload("mm", B, Hq, Hkv, W, C, ctx_len, ctx_min=ctx_min, page_table="scatter", pool_slack=1.2, seed=C + B)
    cpu = wl.make_inputs(w)
    if ctx_min == 0:
        cpu.ctx_lens[0] = 0
        cpu.ctx_lens[B - 1] = 0
    dev = to_dev(cpu)
    p = params_for(cpu, agg=agg)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    ctx = api.Context(p, pack=pack)
    ctx.set_select_mode(2)                                   # the fused kernels, whatever the share plan says
    share, shares, cand = api.select_plan(p, pack)
    assert shares > 1, "the case must cut its rows into shares"

    def run():
        if pack == 1:
            return [api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)]
        sel = [(torch.empty((B, Hkv, C), dtype=torch.int32, device="cuda"), torch.empty((B, Hkv), dtype=torch.int32, device="cuda"))
               for _ in range(pack)]
        qs = [(dev.q_win.roll(l, dims=1).contiguous(), dev.q_cur.roll(l, dims=1).contiguous()) for l in range(pack)]
        api.as_select_step_pack(ctx, p, [api.layer_io(kv, qs[l][0], qs[l][1], *sel[l]) for l in range(pack)])
        return sel

    ctx.set_merge_mode(1)
    ref = run()
    torch.cuda.synchronize()
    ctx.set_merge_mode(0)
    for rep in range(6):                                     # counters return to zero: every repetition is a fresh count
        got = run()
        torch.cuda.synchronize()
        for (gi, gc), (ri, rc) in zip(got, ref):
            assert torch.equal(gi, ri) and torch.equal(gc, rc), rep
    rq, rs, ridx, rcnt = oracle.select_step(cpu.k_pool, cpu.block_table, cpu.ctx_lens, cpu.q_win, cpu.q_cur, C, f32(1e-2),
                                            agg=agg, sm_scale=p.sm_scale)
    swaps = compare_selection(ref[0][0], ref[0][1], ridx, rcnt, rs, cpu.ctx_lens, C)
    threads = 512 if (Hq // Hkv > 16 and agg != 1) else 1024
    in_kernel = shares * cand <= 8 * threads and shares <= threads // 4
    print(f"  plan {(share, shares, cand)}, merged in the kernel: {in_kernel}, tie swaps vs oracle {swaps}", flush=True)
