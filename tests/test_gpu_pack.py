"""GPU parity of the depth-wise packed selection (Sec. 4.3, "Depth-wise Parallelism on Cache Rank"):
one as_select_step_pack call over several layers against the oracle's per-layer selection, and bit
for bit against separate as_select_step calls."""
import pytest
import torch

import oracle
from paper_2510_07486_amd import api
from paper_2510_07486_amd import workloads as wl
from gpu_common import f32, params_for, to_dev
from helpers import compare_selection

pytestmark = pytest.mark.gpu


def note(*a):
    print(*a, flush=True)


def run_pack(w, n_layers, shared_table=True, eps=1e-2, agg=0):
    """Layers differ in K, V and queries; the page table and context lengths are shared (as in a
    serving engine) or per layer."""
    cpus = [wl.make_inputs(wl.scaled(w, seed=w.seed + (0 if shared_table else 31 * l)), layer=l)
            for l in range(n_layers)]
    devs = [to_dev(c) for c in cpus]
    if shared_table:
        for d in devs[1:]:
            d.block_table, d.ctx_lens = devs[0].block_table, devs[0].ctx_lens
    p = params_for(cpus[0], eps=eps, agg=agg)
    ctx = api.Context(p, pack=n_layers)
    kvs = [api.kv_view(d.k_pool, d.v_pool, d.block_table, d.ctx_lens) for d in devs]
    B, Hkv, C = w.batch, w.n_kv_heads, w.budget
    sel = [(torch.full((B, Hkv, C), -7, dtype=torch.int32, device="cuda"),
            torch.full((B, Hkv), -7, dtype=torch.int32, device="cuda")) for _ in range(n_layers)]
    ios = [api.layer_io(kvs[l], devs[l].q_win, devs[l].q_cur, sel[l][0], sel[l][1]) for l in range(n_layers)]
    api.as_select_step_pack(ctx, p, ios)
    torch.cuda.synchronize()
    plan = api.select_plan(p, n_layers)
    swaps = 0
    for l in range(n_layers):
        c = cpus[l]
        q_hat, sc, ridx, rcnt = oracle.select_step(c.k_pool, c.block_table, c.ctx_lens, c.q_win, c.q_cur, C, f32(eps),
                                                   1.0, agg)
        swaps += compare_selection(sel[l][0], sel[l][1], ridx, rcnt, sc, c.ctx_lens, C)
        one_idx, one_cnt = api.as_select_step(ctx, p, kvs[l], devs[l].q_win, devs[l].q_cur)
        assert torch.equal(one_cnt, sel[l][1]), l
        assert torch.equal(one_idx, sel[l][0]), l
    note(f"  pack of {n_layers}: plan (share, shares/row, cand) = {plan}, tie swaps vs oracle {swaps}")
    return plan


@pytest.mark.parametrize("n_layers", [1, 3, 16])
def test_pack_matches_oracle_and_single_layer_calls(n_layers):
    note("pack", n_layers)
    w = wl.Workload("pk", 3, 8, 2, 8, 200, 3000, ctx_min=40, page_table="scatter", pool_slack=1.2, seed=11)
    run_pack(w, n_layers)


def test_pack_multi_share_rows_and_per_layer_tables():
    # few rows of a longer context: rows are cut into several shares, candidates of all layers share the workspace
    w = wl.Workload("pk", 1, 8, 2, 16, 256, 9000, ctx_min=5000, page_table="permute", seed=12)
    plan = run_pack(w, 4, shared_table=False)
    assert plan[1] > 1
    # ragged batch with an empty sequence and a group of 16, sum aggregation
    w = wl.Workload("pk", 5, 32, 2, 4, 64, 2500, ctx_min=1, page_table="scatter", pool_slack=1.3, seed=13)
    run_pack(w, 5, agg=1)


def test_pack_c2_shape_pack_of_four():
    # Qwen3-8B head shape at batch 1 (workload c2), context 16384, four layers in one launch
    run_pack(wl.CONFIGS["c2"], 4)


def test_pack_argument_errors():
    w = wl.Workload("pk", 2, 8, 2, 4, 32, 256, seed=3)
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    p = params_for(cpu)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    idx = torch.empty((2, 2, 32), dtype=torch.int32, device="cuda")
    cnt = torch.empty((2, 2), dtype=torch.int32, device="cuda")
    io = api.layer_io(kv, dev.q_win, dev.q_cur, idx, cnt)
    ctx = api.Context(p, pack=2)
    assert api.as_workspace_bytes_pack(p, 0) == 0 and api.as_workspace_bytes_pack(p, api.AS_MAX_PACK + 1) == 0
    with pytest.raises(api.AsError) as e:
        api.as_select_step_pack(ctx, p, [io] * (api.AS_MAX_PACK + 1))
    assert e.value.code == 2                         # unsupported pack size
    with pytest.raises(api.AsError) as e:
        api.as_select_step_pack(ctx, p, [])
    assert e.value.code == 1
    small = api.Context(p, workspace_bytes=256)
    with pytest.raises(api.AsError) as e:
        api.as_select_step_pack(small, p, [io, io])
    assert e.value.code == 3                         # workspace too small
    bad = api.AsLayerIo(kv, None, io.q_cur, io.sel_idx, io.sel_cnt)
    with pytest.raises(api.AsError) as e:
        api.as_select_step_pack(ctx, p, [io, bad])
    assert e.value.code == 1
