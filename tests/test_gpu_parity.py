"""GPU parity: every stage of the HIP path against the CPU oracle on the same seeded inputs,
stage-isolated (each stage fed the oracle's previous-stage output) and end to end, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_07486_amd import api
from paper_2510_07486_amd import workloads as wl
from gpu_common import SCALE, SCORE_REL_ABSDOT, absdot_bound, f32, params_for, to_dev
from helpers import compare_selection

pytestmark = pytest.mark.gpu

Q_HAT_TOL = 2e-2       # spec bound (max-abs) for predicted queries and attention outputs
OUT_TOL = 2e-2


def note(*a):
    print(*a, flush=True)


# --------------------------------------------------------------------------- predictor
@pytest.mark.parametrize("W", [1, 2, 5, 8, 16, 33, 64])
@pytest.mark.parametrize("eps,beta", [(1e-2, 1.0), (1e-4, 1.0), (1.0, -1.0)])
def test_predict_matches_oracle(W, eps, beta):
    note("predict", W, eps, beta)
    w = wl.Workload("p", 3, 8, 2, W, 16, 64, rho_range=(0.8, 0.99), seed=W)
    qw, qc, _ = wl.make_queries(w)
    ref = oracle.predict_query(qw, qc, f32(eps), beta)
    p = api.make_params(3, 8, 2, W, 16, 4, ridge_eps=f32(eps), softmax_beta=beta)
    ctx = api.Context(p)
    got = api.as_predict_query(ctx, p, qw.cuda(), qc.cuda()).cpu()
    err = (got - ref).abs().max().item()
    note("  max abs err", err)
    assert err <= Q_HAT_TOL
    # fp64 inside on both sides: in practice they agree to fp32 rounding
    assert err <= 2e-6 * max(1.0, ref.abs().max().item())
    if W == 1:
        assert torch.equal(got, qc.float())


@pytest.mark.parametrize("W", [1, 2, 5, 8, 16, 33, 64])
@pytest.mark.parametrize("eps,beta", [(1e-2, 1.0), (1e-3, -1.0)])
def test_single_solve_predictor_matches_oracle(W, eps, beta):
    """Alg. 1 steps 3-5: one ridge solve over the whole window, truncated and renormalised per window size."""
    note("predict single-solve", W, eps, beta)
    w = wl.Workload("p", 3, 8, 2, W, 16, 64, rho_range=(0.8, 0.99), seed=100 + W)
    qw, qc, _ = wl.make_queries(w)
    ref = oracle.predict_query(qw, qc, f32(eps), beta, single_solve=True)
    p = api.make_params(3, 8, 2, W, 16, 4, ridge_eps=f32(eps), softmax_beta=beta, predictor=api.AS_PRED_SINGLE_SOLVE)
    ctx = api.Context(p)
    got = api.as_predict_query(ctx, p, qw.cuda(), qc.cuda()).cpu()
    err = (got - ref).abs().max().item()
    assert err <= 2e-6 * max(1.0, ref.abs().max().item())
    if W > 2:      # and it is a different predictor from the per-window-size one
        other = oracle.predict_query(qw, qc, f32(eps), beta)
        assert (other - ref).abs().max().item() > 1e-5


# --------------------------------------------------------------------------- scoring
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (8, 8), (16, 2), (4, 2), (32, 2), (6, 2), (1, 1), (32, 1), (48, 2), (64, 1),
                                    (128, 2)])
@pytest.mark.parametrize("agg", [0, 1])
def test_score_matches_oracle(Hq, Hkv, agg):
    note("score", Hq, Hkv, agg)
    w = wl.Workload("s", 3, Hq, Hkv, 4, 16, 1100, ctx_min=1, n_outlier=4, page_table="scatter", pool_slack=1.3,
                    seed=Hq * 10 + Hkv)
    cpu = wl.make_inputs(w)
    cpu.ctx_lens[0] = 1100          # full length, last page partial (1100 = 68*16 + 12)
    cpu.ctx_lens[1] = 17
    dev = to_dev(cpu)
    g = torch.Generator().manual_seed(5)
    q_hat = torch.randn((3, Hq, 128), generator=g)
    ref = oracle.score_keys(cpu.k_pool, cpu.block_table, cpu.ctx_lens, q_hat, Hkv, agg, fill=-7.0)
    p = params_for(cpu, agg=agg)
    ctx = api.Context(p)
    got = api.as_score_keys(ctx, p, api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens),
                            q_hat.cuda(), fill=-7.0).cpu()
    bound = SCORE_REL_ABSDOT * absdot_bound(cpu, q_hat) + 1e-30
    for b in range(3):
        n = int(cpu.ctx_lens[b])
        d = (got[b, :, :n].double() - ref[b, :, :n].double()).abs()
        assert (d <= bound[b, :, :n]).all(), (b, d.max().item())
        assert (got[b, :, n:] == -7.0).all()          # nothing written past the context
    assert not (got.view(torch.int32) == -2147483648).any()   # no -0 escapes


def test_score_page_permutation_invariance():
    w = wl.Workload("s", 2, 8, 2, 4, 16, 500, page_table="identity", seed=9)
    cpu = wl.make_inputs(w)
    q_hat = torch.randn((2, 8, 128), generator=torch.Generator().manual_seed(1)).cuda()
    p = params_for(cpu)
    ctx = api.Context(p)
    dev = to_dev(cpu)
    a = api.as_score_keys(ctx, p, api.kv_view(dev.k_pool, None, dev.block_table, dev.ctx_lens), q_hat, fill=0.0)
    perm = torch.randperm(cpu.num_pages, generator=torch.Generator().manual_seed(2))
    inv = torch.empty_like(perm); inv[perm] = torch.arange(cpu.num_pages)
    k2 = cpu.k_pool[perm].contiguous().cuda()
    bt2 = inv[cpu.block_table.long()].to(torch.int32).cuda()
    b = api.as_score_keys(ctx, p, api.kv_view(k2, None, bt2, dev.ctx_lens), q_hat, fill=0.0)
    assert torch.equal(a, b)


# --------------------------------------------------------------------------- top-k
def topk_case(rows: np.ndarray, lens, C):
    s = torch.tensor(rows, dtype=torch.float32)            # [B, H, N]
    B, H, N = s.shape
    lens_t = torch.tensor(lens, dtype=torch.int32)
    ri, rc = oracle.topk_select(s, lens_t, C)
    p = api.make_params(B, H, H, 1, C, (N + 15) // 16 if N % 16 == 0 else N // 16 + 1)
    stride_needed = p.max_pages_per_seq * 16
    if stride_needed > N:
        s = torch.nn.functional.pad(s, (0, stride_needed - N), value=float("nan"))
    ctx = api.Context(p)
    gi, gc = api.as_topk_select(ctx, p, s.cuda(), lens_t.cuda())
    assert torch.equal(gc.cpu(), rc)
    assert torch.equal(gi.cpu(), ri)


@pytest.mark.parametrize("N,C", [(16, 4), (1000, 37), (4096, 256), (5000, 5000), (5000, 4999), (33000, 2048),
                                 (70000, 4096), (70000, 65536)])
def test_topk_bit_exact_random_and_ties(N, C):
    note("topk", N, C)
    rng = np.random.default_rng(N + C)
    rows = rng.standard_normal((2, 3, N)).astype(np.float32)
    rows[0, 1] = np.round(rows[0, 1] * 4) / 4                  # heavy exact ties
    rows[1, 0] = 1.5                                           # all equal: lowest indices win
    rows[1, 1, ::3] = -0.0
    rows[1, 1, 1::3] = 0.0                                      # signed zeros tie
    rows[1, 2] = np.abs(rows[1, 2]) * 1e-39                     # subnormals
    topk_case(rows, [N, max(1, N - 7)], C)


def test_topk_special_values_and_short_rows():
    rows = np.zeros((3, 1, 64), dtype=np.float32)
    rows[0, 0, :8] = [np.nan, -np.inf, np.inf, 1.0, -1.0, np.nan, 3e38, -3e38]
    rows[1, 0] = np.arange(64)
    rows[2, 0] = -np.arange(64)
    topk_case(rows, [64, 5, 0], 6)        # ctx 5 < C and an empty sequence


# --------------------------------------------------------------------------- attention
def attn_case(w, sel="topk", tail=None, budget=None):
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    C = budget or w.budget
    q_hat = oracle.predict_query(cpu.q_win, cpu.q_cur, f32(1e-2))
    sc = oracle.score_keys(cpu.k_pool, cpu.block_table, cpu.ctx_lens, q_hat, w.n_kv_heads)
    lens_sel = cpu.ctx_lens.clone() if tail is None else torch.clamp(cpu.ctx_lens - tail, min=0)
    idx, cnt = oracle.topk_select(sc, lens_sel, C)
    sel_ctx = None if tail is None else lens_sel
    ref, ref_lse = oracle.sparse_decode_attn(cpu.k_pool, cpu.v_pool, cpu.block_table, cpu.ctx_lens, cpu.q_real,
                                             idx, cnt, f32(SCALE), sel_ctx)
    p = params_for(cpu, budget=C)
    ctx = api.Context(p)
    out, lse = api.as_sparse_decode_attn(ctx, p, api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens),
                                         dev.q_real, idx.cuda(), cnt.cuda(),
                                         None if sel_ctx is None else sel_ctx.cuda())
    err = (out.cpu().float() - ref.float()).abs().max().item()
    note("  attn max abs err", err)
    assert err <= OUT_TOL
    fin = torch.isfinite(ref_lse)
    assert torch.equal(torch.isfinite(lse.cpu()), fin)
    assert (lse.cpu()[fin] - ref_lse[fin]).abs().max().item() <= 1e-3 if fin.any() else True
    assert (out.cpu()[~fin].float() == 0).all()
    return err


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (16, 2), (4, 4), (6, 2), (32, 2), (32, 1), (48, 2), (128, 2)])
def test_attn_matches_oracle(Hq, Hkv):
    note("attn", Hq, Hkv)
    w = wl.Workload("a", 3, Hq, Hkv, 4, 300, 2000, ctx_min=100, page_table="scatter", pool_slack=1.2, seed=Hq + Hkv)
    attn_case(w)


def test_attn_budget_above_context_and_tail_and_empty():
    w = wl.Workload("a", 4, 8, 2, 4, 700, 600, ctx_min=1, page_table="scatter", pool_slack=1.2, seed=21)
    attn_case(w)                       # budget 700 > every context: dense attention
    attn_case(w, tail=1)               # own-token tail
    attn_case(w, tail=450, budget=64)  # long dense tail handled by the last split's loop
    w0 = wl.scaled(w, ctx=40, ctx_min=1)
    cpu = wl.make_inputs(w0)
    cpu.ctx_lens[0] = 0                # empty sequence: out = 0, lse = -inf
    dev = to_dev(cpu)
    idx = torch.full((4, 2, 16), -1, dtype=torch.int32)
    cnt = torch.zeros((4, 2), dtype=torch.int32)
    p = params_for(cpu, budget=16)
    ctx = api.Context(p)
    out, lse = api.as_sparse_decode_attn(ctx, p, api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens),
                                         dev.q_real, idx.cuda(), cnt.cuda())
    assert (out.float() == 0).all() and torch.isinf(lse).all()


def test_attn_single_token_returns_value_row():
    w = wl.Workload("a", 2, 8, 2, 4, 8, 64, seed=4)
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    idx = torch.full((2, 2, 8), -1, dtype=torch.int32)
    idx[:, :, 0] = torch.tensor([[3, 40], [63, 0]], dtype=torch.int32)
    cnt = torch.ones((2, 2), dtype=torch.int32)
    p = params_for(cpu)
    ctx = api.Context(p)
    out, _ = api.as_sparse_decode_attn(ctx, p, api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens),
                                       dev.q_real, idx.cuda(), cnt.cuda())
    ref, _ = oracle.sparse_decode_attn(cpu.k_pool, cpu.v_pool, cpu.block_table, cpu.ctx_lens, cpu.q_real, idx, cnt,
                                       f32(SCALE))
    assert torch.equal(out.cpu(), ref)         # softmax over one token is exactly 1


# --------------------------------------------------------------------------- end to end
def end_to_end(w, eps=1e-2, beta=1.0, agg=0, streams=False, single_solve=False):
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    q_hat, sc, ridx, rcnt = oracle.select_step(cpu.k_pool, cpu.block_table, cpu.ctx_lens, cpu.q_win, cpu.q_cur,
                                               w.budget, f32(eps), beta, agg, single_solve=single_solve)
    p = params_for(cpu, eps=eps, beta=beta, agg=agg)
    p.predictor = api.AS_PRED_SINGLE_SOLVE if single_solve else api.AS_PRED_PER_WINDOW
    ctx = api.Context(p)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    gidx, gcnt = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    swaps = compare_selection(gidx, gcnt, ridx, rcnt, sc, cpu.ctx_lens, w.budget)
    out, lse = api.as_sparse_decode_attn(ctx, p, kv, dev.q_real, gidx, gcnt)
    # the oracle attends over the GPU's own selection so that tie swaps do not enter the comparison
    ref, ref_lse = oracle.sparse_decode_attn(cpu.k_pool, cpu.v_pool, cpu.block_table, cpu.ctx_lens, cpu.q_real,
                                             gidx.cpu(), gcnt.cpu(), f32(SCALE))
    err = (out.cpu().float() - ref.float()).abs().max().item()
    note(f"  {w.name}: tie swaps {swaps}, attn max abs err {err:.3e}")
    assert err <= OUT_TOL
    return swaps, (gidx, gcnt, out)


def fused_vs_separate(w):
    """as_select_step's fused scoring + top-k against the separate kernels: identical index sets, whichever of the
    two the library would pick for the shape by itself."""
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    p = params_for(cpu)
    ctx = api.Context(p)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    a_idx, a_cnt = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)       # the library's own choice
    ctx.set_select_mode(1)                                                    # always the stand-alone stages
    b_idx, b_cnt = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    ctx.set_select_mode(2)                                                    # always the fused kernels
    f_idx, f_cnt = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    assert torch.equal(a_cnt, b_cnt) and torch.equal(a_cnt, f_cnt)
    assert torch.equal(a_idx, b_idx) and torch.equal(a_idx, f_idx)
    # stage-isolated: the fused kernel fed the oracle's q_hat reproduces the oracle's selection of its own scores
    q_hat = oracle.predict_query(cpu.q_win, cpu.q_cur, f32(1e-2))
    sc = oracle.score_keys(cpu.k_pool, cpu.block_table, cpu.ctx_lens, q_hat, w.n_kv_heads)
    ridx, rcnt = oracle.topk_select(sc, cpu.ctx_lens, w.budget)
    c_idx, c_cnt = api.as_score_topk(ctx, p, kv, q_hat.cuda())
    swaps = compare_selection(c_idx, c_cnt, ridx, rcnt, sc, cpu.ctx_lens, w.budget)
    ctx.set_select_mode(0)
    d_idx, d_cnt = api.as_score_topk(ctx, p, kv, q_hat.cuda())
    assert torch.equal(c_idx, d_idx) and torch.equal(c_cnt, d_cnt)
    note("  tie swaps vs oracle:", swaps, " share plan", api.select_plan(p, 1))


@pytest.mark.parametrize("kw", [
    dict(batch=64, n_q_heads=32, n_kv_heads=8, ctx=1000, ctx_min=1, budget=300),     # one slice per row
    dict(batch=64, n_q_heads=32, n_kv_heads=8, ctx=1000, ctx_min=1, budget=2048),    # budget above every context
    dict(batch=2, n_q_heads=8, n_kv_heads=2, ctx=5000, ctx_min=3000, budget=700),    # many short slices
    dict(batch=40, n_q_heads=16, n_kv_heads=8, ctx=20000, ctx_min=15000, budget=2048),  # long slices, two per row
    dict(batch=9, n_q_heads=64, n_kv_heads=4, ctx=3333, ctx_min=100, budget=64),     # group of 16
    dict(batch=5, n_q_heads=32, n_kv_heads=1, ctx=9000, ctx_min=3000, budget=512),   # MQA, 32 heads on one KV head
    dict(batch=3, n_q_heads=128, n_kv_heads=2, ctx=6000, ctx_min=500, budget=300),   # groups of 64
    dict(batch=2, n_q_heads=48, n_kv_heads=2, ctx=2000, ctx_min=900, budget=100),    # group of 24 (not a power of two)
    dict(batch=1, n_q_heads=8, n_kv_heads=2, ctx=4096, budget=256),      # few rows: shares no longer than the budget,
    dict(batch=1, n_q_heads=32, n_kv_heads=8, ctx=16384, budget=2048),   # which the library runs as separate stages
    dict(batch=1, n_q_heads=8, n_kv_heads=2, ctx=40000, budget=9000),    # budget above the pruning limit: buffer-sized
                                                                         # shares, merge over global candidates
])
def test_fused_select_equals_separate_kernels(kw):
    note("fused-vs-separate", kw)
    fused_vs_separate(wl.Workload("f", window=8, page_table="scatter", pool_slack=1.1, seed=17, **kw))


def test_end_to_end_single_slice_rows_and_long_slices():
    end_to_end(wl.Workload("f1", 64, 32, 8, 16, 300, 1000, ctx_min=1, page_table="scatter", pool_slack=1.1, seed=5))
    end_to_end(wl.Workload("f2", 33, 32, 8, 16, 2048, 20000, ctx_min=9000, page_table="permute", seed=6))


def test_end_to_end_c1():
    end_to_end(wl.CONFIGS["c1"])


def test_end_to_end_c2_full_size():
    end_to_end(wl.CONFIGS["c2"])


@pytest.mark.parametrize("name,kw", [
    ("c3", dict(batch=3, ctx=4096, budget=512)),
    ("c4", dict(batch=2, ctx=4096, budget=1024)),
    ("c5", dict(batch=6, ctx=8192, ctx_min=1000, budget=1024)),
    ("c5", dict(batch=4, ctx=3000, ctx_min=500, budget=4096)),      # budget above every context
])
def test_end_to_end_scaled_configs(name, kw):
    note("e2e", name, kw)
    end_to_end(wl.scaled(wl.CONFIGS[name], layers=1, **kw))


@pytest.mark.parametrize("agg,beta", [(1, 1.0), (0, -1.0)])
def test_end_to_end_variants(agg, beta):
    end_to_end(wl.scaled(wl.CONFIGS["c2"], ctx=4096, budget=256), agg=agg, beta=beta)


def test_end_to_end_mqa_groups():
    # multi-query layouts of the paper's batched-matmul figure: every query head on one KV head
    end_to_end(wl.Workload("mqa32", 4, 32, 1, 16, 512, 8192, ctx_min=2000, page_table="scatter", pool_slack=1.2, seed=61))
    end_to_end(wl.Workload("mqa64", 2, 64, 1, 16, 256, 5000, ctx_min=2000, page_table="permute", seed=62), agg=1)
    end_to_end(wl.Workload("gqa64", 2, 128, 2, 8, 384, 4000, ctx_min=100, page_table="scatter", pool_slack=1.1, seed=63))


def test_end_to_end_single_solve_predictor():
    end_to_end(wl.scaled(wl.CONFIGS["c2"], ctx=4096, budget=256), single_solve=True)
    end_to_end(wl.scaled(wl.CONFIGS["c1"], ctx=2048, budget=128), beta=-1.0, single_solve=True)   # Alg. 1's sign too


def test_two_stream_overlap_equals_serial():
    """Selection on its own stream, overlapped with the previous layer's attention on another,
    event hand-off: results are bit-identical to the single-stream order."""
    w = wl.scaled(wl.CONFIGS["c3"], batch=4, ctx=8192, budget=512, layers=1)
    layers = [to_dev(wl.make_inputs(w, layer=l)) for l in range(3)]
    p = params_for(layers[0])
    ctx_sel, ctx_att = api.Context(p), api.Context(p)
    kvs = [api.kv_view(x.k_pool, x.v_pool, x.block_table, x.ctx_lens) for x in layers]

    def serial():
        outs = []
        for l, x in enumerate(layers):
            idx, cnt = api.as_select_step(ctx_sel, p, kvs[l], x.q_win, x.q_cur)
            outs.append((idx.clone(), api.as_sparse_decode_attn(ctx_att, p, kvs[l], x.q_real, idx, cnt)[0].clone()))
        torch.cuda.synchronize()
        return outs

    ref = serial()
    s_sel, s_att = torch.cuda.Stream(), torch.cuda.Stream()
    sel = [(torch.empty((w.batch, w.n_kv_heads, w.budget), dtype=torch.int32, device="cuda"),
            torch.empty((w.batch, w.n_kv_heads), dtype=torch.int32, device="cuda")) for _ in layers]
    outs = [torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.bfloat16, device="cuda") for _ in layers]
    torch.cuda.synchronize()
    evs = []
    for l, x in enumerate(layers):                      # all selections queue on the SEL stream
        api.as_select_step(ctx_sel, p, kvs[l], x.q_win, x.q_cur, sel[l][0], sel[l][1], stream=s_sel)
        ev = torch.cuda.Event(); ev.record(s_sel); evs.append(ev)
    for l, x in enumerate(layers):                      # attention of layer l waits only for its own selection
        s_att.wait_event(evs[l])
        api.as_sparse_decode_attn(ctx_att, p, kvs[l], x.q_real, sel[l][0], sel[l][1], out=outs[l], stream=s_att,
                                  want_lse=False)
    torch.cuda.synchronize()
    for l in range(3):
        assert torch.equal(sel[l][0], ref[l][0])
        assert torch.equal(outs[l], ref[l][1])


def test_select_is_invariant_to_query_scaling_and_constant_window():
    # positive scaling of every query leaves the selection unchanged; a constant query sequence predicts itself
    w = wl.scaled(wl.CONFIGS["c1"], ctx=2048, budget=128)
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    p = params_for(cpu)
    ctx = api.Context(p)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    const_win = dev.q_cur[:, :, None, :].expand(-1, -1, w.window, -1).contiguous()
    q_hat = api.as_predict_query(ctx, p, const_win, dev.q_cur)
    assert (q_hat - dev.q_cur.float()).abs().max().item() <= 1e-6 * dev.q_cur.float().abs().max().item()
    a, _ = api.as_select_step(ctx, p, kv, const_win, dev.q_cur)
    sc = api.as_score_keys(ctx, p, kv, dev.q_cur.float().contiguous())
    b, _ = api.as_topk_select(ctx, p, sc, dev.ctx_lens)
    ref = oracle.topk_select(sc.cpu(), cpu.ctx_lens, w.budget)[0]
    assert torch.equal(b.cpu(), ref)
    overlap = np.mean([len(np.intersect1d(a[0, j].cpu().numpy(), b[0, j].cpu().numpy())) / w.budget
                       for j in range(w.n_kv_heads)])
    note("  overlap ratio (Eq. 1), constant window:", overlap)
    assert overlap >= 0.99


# --------------------------------------------------------------------------- softmax-normalised aggregation
def softmax_sum_case(w, n_layers=1, eps=1e-2):
    """Selection with agg = AS_AGG_SOFTMAX_SUM (two passes over K) against the oracle's selection of its own
    softmax-normalised scores, through as_select_step (or the packed call)."""
    cpus = [wl.make_inputs(w, layer=l) for l in range(n_layers)]
    devs = [to_dev(c) for c in cpus]
    p = params_for(cpus[0], eps=eps, agg=api.AS_AGG_SOFTMAX_SUM)
    ctx = api.Context(p, pack=n_layers)
    kvs = [api.kv_view(d.k_pool, d.v_pool, d.block_table, d.ctx_lens) for d in devs]
    if n_layers == 1:
        got = [api.as_select_step(ctx, p, kvs[0], devs[0].q_win, devs[0].q_cur)]
    else:
        B, Hkv, C = w.batch, w.n_kv_heads, w.budget
        got = [(torch.empty((B, Hkv, C), dtype=torch.int32, device="cuda"),
                torch.empty((B, Hkv), dtype=torch.int32, device="cuda")) for _ in range(n_layers)]
        api.as_select_step_pack(ctx, p, [api.layer_io(kvs[l], devs[l].q_win, devs[l].q_cur, got[l][0], got[l][1])
                                         for l in range(n_layers)])
    torch.cuda.synchronize()
    swaps = 0
    for l, c in enumerate(cpus):
        q_hat, sc, ridx, rcnt = oracle.select_step(c.k_pool, c.block_table, c.ctx_lens, c.q_win, c.q_cur, w.budget,
                                                   f32(eps), agg=2, sm_scale=f32(SCALE))
        swaps += compare_selection(got[l][0], got[l][1], ridx, rcnt, sc, c.ctx_lens, w.budget)
    note(f"  softmax-sum {w.name}: plan {api.select_plan(p, n_layers)}, tie swaps {swaps}")


@pytest.mark.parametrize("kw", [
    dict(batch=40, n_q_heads=32, n_kv_heads=8, ctx=3000, ctx_min=1, budget=256),        # one share per row
    dict(batch=2, n_q_heads=8, n_kv_heads=2, ctx=9000, ctx_min=5000, budget=700),       # rows cut into many shares
    dict(batch=3, n_q_heads=4, n_kv_heads=4, ctx=2500, ctx_min=700, budget=64),         # G = 1
    dict(batch=3, n_q_heads=32, n_kv_heads=2, ctx=2000, ctx_min=100, budget=128),       # G = 16: two operand sets
    dict(batch=2, n_q_heads=48, n_kv_heads=2, ctx=1500, ctx_min=300, budget=100),       # G = 24: four sets, 512 threads
    dict(batch=2, n_q_heads=64, n_kv_heads=1, ctx=1200, ctx_min=600, budget=2048),      # G = 64, budget above context
])
def test_softmax_sum_aggregation_matches_oracle(kw):
    note("softmax-sum", kw)
    softmax_sum_case(wl.Workload("ss", window=8, page_table="scatter", pool_slack=1.2, seed=71, **kw))


def test_softmax_sum_long_single_share_rows_and_pack():
    # 256 rows of 20000 tokens: one share per row, several prunes, as in the benchmark's launch shape
    softmax_sum_case(wl.Workload("ssl", 32, 32, 8, 16, 2048, 20000, ctx_min=12000, page_table="permute", seed=72))
    softmax_sum_case(wl.Workload("ssp", 1, 8, 2, 8, 256, 4096, page_table="identity", seed=73), n_layers=3)


def test_softmax_sum_is_rejected_by_the_stand_alone_scoring_call():
    w = wl.Workload("sr", 1, 8, 2, 4, 16, 64, seed=1)
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    p = params_for(cpu, agg=api.AS_AGG_SOFTMAX_SUM)
    ctx = api.Context(p)
    with pytest.raises(api.AsError) as e:
        api.as_score_keys(ctx, p, api.kv_view(dev.k_pool, None, dev.block_table, dev.ctx_lens),
                          torch.zeros((1, 8, 128), device="cuda"))
    assert e.value.code == 2


def test_predicted_query_beats_the_current_one_when_queries_regress_on_lag_two():
    """The point of the predictor (Sec. 3 Eq. 1, Sec. 4.2): when the next query depends on the window beyond its last
    entry, selecting with q_hat overlaps the real next query's selection more than selecting with Q_t does.  On AR(1)
    chains Q_t is already the best guess; on an AR(2) process with a dominant lag-two coefficient it is not.  Both
    ratios come out of the HIP path and are cross-checked against the oracle's."""
    w = wl.Workload("lag2", 4, 8, 2, 16, 256, 4096, page_table="permute", seed=5, lag2=0.85)
    cpu = wl.make_inputs(w)
    dev = to_dev(cpu)
    p = params_for(cpu)
    ctx = api.Context(p)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    hat = api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    real = api.as_score_topk(ctx, p, kv, dev.q_real.float().contiguous())
    cur = api.as_score_topk(ctx, p, kv, dev.q_cur.float().contiguous())
    o_hat = api.as_overlap_ratio(ctx, p, hat[0], hat[1], real[0], real[1])[1].mean().item()
    o_cur = api.as_overlap_ratio(ctx, p, cur[0], cur[1], real[0], real[1])[1].mean().item()
    note(f"  overlap with the real next query's selection: predicted {o_hat:.3f}, current query {o_cur:.3f}")
    assert o_hat > o_cur + 0.02

    def oracle_sel(q):
        s = oracle.score_keys(cpu.k_pool, cpu.block_table, cpu.ctx_lens, q.float().contiguous(), w.n_kv_heads)
        return oracle.topk_select(s, cpu.ctx_lens, w.budget)

    _, _, ridx, rcnt = oracle.select_step(cpu.k_pool, cpu.block_table, cpu.ctx_lens, cpu.q_win, cpu.q_cur, w.budget,
                                          f32(1e-2))
    ri, rc = oracle_sel(cpu.q_real)
    ci, cc = oracle_sel(cpu.q_cur)
    ref_hat = oracle.overlap_ratio(ridx, rcnt, ri, rc)[1].mean().item()
    ref_cur = oracle.overlap_ratio(ci, cc, ri, rc)[1].mean().item()
    assert abs(ref_hat - o_hat) <= 2e-3 and abs(ref_cur - o_cur) <= 2e-3      # tie swaps move single tokens at most
