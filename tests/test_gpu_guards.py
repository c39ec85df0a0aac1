"""Out-of-bounds writes inside torch's memory pool do not fault, they silently corrupt a neighbour.  Here every
output of every entry point sits between two guard zones filled with a pattern, the inputs are fingerprinted, and
after each call the guards must be intact, the inputs unchanged and the slots the header declares untouched (scores
beyond a sequence's length, padding beyond sel_cnt excepted: that is written as -1) still hold the pattern.  Shapes
are ragged on purpose: lengths that end inside a page, a budget that is no multiple of anything, rows cut into
several shares, group sizes that take the 512-thread selection shape, the dense tail.  The library's own workspace
is checked the same way, through the gaps it keeps between its regions."""
import pytest
import torch

from paper_2510_07486_amd import api
from paper_2510_07486_amd import workloads as wl
from gpu_common import params_for, to_dev

pytestmark = pytest.mark.gpu

PAD = 8192


class Guarded:
    """A contiguous tensor of `shape` in the middle of a larger allocation whose two ends hold a pattern."""

    def __init__(self, shape, dtype, pattern):
        n = 1
        for s in shape:
            n *= s
        self.whole = torch.full((PAD + n + PAD,), pattern, dtype=dtype, device="cuda")
        self.t = self.whole[PAD:PAD + n].view(shape)
        self.pattern = pattern
        self.n = n

    def intact(self):
        w = self.whole
        return bool((w[:PAD] == self.pattern).all()) and bool((w[PAD + self.n:] == self.pattern).all())


def fingerprint(*tensors):
    return [t.view(torch.int16 if t.element_size() == 2 else torch.int32).to(torch.int64).sum().item() for t in tensors]


CASES = [
    dict(batch=3, n_q_heads=8, n_kv_heads=2, window=5, budget=100, ctx=3001, ctx_min=1),       # ragged, short rows
    dict(batch=1, n_q_heads=8, n_kv_heads=2, window=8, budget=333, ctx=20011),                 # one row, many shares
    dict(batch=2, n_q_heads=48, n_kv_heads=2, window=3, budget=77, ctx=2500, ctx_min=900),     # group of 24
    dict(batch=5, n_q_heads=4, n_kv_heads=4, window=16, budget=4096, ctx=1500, ctx_min=17),    # budget above contexts
    dict(batch=2, n_q_heads=16, n_kv_heads=2, window=16, budget=5000, ctx=17000, ctx_min=9000),  # buffer-sized shares
]


@pytest.mark.parametrize("kw", CASES)
@pytest.mark.parametrize("agg", [api.AS_AGG_MAX, api.AS_AGG_SOFTMAX_SUM])
def test_outputs_stay_inside_their_arrays(kw, agg):
    print("guards", kw, agg, flush=True)
    w = wl.Workload("guard", page_table="scatter", pool_slack=1.15, seed=23, **kw)
    dev = to_dev(wl.make_inputs(w))
    p = params_for(dev, agg=agg)
    B, Hq, Hkv, C = w.batch, w.n_q_heads, w.n_kv_heads, w.budget
    stride = dev.block_table.shape[1] * 16
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    inputs = (dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens, dev.q_win, dev.q_cur, dev.q_real)
    before = fingerprint(*inputs)
    ctx, ctx_pack = api.Context(p), api.Context(p, pack=2)     # one workspace layout per context (see the end)

    q_hat = Guarded((B, Hq, 128), torch.float32, 7.5)
    api.as_predict_query(ctx, p, dev.q_win, dev.q_cur, q_hat.t)
    torch.cuda.synchronize()
    assert q_hat.intact()

    outs = {}
    for name in ("select_step", "score_topk", "pack0", "pack1", "fused", "two_launches"):
        outs[name] = (Guarded((B, Hkv, C), torch.int32, -77), Guarded((B, Hkv), torch.int32, -77))
    api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur, outs["select_step"][0].t, outs["select_step"][1].t)
    # the routes the library did not take by itself for this shape (per-ctx development knob; same workspace layout)
    ctx_routes = api.Context(p)
    for name, mode in (("fused", 2), ("two_launches", 1)):
        ctx_routes.set_select_mode(mode)
        api.as_select_step(ctx_routes, p, kv, dev.q_win, dev.q_cur, outs[name][0].t, outs[name][1].t)
    api.as_score_topk(ctx, p, kv, q_hat.t, outs["score_topk"][0].t, outs["score_topk"][1].t)
    api.as_select_step_pack(ctx_pack, p, [api.layer_io(kv, dev.q_win, dev.q_cur, outs[n][0].t, outs[n][1].t)
                                     for n in ("pack0", "pack1")])
    torch.cuda.synchronize()
    for name, (gi, gc) in outs.items():
        assert gi.intact() and gc.intact(), name
        assert torch.equal(gi.t, outs["select_step"][0].t) and torch.equal(gc.t, outs["select_step"][1].t), name
    sel_idx, sel_cnt = outs["select_step"][0].t, outs["select_step"][1].t
    lens = dev.ctx_lens.cpu()
    for b in range(B):
        keep = min(C, int(lens[b]))
        assert (sel_cnt[b] == keep).all()
        assert (sel_idx[b, :, keep:] == -1).all() and (sel_idx[b, :, :keep] >= 0).all()

    if agg == api.AS_AGG_MAX:                       # the stand-alone stages do not offer the normalised aggregation
        scores = Guarded((B, Hkv, stride), torch.float32, 12345.0)
        api.as_score_keys(ctx, p, kv, q_hat.t, scores.t)
        gi, gc = Guarded((B, Hkv, C), torch.int32, -77), Guarded((B, Hkv), torch.int32, -77)
        api.as_topk_select(ctx, p, scores.t, dev.ctx_lens, gi.t, gc.t)
        torch.cuda.synchronize()
        assert scores.intact() and gi.intact() and gc.intact()
        for b in range(B):                          # entries beyond the sequence are left alone
            assert (scores.t[b, :, int(lens[b]):] == 12345.0).all()
        assert torch.equal(gi.t, sel_idx) and torch.equal(gc.t, sel_cnt)

    tail = torch.clamp(dev.ctx_lens - 3, min=0)     # the last three tokens attended densely
    for dense, use_tail in ((False, False), (False, True), (True, False)):
        out, lse = Guarded((B, Hq, 128), torch.bfloat16, 3.0), Guarded((B, Hq), torch.float32, 3.0)
        if dense:
            api.as_dense_decode_attn(ctx, p, kv, dev.q_real, out.t, lse.t)
        else:
            api.as_sparse_decode_attn(ctx, p, kv, dev.q_real, sel_idx, sel_cnt, tail if use_tail else None, out.t, lse.t)
        torch.cuda.synchronize()
        assert out.intact() and lse.intact(), (dense, use_tail)
        assert torch.isfinite(out.t.float()).all()

    cp = api.compact_pages(p)
    k_out = Guarded((B * cp, Hkv, 16, 128), torch.bfloat16, 9.0)
    v_out = Guarded((B * cp, Hkv, 16, 128), torch.bfloat16, 9.0)
    tab, ln = Guarded((B, cp), torch.int32, -77), Guarded((B,), torch.int32, -77)
    api.as_gather_kv(ctx, p, kv, sel_idx, sel_cnt, k_out.t, v_out.t, tab.t, ln.t)
    inter, ratio = Guarded((B, Hkv), torch.int32, -77), Guarded((B, Hkv), torch.float32, 3.0)
    api.as_overlap_ratio(ctx, p, sel_idx, sel_cnt, sel_idx, sel_cnt, inter.t, ratio.t)
    torch.cuda.synchronize()
    assert k_out.intact() and v_out.intact() and tab.intact() and ln.intact() and inter.intact() and ratio.intact()
    assert torch.equal(inter.t, sel_cnt)
    for b in range(B):                              # compact slots at and beyond the count are left alone
        keep = min(C, int(lens[b]))
        flat = k_out.t[b * cp:(b + 1) * cp].permute(1, 0, 2, 3).reshape(Hkv, cp * 16, 128)
        assert (flat[:, keep:] == 9.0).all()

    assert fingerprint(*inputs) == before           # nothing wrote into the cache, the table or the queries
    # the regions of the context workspace (attention partials, q_hat, score rows, candidates) are separated by
    # gaps that hold the pattern as_create wrote: a kernel that outgrew the size computed for its region shows here
    assert ctx.damaged_workspace_gap(p) == -1
    assert ctx_routes.damaged_workspace_gap(p) == -1
    assert ctx_pack.damaged_workspace_gap(p, 2) == -1


def test_state_updates_touch_only_their_rows():
    w = wl.Workload("guard-state", 4, 8, 2, 6, 64, 900, ctx_min=15, page_table="scatter", pool_slack=1.3, seed=29)
    dev = to_dev(wl.make_inputs(w))
    p = params_for(dev)
    ctx = api.Context(p)
    B, Hq, Hkv, W = w.batch, w.n_q_heads, w.n_kv_heads, w.window
    q_win, q_cur = Guarded((B, Hq, W, 128), torch.bfloat16, 5.0), Guarded((B, Hq, 128), torch.bfloat16, 5.0)
    q_win.t.copy_(dev.q_win)
    q_cur.t.copy_(dev.q_cur)
    api.as_window_push(ctx, p, q_win.t, q_cur.t, dev.q_real)
    lens = Guarded((B,), torch.int32, -77)
    lens.t.copy_(dev.ctx_lens)
    k_pool = Guarded(tuple(dev.k_pool.shape), torch.bfloat16, 5.0)
    v_pool = Guarded(tuple(dev.v_pool.shape), torch.bfloat16, 5.0)
    k_pool.t.copy_(dev.k_pool)
    v_pool.t.copy_(dev.v_pool)
    k_new = torch.randn((B, Hkv, 128), device="cuda").to(torch.bfloat16)
    api.as_kv_append(ctx, p, k_pool.t, v_pool.t, dev.block_table, lens.t, k_new, k_new)
    torch.cuda.synchronize()
    assert q_win.intact() and q_cur.intact() and lens.intact() and k_pool.intact() and v_pool.intact()
    assert torch.equal(q_cur.t, dev.q_real) and torch.equal(q_win.t[:, :, -1], dev.q_cur)
    assert torch.equal(lens.t, dev.ctx_lens + 1)
    assert int((k_pool.t != dev.k_pool).any(dim=-1).sum()) <= B * Hkv     # one row per (sequence, head) at most


def test_the_workspace_check_sees_a_write_into_a_gap():
    """The check itself: after calls with one set of shapes, the gaps of a *different* layout (half the query
    heads: its first gap lies where the dense attention call stored its split partials) no longer hold the fill
    pattern."""
    w = wl.Workload("guard-check", 2, 8, 2, 4, 32, 400, page_table="identity", seed=31)
    dev = to_dev(wl.make_inputs(w))
    p = params_for(dev)
    ctx = api.Context(p)
    assert ctx.damaged_workspace_gap(p) == -1                     # fresh workspace
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    api.as_select_step(ctx, p, kv, dev.q_win, dev.q_cur)
    api.as_dense_decode_attn(ctx, p, kv, dev.q_real)
    assert ctx.damaged_workspace_gap(p) == -1
    other = api.make_params(2, 4, 2, 4, 32, dev.max_pages)
    assert ctx.damaged_workspace_gap(other) == 0


def test_corrupt_tables_stay_inside_the_pool_and_inside_their_rows():
    """The header's promise for arrays that break the caller's contract: page ids are clamped into the pool, lengths
    into the block table, indices into the sequence, counts into [0, C].  Sequence 1 gets every kind of damage; the
    calls must finish, leave every guard intact, and give sequences 0 and 2 the results of the undamaged run."""
    w = wl.Workload("corrupt", 3, 8, 2, 8, 96, 2000, ctx_min=700, page_table="scatter", pool_slack=1.2, seed=37)
    clean = to_dev(wl.make_inputs(w))
    p = params_for(clean)
    B, Hq, Hkv, C = w.batch, w.n_q_heads, w.n_kv_heads, w.budget
    num_pages = clean.k_pool.shape[0]

    def run(bt, lens, damage_selection):
        ctx = api.Context(p)
        kv = api.kv_view(clean.k_pool, clean.v_pool, bt, lens)
        sel = (Guarded((B, Hkv, C), torch.int32, -77), Guarded((B, Hkv), torch.int32, -77))
        api.as_select_step(ctx, p, kv, clean.q_win, clean.q_cur, sel[0].t, sel[1].t)
        # the same through the routes the library does not take by itself for this shape (every route has its own clamps)
        ctx_routes = api.Context(p)
        sel_fused = (Guarded((B, Hkv, C), torch.int32, -77), Guarded((B, Hkv), torch.int32, -77))
        sel_two = (Guarded((B, Hkv, C), torch.int32, -77), Guarded((B, Hkv), torch.int32, -77))
        for mode, s_out in ((2, sel_fused), (1, sel_two)):
            ctx_routes.set_select_mode(mode)
            api.as_select_step(ctx_routes, p, kv, clean.q_win, clean.q_cur, s_out[0].t, s_out[1].t)
        q_hat = api.as_predict_query(ctx, p, clean.q_win, clean.q_cur)
        scores = Guarded((B, Hkv, bt.shape[1] * 16), torch.float32, 0.0)
        api.as_score_keys(ctx, p, kv, q_hat, scores.t)
        sel2 = (Guarded((B, Hkv, C), torch.int32, -77), Guarded((B, Hkv), torch.int32, -77))
        api.as_topk_select(ctx, p, scores.t, lens, sel2[0].t, sel2[1].t)
        idx, cnt = sel[0].t.clone(), sel[1].t.clone()
        tail = torch.clamp(lens - 2, min=0)
        if damage_selection:
            idx[1, 0, :5] = torch.tensor([-9, 1 << 30, -1, 5_000_000, 3], dtype=torch.int32, device="cuda")
            cnt[1, 0] = C + 1000
            cnt[1, 1] = -4
            tail[1] = -100
        out, lse = Guarded((B, Hq, 128), torch.bfloat16, 3.0), Guarded((B, Hq), torch.float32, 3.0)
        api.as_sparse_decode_attn(ctx, p, kv, clean.q_real, idx, cnt, tail, out.t, lse.t)
        dense = Guarded((B, Hq, 128), torch.bfloat16, 3.0)
        api.as_dense_decode_attn(ctx, p, kv, clean.q_real, dense.t, want_lse=False)
        cp = api.compact_pages(p)
        k_out = Guarded((B * cp, Hkv, 16, 128), torch.bfloat16, 9.0)
        v_out = Guarded((B * cp, Hkv, 16, 128), torch.bfloat16, 9.0)
        tab, ln = Guarded((B, cp), torch.int32, -77), Guarded((B,), torch.int32, -77)
        api.as_gather_kv(ctx, p, kv, idx, cnt, k_out.t, v_out.t, tab.t, ln.t)
        inter = Guarded((B, Hkv), torch.int32, -77)
        api.as_overlap_ratio(ctx, p, idx, cnt, sel2[0].t, sel2[1].t, inter.t)
        k_pool, v_pool = Guarded(tuple(clean.k_pool.shape), torch.bfloat16, 5.0), Guarded(tuple(clean.v_pool.shape), torch.bfloat16, 5.0)
        k_pool.t.copy_(clean.k_pool)
        v_pool.t.copy_(clean.v_pool)
        lens2 = Guarded((B,), torch.int32, -77)
        lens2.t.copy_(lens)
        k_new = torch.ones((B, Hkv, 128), dtype=torch.bfloat16, device="cuda")
        api.as_kv_append(ctx, p, k_pool.t, v_pool.t, bt, lens2.t, k_new, k_new)
        torch.cuda.synchronize()
        guards = (sel[0], sel[1], scores, sel2[0], sel2[1], out, lse, dense, k_out, v_out, tab, ln, inter, k_pool,
                  v_pool, lens2, sel_fused[0], sel_fused[1], sel_two[0], sel_two[1])
        assert all(g.intact() for g in guards)
        assert ctx.damaged_workspace_gap(p) == -1
        assert ctx_routes.damaged_workspace_gap(p) == -1
        return dict(sel=sel[0].t, cnt=sel[1].t, sel2=sel2[0].t, sel_fused=sel_fused[0].t, cnt_fused=sel_fused[1].t,
                    sel_two=sel_two[0].t, cnt_two=sel_two[1].t, out=out.t, lse=lse.t, dense=dense.t, k_out=k_out.t,
                    inter=inter.t)

    ref = run(clean.block_table, clean.ctx_lens, damage_selection=False)
    bt = clean.block_table.clone()
    bt[1, 0::3] = -7                                   # negative page ids
    bt[1, 1::3] = num_pages + 12345                    # page ids beyond the pool
    for bad_len in (-3, 16 * bt.shape[1] + 999):       # a negative length, a length beyond the block table
        lens = clean.ctx_lens.clone()
        lens[1] = bad_len
        print("corrupt", bad_len, flush=True)
        got = run(bt, lens, damage_selection=True)
        for name in ("sel", "cnt", "sel2", "sel_fused", "cnt_fused", "sel_two", "cnt_two", "out", "lse", "dense", "inter"):
            for b in (0, 2):
                assert torch.equal(got[name][b], ref[name][b]), (name, b)
        cp = api.compact_pages(p)
        for b in (0, 2):
            assert torch.equal(got["k_out"][b * cp:(b + 1) * cp], ref["k_out"][b * cp:(b + 1) * cp])
