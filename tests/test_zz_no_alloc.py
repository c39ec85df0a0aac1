"""as_select_step_static, the entry point for callers that cannot allocate: same kernels as as_select_step with
their scratch (q_hat, score rows, per-share candidates) in the library's static device array.  Checked through the
C ABI against as_select_step, bit for bit, on two calls in a row, the second with a smaller input; every route the
call can take (fused kernels with one share per row, with several shares and a merge, scoring and top-k over score
rows, the two-pass softmax aggregation) goes through the shared array.  The callers it is for include code under
HIP graph capture: two calls are captured and replayed, with eager work between the replays."""
import gc

import ctypes as C

import pytest
import torch

from paper_2510_07486_amd import api
from paper_2510_07486_amd import workloads as wl
from gpu_common import params_for, to_dev

pytestmark = pytest.mark.gpu


def _both(w, agg=0):
    dev = to_dev(wl.make_inputs(w))
    p = params_for(dev, agg=agg)
    kv = api.kv_view(dev.k_pool, dev.v_pool, dev.block_table, dev.ctx_lens)
    ref_idx, ref_cnt = api.as_select_step(api.Context(p), p, kv, dev.q_win, dev.q_cur)
    idx = torch.full((w.batch, w.n_kv_heads, w.budget), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((w.batch, w.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    gc.collect()                                   # tensors of earlier cases must not be freed while we watch
    before = torch.cuda.memory_allocated()
    api.as_select_step_static(p, kv, dev.q_win, dev.q_cur, idx, cnt)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(idx, ref_idx) and torch.equal(cnt, ref_cnt), w.name
    return api.select_plan(p, 1)


def test_static_scratch_selection_equals_the_ctx_call_on_two_calls_in_a_row():
    # first call: 32 rows of up to 40000 tokens, cut into several shares (candidates and a merge through the array)
    big = wl.Workload("static-big", 4, 32, 8, 16, 512, 40000, ctx_min=9000, page_table="scatter", pool_slack=1.2, seed=51)
    plan = _both(big)
    assert plan[1] > 1
    # second call, smaller input, same array (it still holds the first call's candidates): score rows, one launch
    small = wl.Workload("static-small", 1, 8, 2, 8, 64, 1500, page_table="permute", seed=52)
    _both(small)
    # a batch that fills the chip with one share per row (nothing but q_hat in the array), ragged, then the same
    # shape again with fewer tokens
    _both(wl.Workload("static-rows", 40, 32, 8, 16, 300, 5000, ctx_min=1, page_table="scatter", pool_slack=1.1, seed=53))
    _both(wl.Workload("static-rows2", 40, 32, 8, 16, 300, 700, ctx_min=1, page_table="scatter", pool_slack=1.1, seed=54))
    # softmax-normalised aggregation: two passes, per-share (max, sum) pairs through the array; then smaller
    _both(wl.Workload("static-sm", 2, 16, 4, 8, 256, 12000, ctx_min=3000, page_table="permute", seed=55), agg=2)
    _both(wl.Workload("static-sm2", 1, 16, 4, 8, 100, 2000, page_table="permute", seed=56), agg=2)


def test_static_scratch_refuses_what_does_not_fit():
    """Parameters that need more than the array holds are refused on the host, before any launch (the pointers
    are never touched); bad arguments are reported as for as_select_step."""
    L = api.lib()
    one = C.c_void_p(1)
    kv = api.AsKvView(1, 1, 1, 1, 1)
    big = api.make_params(128, 32, 8, 16, 4096, 8192)          # candidates of 1024 rows x 2 shares x 4096 x 8 B = 64 MiB
    share, shares, cand = api.select_plan(big, 1)
    assert shares > 1 and 1024 * shares * cand * 8 > api.AS_STATIC_SCRATCH_BYTES
    assert L.as_select_step_static(C.byref(big), C.byref(kv), one, one, one, one, None) == 5
    assert L.as_status_str(5).decode().startswith("parameters need more")
    ok = api.make_params(1, 8, 2, 4, 16, 4)
    assert L.as_select_step_static(C.byref(ok), C.byref(kv), None, one, one, one, None) == 1
    assert L.as_select_step_static(C.byref(api.make_params(1, 8, 2, 4, 16, 4, ridge_eps=0.0)), C.byref(kv), one, one, one,
                                   one, None) == 1


def test_static_entry_captured_into_a_graph_replays_like_eager():
    """Two static-scratch calls of different shapes (several shares with a merge inside the kernel; score rows in
    one launch) captured into one HIP graph and replayed four times, with the queries changed in place and eager
    work between the replays; every replay equals the ctx calls on the same inputs."""
    ws = [wl.Workload("cap-a", 4, 32, 8, 16, 256, 36000, ctx_min=8000, page_table="scatter", pool_slack=1.2, seed=61),
          wl.Workload("cap-b", 1, 8, 2, 8, 64, 3000, page_table="permute", seed=62)]
    devs = [to_dev(wl.make_inputs(w)) for w in ws]
    ps = [params_for(d) for d in devs]
    kvs = [api.kv_view(d.k_pool, d.v_pool, d.block_table, d.ctx_lens) for d in devs]
    ctxs = [api.Context(p) for p in ps]
    outs = [(torch.empty((w.batch, w.n_kv_heads, w.budget), dtype=torch.int32, device="cuda"),
             torch.empty((w.batch, w.n_kv_heads), dtype=torch.int32, device="cuda")) for w in ws]

    def both(stream):
        for p, kv, d, (oi, oc) in zip(ps, kvs, devs, outs):
            api.as_select_step_static(p, kv, d.q_win, d.q_cur, oi, oc, stream=stream)

    both(torch.cuda.current_stream())                 # warm-up: the array's address is resolved outside the capture
    torch.cuda.synchronize()
    gc.collect()
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=s):
        both(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(4):
        for w, d in zip(ws, devs):
            qw, qc, _ = wl.make_queries(wl.scaled(w, seed=200 + rep))
            d.q_win.copy_(qw)
            d.q_cur.copy_(qc)
        refs = [api.as_select_step(c, p, kv, d.q_win, d.q_cur) for c, p, kv, d in zip(ctxs, ps, kvs, devs)]
        for oi, oc in outs:
            oi.fill_(-9)
            oc.fill_(-9)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for (oi, oc), (ri, rc) in zip(outs, refs):
            assert torch.equal(oi, ri) and torch.equal(oc, rc), rep
