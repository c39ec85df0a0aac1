"""The library's calls neither allocate nor synchronise, so a whole decode step can be captured into a HIP
graph and replayed.  Replays are checked against eager execution bit for bit, several times, with eager work and
host synchronisation between the replays and with the inputs changed in place (the graph holds pointers, not data)."""
import gc

import pytest
import torch

from paper_2510_07486_amd import api
from paper_2510_07486_amd import workloads as wl
from gpu_common import params_for, to_dev

pytestmark = pytest.mark.gpu


def note(*a):
    print(*a, flush=True)


def make_layers(w, n):
    return [to_dev(wl.make_inputs(w, layer=l)) for l in range(n)]


def fresh_queries(w, layers, seed):
    """New query windows written into the existing device buffers (same pointers)."""
    for l, x in enumerate(layers):
        qw, qc, qr = wl.make_queries(wl.scaled(w, seed=seed), layer=l)
        x.q_win.copy_(qw)
        x.q_cur.copy_(qc)
        x.q_real.copy_(qr)


@pytest.mark.parametrize("packed", [False, True])
def test_graph_replay_of_a_decode_step_equals_eager(packed):
    w = wl.Workload("g", 2, 8, 2, 8, 128, 3000, ctx_min=500, page_table="scatter", pool_slack=1.2, seed=3)
    n_layers = 3
    layers = make_layers(w, n_layers)
    p = params_for(layers[0])
    ctx_sel, ctx_att = api.Context(p, pack=n_layers), api.Context(p)
    kvs = [api.kv_view(x.k_pool, x.v_pool, x.block_table, x.ctx_lens) for x in layers]
    B, Hq, Hkv, C = w.batch, w.n_q_heads, w.n_kv_heads, w.budget
    sel = [(torch.empty((B, Hkv, C), dtype=torch.int32, device="cuda"),
            torch.empty((B, Hkv), dtype=torch.int32, device="cuda")) for _ in range(n_layers)]
    outs = [torch.empty((B, Hq, 128), dtype=torch.bfloat16, device="cuda") for _ in range(n_layers)]
    ios = [api.layer_io(kvs[l], layers[l].q_win, layers[l].q_cur, sel[l][0], sel[l][1]) for l in range(n_layers)]
    ios_arr = (api.AsLayerIo * n_layers)(*ios)

    def step(stream):
        if packed:
            api.as_select_step_pack(ctx_sel, p, ios_arr, stream=stream)
        for l, x in enumerate(layers):
            if not packed:
                api.as_select_step(ctx_sel, p, kvs[l], x.q_win, x.q_cur, sel[l][0], sel[l][1], stream=stream)
            api.as_sparse_decode_attn(ctx_att, p, kvs[l], x.q_real, sel[l][0], sel[l][1], out=outs[l], stream=stream,
                                      want_lse=False)

    def eager():
        step(torch.cuda.current_stream())
        torch.cuda.synchronize()
        return [s[0].clone() for s in sel], [o.clone() for o in outs]

    eager()                                           # warm-up: function attributes, lazy module loading
    gc.collect()                                      # a context collected during the capture would hipFree: not capturable
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=s):
        step(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(4):
        fresh_queries(w, layers, seed=100 + rep)      # eager work between replays, inputs changed in place
        ref_sel, ref_out = eager()
        for t in sel:
            t[0].fill_(-5)
        for o in outs:
            o.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for l in range(n_layers):
            assert torch.equal(sel[l][0], ref_sel[l]), (rep, l)
            assert torch.equal(outs[l], ref_out[l]), (rep, l)
    note("  graph replays identical to eager, packed =", packed)


def test_graph_with_selection_on_a_forked_stream():
    """Capture of the two-stream schedule: selection of layer l forks onto a side stream and joins before the
    attention that needs it (here: the next replay's), attention runs on the capture stream."""
    w = wl.Workload("g2", 3, 16, 4, 16, 256, 5000, ctx_min=2000, page_table="permute", seed=9)
    n_layers = 4
    layers = make_layers(w, n_layers)
    p = params_for(layers[0])
    ctx_sel, ctx_att = api.Context(p), api.Context(p)
    kvs = [api.kv_view(x.k_pool, x.v_pool, x.block_table, x.ctx_lens) for x in layers]
    B, Hq, Hkv, C = w.batch, w.n_q_heads, w.n_kv_heads, w.budget
    cur = [(torch.empty((B, Hkv, C), dtype=torch.int32, device="cuda"),
            torch.empty((B, Hkv), dtype=torch.int32, device="cuda")) for _ in range(n_layers)]
    nxt = [(torch.empty((B, Hkv, C), dtype=torch.int32, device="cuda"),
            torch.empty((B, Hkv), dtype=torch.int32, device="cuda")) for _ in range(n_layers)]
    outs = [torch.empty((B, Hq, 128), dtype=torch.bfloat16, device="cuda") for _ in range(n_layers)]
    for l, x in enumerate(layers):                    # the selection the first step attends over
        api.as_select_step(ctx_sel, p, kvs[l], x.q_win, x.q_cur, cur[l][0], cur[l][1])
    torch.cuda.synchronize()

    def serial():
        for l, x in enumerate(layers):
            api.as_select_step(ctx_sel, p, kvs[l], x.q_win, x.q_cur, nxt[l][0], nxt[l][1])
            api.as_sparse_decode_attn(ctx_att, p, kvs[l], x.q_real, cur[l][0], cur[l][1], out=outs[l], want_lse=False)
        torch.cuda.synchronize()
        return [t[0].clone() for t in nxt], [o.clone() for o in outs]

    ref_nxt, ref_out = serial()
    gc.collect()
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    main.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=main):
        for l, x in enumerate(layers):
            side.wait_stream(main)                    # fork: layer l's queries exist from here on
            api.as_select_step(ctx_sel, p, kvs[l], x.q_win, x.q_cur, nxt[l][0], nxt[l][1], stream=side)
            api.as_sparse_decode_attn(ctx_att, p, kvs[l], x.q_real, cur[l][0], cur[l][1], out=outs[l], stream=main,
                                      want_lse=False)
        main.wait_stream(side)                        # join
    torch.cuda.synchronize()
    for rep in range(3):
        for t in nxt:
            t[0].fill_(-5)
        for o in outs:
            o.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for l in range(n_layers):
            assert torch.equal(nxt[l][0], ref_nxt[l]), (rep, l)
            assert torch.equal(outs[l], ref_out[l]), (rep, l)
        torch.zeros(1024, device="cuda").sum().item()  # unrelated eager work and a host sync between replays
