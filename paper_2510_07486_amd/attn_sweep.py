"""Sweep of the attention split count (development knob) on one layer of a workload:

    python -m paper_2510_07486_amd.attn_sweep c4 1 2 3 4 5 6 8 12 16

prints the time of as_sparse_decode_attn per forced number of splits per (sequence, KV head), 0 = the library's own
choice.  The selection attended over is made once with as_select_step; four copies of the layer are rotated so that
rows come from HBM."""
import sys

import torch

from paper_2510_07486_amd import api, workloads as wl


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "c3"
    counts = [int(x) for x in sys.argv[2:]] or [0, 1, 2, 3, 4, 6, 8, 12, 16]
    w = wl.CONFIGS[name]
    dev = torch.device("cuda:0")
    lens_cpu = wl.draw_ctx_lens(w)
    bt_cpu, num_pages = wl.make_page_table(w, lens_cpu)
    copies = [wl.make_kv(w, num_pages, dev, l) for l in range(4)]
    qw, qc, qr = wl.make_queries(w, dev, 0)
    bt, lens = bt_cpu.to(dev), lens_cpu.to(dev)
    p = api.make_params(w.batch, w.n_q_heads, w.n_kv_heads, w.window, w.budget, bt.shape[1])
    kvs = [api.kv_view(k, v, bt, lens) for k, v in copies]
    idx, cnt = api.as_select_step(api.Context(p), p, kvs[0], qw, qc)
    out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    rows = int(torch.clamp(lens_cpu, max=w.budget).sum()) * w.n_kv_heads
    print(f"{name}: {w.batch * w.n_kv_heads} (sequence, KV head) pairs, budget {w.budget}")
    for n in counts:
        api.lib().as_debug_set_attn_splits(n)
        ctx = api.Context(p)                      # sized for this split count
        for i in range(4):
            api.as_sparse_decode_attn(ctx, p, kvs[i % 4], qr, idx, cnt, out=out, want_lse=False)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 40
        e0.record()
        for i in range(reps):
            api.as_sparse_decode_attn(ctx, p, kvs[i % 4], qr, idx, cnt, out=out, want_lse=False)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        label = "library's choice" if n == 0 else f"{n} splits = {n * w.batch * w.n_kv_heads} workgroups"
        print(f"  {label:36s} {us:7.1f} us  {rows * 512 / us / 1e3:7.0f} GB/s")
    api.lib().as_debug_set_attn_splits(0)


if __name__ == "__main__":
    main()
