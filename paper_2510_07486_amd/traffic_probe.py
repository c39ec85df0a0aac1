"""HBM-traffic probe for rocprofv3 --pmc runs (FETCH_SIZE / WRITE_SIZE).

Launches, on one layer of a workload, (1) the calibration kernel - the paged walk over K with
coalesced loads and one word written per token, whose bytes are known exactly - and (2) the
fused scoring + top-k (as_score_topk), (3) sparse decode attention and (4) the KV re-organisation
(as_gather_kv) followed by dense attention over the compact pool, a few times each, so
that per-dispatch counter values can be scaled by what the same counter reads for the
calibration kernel.

    rocprofv3 --pmc FETCH_SIZE -d out -o fetch --output-format csv -- python3 -m paper_2510_07486_amd.traffic_probe c3
"""
import sys

import torch

from paper_2510_07486_amd import api, workloads as wl


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "c3"
    reps = int(sys.argv[2]) if len(sys.argv) > 2 else 3
    w = wl.CONFIGS[name]
    dev = "cuda"
    inp = wl.make_inputs(w, dev)
    p = api.make_params(w.batch, w.n_q_heads, w.n_kv_heads, w.window, w.budget, inp.max_pages)
    ctx = api.Context(p)
    kv = api.kv_view(inp.k_pool, inp.v_pool, inp.block_table, inp.ctx_lens)
    q_hat = api.as_predict_query(ctx, p, inp.q_win, inp.q_cur)
    scores = torch.empty((w.batch, w.n_kv_heads, inp.max_pages * 16), dtype=torch.float32, device=dev)
    ctx.set_score_variant(1)                        # calibration kernel behind as_score_keys
    for _ in range(reps):
        api.as_score_keys(ctx, p, kv, q_hat, scores)
    torch.cuda.synchronize()
    ctx.set_score_variant(0)
    for _ in range(reps):
        idx, cnt = api.as_score_topk(ctx, p, kv, q_hat)
    torch.cuda.synchronize()
    for _ in range(reps):
        api.as_sparse_decode_attn(ctx, p, kv, inp.q_real, idx, cnt, want_lse=False)
    torch.cuda.synchronize()
    comp = None
    for _ in range(reps):
        comp = api.as_gather_kv(ctx, p, kv, idx, cnt, *(comp or ()))
    torch.cuda.synchronize()
    pc = api.make_params(w.batch, w.n_q_heads, w.n_kv_heads, w.window, 16, api.compact_pages(p))
    ctx_c = api.Context(pc)
    kvc = api.kv_view(*comp)
    for _ in range(reps):
        api.as_dense_decode_attn(ctx_c, pc, kvc, inp.q_real, want_lse=False)
    torch.cuda.synchronize()
    tokens = int(inp.ctx_lens.sum())
    print(f"calibration kernel per launch: reads {tokens * w.n_kv_heads * 256} B of K, writes "
          f"{tokens * w.n_kv_heads * 4} B")


if __name__ == "__main__":
    main()
