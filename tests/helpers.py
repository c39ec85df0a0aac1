"""Shared test helpers (no method arithmetic beyond set comparisons)."""
import numpy as np
import torch

TIE_REL = 1e-3      # relative half-width of the tie band around the k-th score


def gather_keys(pool: torch.Tensor, block_table: torch.Tensor, b: int, j: int, n_tokens: int) -> np.ndarray:
    """[n_tokens, D] fp64 rows of sequence b, kv head j, through the page table (torch indexing)."""
    P = pool.shape[2]
    npg = (n_tokens + P - 1) // P
    pages = block_table[b, :npg].long()
    rows = pool[pages, j].reshape(npg * P, pool.shape[3])[:n_tokens]
    return rows.to(torch.float64).numpy()


def compare_selection(gpu_idx, gpu_cnt, ref_idx, ref_cnt, ref_scores, ctx_lens, budget):
    """Compare index sets per (b, kv head).  Returns the number of tie swaps.

    A difference is accepted (and counted) only if every token in the symmetric difference
    has an oracle score within TIE_REL * max(|tau|, 1e-30) of tau, the oracle's last kept
    score; anything else raises.  Also checks ascending order and -1 padding.
    """
    gpu_idx = gpu_idx.cpu().numpy(); gpu_cnt = gpu_cnt.cpu().numpy()
    ref_idx = ref_idx.cpu().numpy(); ref_cnt = ref_cnt.cpu().numpy()
    sc = ref_scores.cpu().numpy()
    swaps = 0
    B, H, C = ref_idx.shape
    assert C == budget
    for b in range(B):
        n = int(ctx_lens[b])
        for j in range(H):
            c = int(ref_cnt[b, j])
            assert c == min(budget, n)
            assert int(gpu_cnt[b, j]) == c, (b, j, gpu_cnt[b, j], c)
            g = gpu_idx[b, j]
            assert np.all(g[c:] == -1), (b, j)
            gs = g[:c]
            assert np.all(gs >= 0) and np.all(gs < n), (b, j)
            assert np.all(np.diff(gs) > 0), f"not strictly ascending at {(b, j)}"
            rs = ref_idx[b, j, :c]
            if np.array_equal(gs, rs):
                continue
            tau = sc[b, j, rs].min()
            band = TIE_REL * max(abs(float(tau)), 1e-30)
            diff = np.setxor1d(gs, rs)
            bad = np.abs(sc[b, j, diff] - tau) > band
            assert not bad.any(), f"selection differs outside the tie band at {(b, j)}: {diff[bad][:8]}"
            swaps += len(diff) // 2
    return swaps
