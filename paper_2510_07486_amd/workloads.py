"""Seeded synthetic inputs for the KV-selection hot path.

This module only draws random numbers and lays them out in memory; it holds none
of the method's arithmetic, so both the HIP path and the CPU oracle may be fed
from it.  The shapes follow the Qwen3 rows of the paper's Table 1 (8B: 32 query /
8 KV heads, 36 layers; 32B: 64 / 8, 64 layers), the batch / context / budget
ranges of Fig. 2 and Table 3, and page size 16 (Fig. 2 caption).

Recipe
  K, V    i.i.d. N(0,1) drawn in fp32, rounded to bf16.  "Outlier channels":
          for every KV head a seeded choice of `n_outlier` of the 128 channels
          has its K values multiplied by `outlier_scale`.
  queries per (sequence, query head) an AR(1) chain of W+2 states in fp32,
          x_0 ~ N(0,I), x_s = rho*x_{s-1} + (1-rho)*N(0,I), rounded to bf16.
          x_0..x_{W-1} is the cached window (oldest first), x_W the current
          query and x_{W+1} the real next-step query used by the attention.
  pages   token n of sequence b lives in page block_table[b][n // 16], slot
          n % 16; the pool is [num_pages, H_kv, 16, 128].  The table is the
          identity, a random permutation of the sequence's own pool, or a
          random scatter in a pool shared by all sequences.
"""
from __future__ import annotations

import dataclasses
from typing import Optional, Sequence

import torch

HEAD_DIM = 128
PAGE = 16


@dataclasses.dataclass
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    window: int
    budget: int
    ctx: int                        # context length (max when ragged)
    ctx_min: Optional[int] = None   # ragged: lengths uniform in [ctx_min, ctx]
    rho: float = 0.95
    rho_range: Optional[Sequence[float]] = None  # per-head rho ~ U[lo, hi]
    n_outlier: int = 0
    outlier_scale: float = 8.0
    page_table: str = "identity"    # identity | permute | scatter
    layers: int = 1
    seed: int = 0
    pool_slack: float = 1.0         # scatter: pool pages / pages in use
    lag2: float = 0.0               # > 0: AR(2) queries x_s = (rho - lag2) x_{s-1} + lag2 x_{s-2} + (1 - rho) noise

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


# The five benchmark workloads, c1..c5.
CONFIGS = {
    "c1": Workload("c1", 1, 8, 2, 8, 256, 4096, rho=0.9, page_table="identity"),
    "c2": Workload("c2", 1, 32, 8, 16, 2048, 16384, n_outlier=4, page_table="identity"),
    "c3": Workload("c3", 32, 32, 8, 16, 2048, 32768, page_table="permute", layers=36),
    "c4": Workload("c4", 16, 64, 8, 16, 4096, 32768, n_outlier=4, page_table="permute", layers=64),
    "c5": Workload("c5", 64, 32, 8, 16, 1024, 65536, ctx_min=4096, rho_range=(0.8, 0.99),
                   page_table="scatter", pool_slack=1.25),
}


def scaled(w: Workload, **kw) -> Workload:
    return dataclasses.replace(w, **kw)


@dataclasses.dataclass
class Inputs:
    """One layer's tensors.  All on `device`."""
    w: Workload
    k_pool: torch.Tensor        # bf16 [num_pages, H_kv, 16, 128]
    v_pool: torch.Tensor        # bf16 same
    block_table: torch.Tensor   # int32 [B, max_pages]
    ctx_lens: torch.Tensor      # int32 [B]
    q_win: torch.Tensor         # bf16 [B, H_q, W, 128] oldest first
    q_cur: torch.Tensor         # bf16 [B, H_q, 128]
    q_real: torch.Tensor        # bf16 [B, H_q, 128]

    @property
    def max_pages(self) -> int:
        return self.block_table.shape[1]

    @property
    def num_pages(self) -> int:
        return self.k_pool.shape[0]


def _gen(seed: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000003 + stream)
    return g


def _randn_bf16(shape, g, device, chunk_elems=1 << 28) -> torch.Tensor:
    """N(0,1) in fp32 -> bf16, drawn in chunks so fp32 staging stays small."""
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    n = flat.numel()
    for s in range(0, n, chunk_elems):
        e = min(n, s + chunk_elems)
        flat[s:e] = torch.randn(e - s, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    return out


def draw_ctx_lens(w: Workload) -> torch.Tensor:
    """Per-sequence context lengths (CPU int32)."""
    if w.ctx_min is None:
        return torch.full((w.batch,), w.ctx, dtype=torch.int32)
    g = _gen(w.seed, 1, "cpu")
    return torch.randint(w.ctx_min, w.ctx + 1, (w.batch,), generator=g, dtype=torch.int32)


def make_page_table(w: Workload, ctx_lens: torch.Tensor):
    """Returns (block_table int32 [B, max_pages] on CPU, num_pages)."""
    B = w.batch
    pages_per = [(int(n) + PAGE - 1) // PAGE for n in ctx_lens.tolist()]
    max_pages = max(1, (w.ctx + PAGE - 1) // PAGE)
    bt = torch.zeros((B, max_pages), dtype=torch.int32)
    g = _gen(w.seed, 2, "cpu")
    if w.page_table in ("identity", "permute"):
        num_pages = B * max_pages
        for b in range(B):
            ids = torch.arange(b * max_pages, (b + 1) * max_pages, dtype=torch.int64)
            if w.page_table == "permute":
                ids = ids[torch.randperm(max_pages, generator=g)]
            bt[b, :pages_per[b]] = ids[:pages_per[b]].to(torch.int32)
    elif w.page_table == "scatter":
        used = sum(pages_per)
        num_pages = max(1, int(used * w.pool_slack))
        perm = torch.randperm(num_pages, generator=g)[:used].to(torch.int32)
        o = 0
        for b in range(B):
            bt[b, :pages_per[b]] = perm[o:o + pages_per[b]]
            o += pages_per[b]
    else:
        raise ValueError(w.page_table)
    return bt, num_pages


def make_queries(w: Workload, device="cpu", layer: int = 0):
    """AR(1) chains (AR(2) when w.lag2 > 0) -> (q_win, q_cur, q_real), bf16."""
    B, H, W, D = w.batch, w.n_q_heads, w.window, HEAD_DIM
    g = _gen(w.seed, 100 + 7 * layer, device)
    if w.rho_range is not None:
        lo, hi = w.rho_range
        rho = lo + (hi - lo) * torch.rand((B, H, 1), generator=g, device=device, dtype=torch.float32)
    else:
        rho = torch.full((B, H, 1), w.rho, device=device, dtype=torch.float32)
    x = torch.randn((B, H, D), generator=g, device=device, dtype=torch.float32)
    chain = [x]
    prev = x
    for _ in range(W + 1):
        noise = torch.randn((B, H, D), generator=g, device=device, dtype=torch.float32)
        nxt = (rho - w.lag2) * x + w.lag2 * prev + (1.0 - rho) * noise     # lag2 = 0: the AR(1) chain
        prev, x = x, nxt
        chain.append(x)
    chain = torch.stack(chain, dim=2).to(torch.bfloat16)      # [B,H,W+2,D]
    return (chain[:, :, :W].contiguous(), chain[:, :, W].contiguous(), chain[:, :, W + 1].contiguous())


def make_kv(w: Workload, num_pages: int, device="cpu", layer: int = 0):
    """K and V pools for one layer, bf16 [num_pages, H_kv, 16, 128]."""
    shape = (num_pages, w.n_kv_heads, PAGE, HEAD_DIM)
    k = _randn_bf16(shape, _gen(w.seed, 200 + 7 * layer, device), device)
    v = _randn_bf16(shape, _gen(w.seed, 300 + 7 * layer, device), device)
    if w.n_outlier > 0:
        g = _gen(w.seed, 400 + 7 * layer, "cpu")
        for j in range(w.n_kv_heads):
            ch = torch.randperm(HEAD_DIM, generator=g)[: w.n_outlier].to(device)
            k[:, j, :, ch] = (k[:, j, :, ch].float() * w.outlier_scale).to(torch.bfloat16)
    return k, v


def make_inputs(w: Workload, device="cpu", layer: int = 0) -> Inputs:
    ctx_lens = draw_ctx_lens(w)
    bt, num_pages = make_page_table(w, ctx_lens)
    k, v = make_kv(w, num_pages, device, layer)
    q_win, q_cur, q_real = make_queries(w, device, layer)
    return Inputs(w, k, v, bt.to(device), ctx_lens.to(device), q_win, q_cur, q_real)


def extract_sequence(inp: Inputs, b: int) -> Inputs:
    """Copy one sequence of a (possibly device-resident) layer into a stand-alone
    batch-1 CPU problem with an identity page table, for spot checks at full size."""
    w = inp.w
    n = int(inp.ctx_lens[b])
    npg = (n + PAGE - 1) // PAGE
    pages = inp.block_table[b, :npg].long()
    k = inp.k_pool[pages].cpu() if npg else inp.k_pool[:1].cpu()
    v = inp.v_pool[pages].cpu() if npg else inp.v_pool[:1].cpu()
    bt = torch.arange(max(npg, 1), dtype=torch.int32).view(1, -1)
    w1 = scaled(w, batch=1, ctx=max(n, 1), ctx_min=None, page_table="identity", layers=1)
    return Inputs(w1, k, v, bt, torch.tensor([n], dtype=torch.int32),
                  inp.q_win[b:b + 1].cpu(), inp.q_cur[b:b + 1].cpu(), inp.q_real[b:b + 1].cpu())
