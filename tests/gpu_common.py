"""Glue for the GPU parity tests: run the HIP path and the oracle on the same seeded inputs."""
import math

import numpy as np
import torch

import oracle
from paper_2510_07486_amd import api
from paper_2510_07486_amd import workloads as wl

SCALE = 1.0 / math.sqrt(128)
# bf16 hi+lo split of q_hat (2^-17 relative per term) + fp32 accumulation over 128 terms
SCORE_REL_ABSDOT = 1.6e-5


def f32(x) -> float:
    return float(np.float32(x))


def to_dev(inp: wl.Inputs, device="cuda") -> wl.Inputs:
    return wl.Inputs(inp.w, inp.k_pool.to(device), inp.v_pool.to(device), inp.block_table.to(device),
                     inp.ctx_lens.to(device), inp.q_win.to(device), inp.q_cur.to(device), inp.q_real.to(device))


def params_for(inp: wl.Inputs, eps=1e-2, beta=1.0, agg=0, budget=None):
    w = inp.w
    return api.make_params(w.batch, w.n_q_heads, w.n_kv_heads, w.window, budget or w.budget, inp.max_pages,
                           ridge_eps=f32(eps), softmax_beta=beta, sm_scale=f32(SCALE), agg=agg)


def absdot_bound(inp_cpu: wl.Inputs, q_hat: torch.Tensor) -> torch.Tensor:
    """max over the group of sum_d |q_hat_d| |K_d| per (b, j, n): scale of the rounding error of a score."""
    w = inp_cpu.w
    B, Hkv, G = w.batch, w.n_kv_heads, w.group
    stride = inp_cpu.max_pages * wl.PAGE
    out = torch.zeros((B, Hkv, stride), dtype=torch.float64)
    for b in range(B):
        n = int(inp_cpu.ctx_lens[b])
        npg = (n + wl.PAGE - 1) // wl.PAGE
        if npg == 0:
            continue
        pages = inp_cpu.block_table[b, :npg].long()
        K = inp_cpu.k_pool[pages].double().abs()                       # [npg, Hkv, 16, D]
        K = K.permute(1, 0, 2, 3).reshape(Hkv, npg * wl.PAGE, -1)
        qa = q_hat[b].double().abs().view(Hkv, G, -1)
        ad = torch.einsum("jnd,jgd->jgn", K, qa)
        out[b, :, : npg * wl.PAGE] = ad.sum(dim=1)                     # sum covers both max and sum aggregation
    return out
