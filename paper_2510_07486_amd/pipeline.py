"""The selection / attention schedule of one decode step on one GPU (Sec. 4.1 workflow, Sec. 4.3 feasibility
conditions), as reusable orchestration: streams, events and double-buffered selections.  No arithmetic happens
here; every piece of work is a call into the C ABI.

The paper runs selection on a second GPU (the cache rank) one step ahead of the model (the inference rank).  Here
the cache rank is a set of HIP streams: at decode step t the attention of layer l (attention stream) reads the
selection that was made during step t-1 from the query predicted for step t, and as soon as layer l's step-t
query, key and value exist, the selection of layer l for step t+1 starts on a selection stream.  Selections are
double-buffered (step t reads buffer t % 2 and writes buffer (t + 1) % 2) and handed over through events:
attention waits for exactly the selection it reads, a selection waits for the layer state it needs.  With
pack > 1 the selections of `pack` consecutive layers go out as one as_select_step_pack call once the pack's last
layer has its state (depth-wise packing, Sec. 4.3).
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Sequence

import torch

from . import api


@dataclasses.dataclass
class LayerState:
    """What one decoder layer contributes to a decode step; every tensor is caller-owned device memory and may be
    updated in place between steps (as_kv_append, as_window_push)."""
    kv: api.AsKvView
    q_win: torch.Tensor     # bf16 [B, Hq, W, 128], oldest first
    q_cur: torch.Tensor     # bf16 [B, Hq, 128]: this step's query = regression target
    q_attn: torch.Tensor    # bf16 [B, Hq, 128]: the query this step's attention runs with
    sel_ctx_lens: Optional[torch.Tensor] = None   # int32 [B] or None: tokens from here on are attended densely


class SelectionPipeline:
    def __init__(self, p: api.AsParams, layers: Sequence[LayerState], sel_streams: int = 2, pack: int = 1,
                 device: int = 0):
        self.p = p
        self.layers: List[LayerState] = list(layers)
        self.n_layers = len(self.layers)
        self.pack = max(1, min(pack, api.AS_MAX_PACK, self.n_layers))
        self.n_packs = (self.n_layers + self.pack - 1) // self.pack
        n_sel = max(1, sel_streams)
        dev = torch.device("cuda", device)
        B, Hq, Hkv, C = p.batch, p.n_q_heads, p.n_kv_heads, p.budget
        self.ctx_sel = [api.Context(p, device=device, pack=self.pack) for _ in range(n_sel)]
        self.ctx_att = api.Context(p, device=device)
        self.s_sel = [torch.cuda.Stream(device=dev) for _ in range(n_sel)]
        self.s_att = torch.cuda.Stream(device=dev)
        self.q_hat = [torch.empty((B, Hq, p.head_dim), dtype=torch.float32, device=dev) for _ in range(n_sel)]
        # sel[parity][layer] = (sel_idx, sel_cnt)
        self.sel = [[(torch.empty((B, Hkv, C), dtype=torch.int32, device=dev),
                      torch.empty((B, Hkv), dtype=torch.int32, device=dev)) for _ in range(self.n_layers)]
                    for _ in range(2)]
        self._pack_ios = None
        if self.pack > 1:
            self._pack_ios = [[self._make_pack(parity, g) for g in range(self.n_packs)] for parity in range(2)]
        # recorded on a selection stream when a pack's selection into sel[parity] is complete
        self._sel_done = [[None] * self.n_packs for _ in range(2)]
        # hand-over events, made once and recorded again every step (a wait refers to the record that precedes it in
        # program order): creating two events per layer and step costs more host time than a small layer's kernels
        self._ready_ev = [torch.cuda.Event() for _ in range(self.n_packs)]
        self._done_ev = [[torch.cuda.Event() for _ in range(self.n_packs)] for _ in range(2)]

    # ------------------------------------------------------------------ pieces
    def _pack_range(self, g: int):
        return range(g * self.pack, min(self.n_layers, (g + 1) * self.pack))

    def _make_pack(self, parity: int, g: int):
        ios = [api.layer_io(self.layers[l].kv, self.layers[l].q_win, self.layers[l].q_cur,
                            self.sel[parity][l][0], self.sel[parity][l][1]) for l in self._pack_range(g)]
        arr = (api.AsLayerIo * len(ios))(*ios)
        arr._keep_alive = ios
        return arr

    def select_layer(self, l: int, parity: int, stream, lane: int = 0, events=None):
        """Selection of layer l into buffer `parity`.  With `events` (a pair of timing events) the predictor and the
        K-streaming part are issued as the two calls as_select_step makes, the second bracketed by the events."""
        L = self.layers[l]
        idx, cnt = self.sel[parity][l]
        if events is None:
            api.as_select_step(self.ctx_sel[lane], self.p, L.kv, L.q_win, L.q_cur, idx, cnt, stream=stream)
            return
        api.as_predict_query(self.ctx_sel[lane], self.p, L.q_win, L.q_cur, self.q_hat[lane], stream=stream)
        events[0].record(stream)
        api.as_score_topk(self.ctx_sel[lane], self.p, L.kv, self.q_hat[lane], idx, cnt, stream=stream)
        events[1].record(stream)

    def select_pack(self, g: int, parity: int, stream, lane: int = 0, events=None):
        if events is not None:
            events[0].record(stream)
        api.as_select_step_pack(self.ctx_sel[lane], self.p, self._pack_ios[parity][g], stream=stream)
        if events is not None:
            events[1].record(stream)

    def attend(self, l: int, parity: int, out: torch.Tensor, stream, lse: Optional[torch.Tensor] = None):
        L = self.layers[l]
        idx, cnt = self.sel[parity][l]
        api.as_sparse_decode_attn(self.ctx_att, self.p, L.kv, L.q_attn, idx, cnt, L.sel_ctx_lens, out=out, lse=lse,
                                  stream=stream, want_lse=lse is not None)

    # ------------------------------------------------------------------ schedules
    def prime(self):
        """Fills both selection buffers from the current layer state (what a prefill would leave behind)."""
        for parity in range(2):
            for l in range(self.n_layers):
                self.select_layer(l, parity, self.s_sel[0])
        torch.cuda.synchronize()

    def step(self, t: int, outs, timing=None, join: bool = False):
        """Enqueues decode step t: attention of every layer on the attention stream, the selections for step t + 1 on
        the selection streams.  outs: one output tensor, or one per layer.  timing: a list that receives one pair
        of timing events per selection call.  join=True (stream capture: events cannot cross graph launches) makes
        the attention stream wait for every selection stream at the end of the step instead of handing over
        per-pack events to the next step."""
        cur, nxt = t % 2, (t + 1) % 2
        per_layer = isinstance(outs, (list, tuple))
        for l in range(self.n_layers):
            g = l // self.pack
            if l % self.pack == 0 and self._sel_done[cur][g] is not None and not join:
                self.s_att.wait_event(self._sel_done[cur][g])
            if l == self._pack_range(g)[-1]:           # a pack is selected once its last layer's state exists
                lane = g % len(self.s_sel)
                ready = self._ready_ev[g]
                ready.record(self.s_att)               # layer l's step-t state exists from here on; every earlier
                self.s_sel[lane].wait_event(ready)     # reader of buffer `nxt` has been enqueued before it
                pair = None
                if timing is not None:
                    pair = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                    timing.append(pair)
                if self.pack > 1:
                    self.select_pack(g, nxt, self.s_sel[lane], lane, pair)
                else:
                    self.select_layer(l, nxt, self.s_sel[lane], lane, pair)
                if not join:
                    done = self._done_ev[nxt][g]
                    done.record(self.s_sel[lane])
                    self._sel_done[nxt][g] = done
            self.attend(l, cur, outs[l] if per_layer else outs, self.s_att)
        if join:
            for s in self.s_sel:
                done = torch.cuda.Event()
                done.record(s)
                self.s_att.wait_event(done)

    def step_serial(self, t: int, outs, timing=None, stream=None):
        """The same work in single-stream order (select, then attend, layer by layer): the reference schedule."""
        stream = stream or self.s_att
        cur, nxt = t % 2, (t + 1) % 2
        per_layer = isinstance(outs, (list, tuple))
        for l in range(self.n_layers):
            g = l // self.pack
            if l == self._pack_range(g)[-1]:
                pair = None
                if timing is not None:
                    pair = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                    timing.append(pair)
                if self.pack > 1:
                    self.select_pack(g, nxt, stream, 0, pair)
                else:
                    self.select_layer(l, nxt, stream, 0, pair)
            self.attend(l, cur, outs[l] if per_layer else outs, stream)

    def fork(self):
        """Inside a stream capture that started on the attention stream: brings the selection streams in."""
        for s in self.s_sel:
            s.wait_stream(self.s_att)
