"""The decode-step schedule of paper_2510_07486_amd/pipeline.py, checked on the CPU as a dependency graph: streams
and events are replaced by vector clocks, the library calls by recorders.  For per-layer and packed selection, one or
two selection streams, event hand-off and the join mode used under stream capture:
  * every attention call happens after the selection that wrote the buffer it reads (read after write),
  * every selection happens after the previous step's attention calls that read the buffer it overwrites
    (write after read), and after the attention call that marks its last layer's state as ready,
  * both hold across steps, which is where double buffering can go wrong.
GPU tests compare results; this one shows the results are not a matter of timing."""
import types

import pytest
import torch

from paper_2510_07486_amd import api, pipeline


class Stream:
    count = 0
    every = []

    def __init__(self, device=None):
        Stream.count += 1
        self.name = f"s{Stream.count}"
        self.clock = {}
        Stream.every.append(self)

    @staticmethod
    def synchronize():
        """A device-wide synchronisation: everything enqueued so far precedes everything enqueued later."""
        top = {}
        for s in Stream.every:
            for k, v in s.clock.items():
                top[k] = max(top.get(k, 0), v)
        for s in Stream.every:
            s.clock = dict(top)

    def tick(self):
        self.clock[self.name] = self.clock.get(self.name, 0) + 1
        return dict(self.clock)

    def merge(self, vc):
        for k, v in vc.items():
            self.clock[k] = max(self.clock.get(k, 0), v)

    def wait_event(self, ev):
        assert ev.vc is not None, "waiting for an event that was never recorded"
        self.merge(ev.vc)

    def wait_stream(self, other):
        self.merge(other.clock)


class Event:
    def __init__(self, enable_timing=False):
        self.vc = None

    def record(self, stream):
        self.vc = dict(stream.clock)


def before(a, b):
    """op a happens before op b"""
    return a["vc"][a["stream"]] <= b["vc"].get(a["stream"], 0)


@pytest.fixture
def recorder(monkeypatch):
    log = []
    Stream.every.clear()
    shim = types.SimpleNamespace(
        device=lambda *a: "cpu",
        empty=lambda *a, device=None, **k: torch.empty(*a, **k),
        cuda=types.SimpleNamespace(Stream=Stream, Event=Event, synchronize=Stream.synchronize),
        int32=torch.int32, float32=torch.float32, Tensor=torch.Tensor)
    monkeypatch.setattr(pipeline, "torch", shim)

    class Ctx:
        def __init__(self, p, device=0, pack=1):
            pass

    def op(kind, stream, **kw):
        log.append(dict(kind=kind, stream=stream.name, vc=stream.tick(), **kw))

    monkeypatch.setattr(api, "Context", Ctx)
    monkeypatch.setattr(api, "as_select_step",
                        lambda c, p, kv, qw, qc, idx, cnt, stream=None: op("select", stream, bufs=[idx.data_ptr()]))
    monkeypatch.setattr(api, "as_predict_query", lambda c, p, qw, qc, qh, stream=None: op("predict", stream))
    monkeypatch.setattr(api, "as_score_topk",
                        lambda c, p, kv, qh, idx, cnt, stream=None: op("select", stream, bufs=[idx.data_ptr()]))
    monkeypatch.setattr(api, "as_select_step_pack",
                        lambda c, p, ios, stream=None: op("select", stream, bufs=[io.sel_idx for io in ios]))
    monkeypatch.setattr(api, "as_sparse_decode_attn",
                        lambda c, p, kv, q, idx, cnt, tail, out=None, lse=None, stream=None, want_lse=True:
                        op("attend", stream, bufs=[idx.data_ptr()]))
    return log


@pytest.mark.parametrize("n_layers,pack,sel_streams,join,timing", [
    (5, 1, 2, False, False), (5, 1, 1, False, True), (6, 2, 2, False, False), (7, 3, 2, False, True),
    (4, 4, 1, False, False), (5, 1, 2, True, False), (7, 3, 2, True, False), (1, 1, 2, False, False)])
def test_schedule_orders_every_read_and_write_of_the_selection_buffers(recorder, n_layers, pack, sel_streams, join, timing):
    p = api.make_params(2, 8, 2, 4, 16, 8)
    kv = api.AsKvView(1, 1, 1, 1, 1)
    t = torch.zeros(1)
    layers = [pipeline.LayerState(kv, t, t, t) for _ in range(n_layers)]
    pipe = pipeline.SelectionPipeline(p, layers, sel_streams=sel_streams, pack=pack)
    owner = {pipe.sel[par][l][0].data_ptr(): (par, l) for par in range(2) for l in range(n_layers)}
    pipe.prime()
    marks = [len(recorder)]
    n_steps = 5
    for step in range(n_steps):
        if join:
            pipe.fork()
        pipe.step(step, t, timing=[] if timing else None, join=join)
        marks.append(len(recorder))
    ops = [dict(o, step=next(s for s in range(-1, n_steps) if i < marks[s + 1])) for i, o in enumerate(recorder)]
    attends = [o for o in ops if o["kind"] == "attend"]
    selects = [o for o in ops if o["kind"] == "select"]
    assert len(attends) == n_steps * n_layers
    # one selection call per pack and step, after the priming ones
    assert len([s for s in selects if s["step"] >= 0]) == n_steps * ((n_layers + pack - 1) // pack)
    for a in attends:
        (par, l), = [owner[b] for b in a["bufs"]]
        assert par == a["step"] % 2
        writers = [s for s in selects if (par, l) in [owner[b] for b in s["bufs"]] and s["step"] < a["step"]]
        last_writer = writers[-1]
        assert last_writer["step"] == a["step"] - 1 or last_writer["step"] == -1 and a["step"] < 2
        assert before(last_writer, a), ("read before write", a["step"], l)
    for s in selects:
        if s["step"] < 0:
            continue
        for par, l in [owner[b] for b in s["bufs"]]:
            assert par == (s["step"] + 1) % 2
            readers = [a for a in attends if owner[a["bufs"][0]] == (par, l) and a["step"] == s["step"] - 1]
            for a in readers:
                assert before(a, s), ("overwritten while still being read", s["step"], l)
            later = [a for a in attends if owner[a["bufs"][0]] == (par, l) and a["step"] == s["step"] + 1]
            for a in later:
                assert before(s, a)
        # the pack's last layer must have been reached by the attention stream of this step
        last_layer = max(l for _, l in [owner[b] for b in s["bufs"]])
        if last_layer > 0:
            prev_att = [a for a in attends if a["step"] == s["step"] and owner[a["bufs"][0]][1] == last_layer - 1]
            assert before(prev_att[0], s)
