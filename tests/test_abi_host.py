"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

from paper_2510_07486_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header="asyncspade.h"):
    hdr = open(os.path.join(ROOT, "include", header)).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    return sorted(set(re.findall(r"\b(as_[a-z_]+)\s*\(", hdr)))


def exported_symbols():
    """Every dynamic symbol the built library defines (nm -D)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", api.LIB_PATH], capture_output=True, text=True, check=True).stdout
    return sorted(ln.split()[-1] for ln in out.splitlines() if ln.strip())


def test_library_exports_exactly_the_declared_symbols():
    """Header and library agree in both directions: every declared entry point is exported, and nothing else is
    (no internal C++ symbol, no kernel stub, no undeclared knob).  The method's calls live in asyncspade.h, the
    development and measurement calls in asyncspade_debug.h."""
    L = api.lib()
    names = declared_symbols()
    debug = declared_symbols("asyncspade_debug.h")
    assert set(api.EXPORTS) == set(names)
    assert set(api.DEBUG_EXPORTS) == set(debug) and all(n.startswith("as_debug_") for n in debug)
    for n in names + debug:
        assert getattr(L, n) is not None
    assert exported_symbols() == sorted(names + debug)


def test_workspace_bytes_and_param_validation():
    p = api.make_params(32, 32, 8, 16, 2048, 2048)
    n = api.as_workspace_bytes(p)
    # q_hat + score rows + attention partials (one set per head: rows of this shape are not split)
    assert n >= 32 * 32 * 128 * 4 + 32 * 8 * 32768 * 4 + 32 * 32 * 130 * 4
    # the attention calls need only the leading part of the layout
    assert 32 * 32 * 130 * 4 <= api.as_workspace_bytes_attn(p) < n // 8
    # a forced split count (development knob) asks for that many partial sets
    assert api.attn_workspace_bytes_forced(p, 4) >= 32 * 32 * 4 * 130 * 4
    assert api.as_workspace_bytes_attn(api.make_params(1, 6, 4, 16, 64, 8)) == 0
    bad = api.make_params(1, 6, 4, 16, 64, 8)            # 6 % 4 != 0
    assert api.as_workspace_bytes(bad) == 0
    L = api.lib()
    dummy = C.c_void_p(0)
    for kw, code in [(dict(n_q_heads=6, n_kv_heads=4), 1), (dict(ridge_eps=0.0), 1), (dict(window=0), 1),
                     (dict(budget=0), 1), (dict(head_dim=64), 2), (dict(page_size=32), 2), (dict(window=65), 2),
                     (dict(budget=65537), 2), (dict(n_q_heads=65, n_kv_heads=1), 2), (dict(agg=7), 1), (dict(agg=3), 1),
                     (dict(predictor=2), 1), (dict(batch=65536), 2), (dict(n_q_heads=65536, n_kv_heads=65536), 2),
                     (dict(batch=65535, n_q_heads=65535, n_kv_heads=65535), 2),          # rows beyond 2^31 - 1
                     (dict(n_q_heads=17 * 40000, n_kv_heads=40000), 2),                  # attention grid.y beyond 65535
                     (dict(max_pages_per_seq=(1 << 25) // 16 + 1), 2)]:
        args = dict(batch=1, n_q_heads=8, n_kv_heads=2, window=4, budget=16, max_pages_per_seq=4)
        args.update(kw)
        q = api.make_params(**args)
        assert L.as_predict_query(dummy, C.byref(q), dummy, dummy, dummy, dummy) == code, kw
    ok = api.make_params(1, 8, 2, 4, 16, 4)
    # null ctx / null pointers are invalid arguments, reported without touching the device
    assert L.as_predict_query(None, C.byref(ok), None, None, None, None) == 1
    assert L.as_select_step(None, C.byref(ok), None, None, None, None, None, None) == 1
    assert L.as_status_str(3).decode() == "ctx workspace too small"


def test_pack_workspace_and_share_plan():
    """Host logic of the depth-wise packed selection: workspace sizes and the share plan."""
    L = api.lib()
    small = api.make_params(1, 8, 2, 8, 256, 256)          # workload c1 shape
    big = api.make_params(32, 32, 8, 16, 2048, 2048)       # workload c3 shape
    assert api.as_workspace_bytes_pack(small, 1) == api.as_workspace_bytes(small)
    assert api.as_workspace_bytes_pack(small, 0) == 0
    assert api.as_workspace_bytes_pack(small, api.AS_MAX_PACK + 1) == 0
    for n in range(2, api.AS_MAX_PACK + 1):                # one q_hat block per layer + the pack's candidates
        shares, cand = api.select_plan(small, n)[1:]
        need = n * 8 * 128 * 4 + (n * 2 * shares * (cand * 8 + 4) if shares > 1 else 0)
        assert api.as_workspace_bytes_pack(small, n) >= need
    # a batch that fills the chip keeps whole rows; a single short sequence is cut into shares, fewer
    # of them when more layers share the launch
    assert api.select_plan(big, 1)[1] == 1 and api.select_plan(big, 12)[1] == 1
    one, twelve = api.select_plan(small, 1), api.select_plan(small, 12)
    assert one[1] > twelve[1] >= 1
    for n in (1, 4, 16):
        share, shares, cand = api.select_plan(small, n)
        assert share * shares >= 4096 and share % 64 == 0 and cand == min(256, share)
    # a budget above half the candidate buffer forces buffer-sized shares: beyond 1024 of them per row there is no plan
    huge = api.make_params(1, 8, 2, 4, 5000, (1 << 25) // 16)
    assert api.select_plan(huge, 1)[1] > 1024
    # ... and then no candidate arrays are sized from it: the workspace is the score rows plus small change
    assert api.as_workspace_bytes(huge) < 2 * (1 << 25) * 4 + (8 << 20)
    # (single-layer calls then run the stand-alone stages; the softmax-normalised aggregation and packs, which
    # exist only in the fused kernels, are refused before anything touches the context or the device)
    huge_sm = api.make_params(1, 8, 2, 4, 5000, (1 << 25) // 16, agg=api.AS_AGG_SOFTMAX_SUM)
    assert L.as_score_topk(C.c_void_p(1), C.byref(huge_sm), C.byref(api.AsKvView(1, 1, 1, 1, 1)), C.c_void_p(1),
                           C.c_void_p(1), C.c_void_p(1), None) == 2
    fake = api.AsLayerIo(api.AsKvView(1, 1, 1, 1, 1), 1, 1, 1, 1)
    assert L.as_select_step_pack(C.c_void_p(1), C.byref(huge), (api.AsLayerIo * 2)(fake, fake), 2, None) == 2
    assert api.select_plan(api.make_params(1, 8, 2, 4, 4096, (1 << 25) // 16), 1)[1] <= 1024
    # null layer array / bad pack sizes are rejected before anything touches the device
    assert L.as_select_step_pack(None, C.byref(small), None, 1, None) == 1


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own, with no HIP or C++ in sight."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "asyncspade.h"\n'
                   "int main(void) { as_params p; as_kv_view kv; as_layer_io io; (void)p; (void)kv; (void)io;\n"
                   "  return (int)sizeof(as_status) > 0 && AS_MAX_PACK == 16 ? 0 : 1; }\n")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_share_plan_invariants_over_random_shapes():
    """Host planner: whatever the shape, the shares cover the longest context, respect the kernel's limits
    (share <= 32768 tokens; buffer-sized shares when the budget exceeds half the candidate buffer) and the workspace
    holds every candidate array the plan implies."""
    import random
    rnd = random.Random(7)
    for _ in range(300):
        hkv = rnd.choice([1, 2, 4, 8])
        g = rnd.choice([1, 2, 4, 8, 16, 24, 64])
        batch = rnd.choice([1, 2, 3, 8, 32, 64, 200])
        pages = rnd.choice([1, 7, 64, 256, 1024, 2048, 4096, 20000])
        budget = rnd.choice([1, 16, 256, 2048, 4096, 5000, 65536])
        layers = rnd.choice([1, 1, 2, 4, 16])
        agg = rnd.choice([0, 1, 2])
        p = api.make_params(batch, hkv * g, hkv, 16, budget, pages, agg=agg)
        share, shares, cand = api.select_plan(p, layers)
        max_ctx = pages * 16
        wide = g > 16 and agg != 1                     # MQA-sized groups run the 512-thread shape
        buf, cap = (4096, 16384) if wide else (8192, 65536)
        assert share * shares >= max_ctx and (shares - 1) * share < max(max_ctx, 1) or shares == 1
        assert 256 <= share <= cap and share % 64 == 0
        if budget > buf // 2:
            assert share <= buf
        assert cand == min(budget, share)
        if shares <= 1024:
            need = layers * batch * hkv * g * 128 * 4
            if shares > 1:
                need += layers * batch * hkv * shares * (cand * 8 + 4)
            if agg == 2:
                need += layers * batch * hkv * g * shares * 8
            assert api.as_workspace_bytes_pack(p, layers) >= need


def test_one_launch_selection_plan_invariants_over_random_shapes():
    """Host side of the one-launch selection over score rows: it serves only shapes its kernel can index (rows within
    the register top-k, groups of up to 16 heads unless the query is pre-summed, plain aggregation, one arrival counter
    per row); its shares are whole workgroup iterations of 32 pages, at most 1024 pages, cover the block table and keep
    the grid within one workgroup per compute unit unless a row is a single share; it is preferred only for at most
    128 rows and 2^20 tokens (or where no share of the fused kernel could prune); and a pack's workspace holds the
    pack's score rows whenever the pack takes it."""
    import random
    rnd = random.Random(11)
    seen_ok = seen_pref = 0
    for _ in range(400):
        hkv = rnd.choice([1, 2, 4, 8])
        g = rnd.choice([1, 2, 4, 8, 16, 24, 64])
        batch = rnd.choice([1, 2, 3, 8, 16, 32, 64, 200])
        pages = rnd.choice([0, 1, 7, 64, 256, 1024, 2048, 2049, 4096])
        budget = rnd.choice([1, 16, 256, 2048, 4096])
        layers = rnd.choice([1, 1, 2, 4, 12, 16])
        agg = rnd.choice([0, 0, 1, 2])
        p = api.make_params(batch, hkv * g, hkv, 16, budget, pages, agg=agg)
        ok, pref, share_pages, nshares = api.rows_plan(p, layers)
        rows = batch * hkv * layers
        if ok:
            seen_ok += 1
            assert agg != 2 and (agg == 1 or g <= 16)
            assert pages * 16 <= 32768 and rows <= 16384 and batch * layers <= 65535
            assert share_pages % 32 == 0 and 32 <= share_pages <= 1024
            assert share_pages * nshares >= pages and (nshares - 1) * share_pages < max(pages, 1)
            assert nshares == 1 or rows * nshares <= 256
        else:
            assert (share_pages, nshares) == (0, 0)
            assert agg == 2 or (agg == 0 and g > 16) or pages * 16 > 32768 or rows > 16384 or \
                (rows > 256 and pages > 1024) or (pages + max(1, 256 // rows) - 1) // max(1, 256 // rows) > 1024
        if pref:
            seen_pref += 1
            assert ok
            if layers > 1:
                assert rows <= 128 and rows * pages * 16 <= 1 << 20
                assert api.as_workspace_bytes_pack(p, layers) >= rows * pages * 16 * 4 + layers * batch * hkv * g * 128 * 4
    assert seen_ok > 50 and seen_pref > 20


def test_binding_fails_loudly_without_the_library(tmp_path, monkeypatch):
    """No CPU fallback anywhere above the C ABI: without the built library the binding raises, and neither the binding
    nor the pipeline module imports the oracle."""
    monkeypatch.setattr(api, "_lib", None)
    monkeypatch.setattr(api, "LIB_PATH", str(tmp_path / "libasyncspade.so"))
    with pytest.raises(RuntimeError, match="missing"):
        api.as_workspace_bytes(api.make_params(1, 8, 2, 8, 64, 16))
    with pytest.raises(RuntimeError, match="missing"):
        api.Context(api.make_params(1, 8, 2, 8, 64, 16))
    pkg = os.path.join(ROOT, "paper_2510_07486_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            src = open(os.path.join(pkg, name)).read()
            assert "import oracle" not in src and "from oracle" not in src, name
    for name in os.listdir(os.path.join(pkg, "csrc")):
        assert "oracle" not in open(os.path.join(pkg, "csrc", name)).read(), name
