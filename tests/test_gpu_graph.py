"""The whole tower step captured in a HIP graph and replayed.

The library's hot calls only enqueue kernels on the caller's stream (no allocation, no
synchronisation, no memset nodes), so a caller can capture lookup -> training forward -> Tower
Module backward -> sparse update once and replay it.  Every replay, with eager work and
synchronisations in between, must leave the tables, the optimizer states and the outputs exactly
where the same number of eager steps leaves them (the path is bit-reproducible).
"""
import numpy as np
import pytest
import torch

import workloads as wl
from harness import DeviceWorkload, TowerModules

pytestmark = pytest.mark.gpu


def _make(w):
    dw = DeviceWorkload(w, with_state=True)
    tm = TowerModules(dw)
    dmt = dw.dmt
    B = w.batch
    idx, off = wl.lookup_batch(w)
    st = dict(dw=dw, tm=tm, B=B,
              idx=torch.from_numpy(idx).cuda(), off=torch.from_numpy(off).cuda(),
              dy=torch.from_numpy(wl.grad_tm_out(w)).cuda())
    f32 = lambda *shape: torch.zeros(shape, dtype=torch.float32, device="cuda")
    widths = w.tower_widths()
    grads = [dict(dw_proj=f32(o, k), db_proj=f32(o)) for o, k in zip(w.tm_out, w.tm_in_dims())]
    st["grads"] = grads
    st["arr"] = dmt.make_tm_grads(grads)
    st["pooled"] = torch.zeros(B * sum(widths), dtype=torch.bfloat16 if tm.dtype == "bf16" else
                               (torch.float16 if tm.dtype == "f16" else torch.float32), device="cuda")
    st["y"] = torch.zeros(B * sum(w.tm_out), dtype=st["pooled"].dtype, device="cuda")
    st["dx"] = torch.zeros(B * sum(widths), dtype=torch.float32, device="cuda")
    nk = dmt.dmt_tm_kept_bytes(dw.plan, tm.params, B, tm.dtype)
    st["kept"] = torch.empty(nk, dtype=torch.uint8, device="cuda") if nk else None
    st["ws_bwd"] = torch.empty(dmt.dmt_tm_bwd_workspace_bytes(dw.plan, tm.params, B), dtype=torch.uint8, device="cuda")
    st["ws_upd"] = torch.empty(max(dmt.dmt_bwd_workspace_bytes(dw.plan, B, len(idx)), 256), dtype=torch.uint8,
                               device="cuda")
    return st


def _step(st):
    dw, tm, B = st["dw"], st["tm"], st["B"]
    dmt, w = dw.dmt, dw.w
    dmt.dmt_tower_lookup_fwd(dw.plan, st["idx"], st["off"], B, st["pooled"])
    dmt.dmt_tower_module_fwd_keep(dw.plan, tm.params, st["pooled"], B, st["y"], st["kept"], tm.workspace)
    dmt.dmt_tower_module_bwd(dw.plan, tm.params, st["pooled"], st["y"], B, st["dy"], st["dx"], st["arr"],
                             st["ws_bwd"], kept=st["kept"])
    dmt.dmt_tower_lookup_bwd_update(dw.plan, st["idx"], st["off"], B, st["dx"], w.lr, w.eps, st["ws_upd"])


def _snapshot(st):
    dw = st["dw"]
    return ([t.clone() for t in dw.tables], [s.clone() for s in dw.states], st["y"].clone(), st["dx"].clone(),
            [g["dw_proj"].clone() for g in st["grads"]])


@pytest.mark.parametrize("which", ["tiny", "mid"])
def test_captured_step_replays_like_eager_steps(which):
    w = wl.tiny() if which == "tiny" else wl.scaled(wl.mid(True), max_rows=5000, batch=301, num_tables=16)
    eager, graphed = _make(w), _make(w)
    # reference: eager steps, snapshot after each
    refs = []
    for _ in range(4):
        _step(eager)
        torch.cuda.synchronize()
        refs.append(_snapshot(eager))
    # one eager warm-up step on the graphed copy (first-call set-up happens outside the capture)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        _step(graphed)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        _step(graphed)
    torch.cuda.synchronize()
    # the capture itself ran nothing: the copy is one step in; replays take it to 2, 3, 4
    for n in range(1, 4):
        g.replay()
        torch.cuda.synchronize()
        scratch = torch.randn(1 << 16, device="cuda").sum().item()      # eager work between replays
        assert np.isfinite(scratch)
        got = _snapshot(graphed)
        want = refs[n]
        for a, b in zip(got[0] + got[1] + [got[2], got[3]] + got[4], want[0] + want[1] + [want[2], want[3]] + want[4]):
            bits = {2: torch.int16, 4: torch.int32}[a.element_size()]
            assert torch.equal(a.view(bits), b.view(bits)), "replay %d differs from %d eager steps" % (n, n + 1)
    assert graphed["dw"].dmt.dmt_last_device_error(graphed["dw"].plan) == -1


def test_partitioner_and_shuffle_calls_capture_too():
    """dmt_tp_interaction and the SPTT shuffle steps also only enqueue kernels: captured after one
    eager call each, every replay on fresh pooled values gives the eager result bit for bit."""
    import paper_2403_00877_amd as dmt
    w = wl.scaled(wl.mid(), max_rows=3000, batch=256, num_tables=16)
    dw = DeviceWorkload(w)
    F, B = w.num_tables, w.batch
    n = B * sum(w.tower_widths())
    pooled = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    I = torch.zeros(F, F, dtype=torch.float32, device="cuda")
    ws = torch.empty(dmt.dmt_tp_workspace_bytes(dw.plan, B), dtype=torch.uint8, device="cuda")
    src = pooled.view(torch.uint8)
    permuted, shuffled = torch.zeros_like(src), torch.zeros_like(src)
    block = src.numel() // (F * 8)

    def calls():
        dmt.dmt_tp_interaction(dw.plan, pooled, B, I, ws)
        dmt.dmt_sptt_peer_permute(src, permuted, F, 8, 4, block)
        dmt.dmt_sptt_shuffle(src, shuffled, F, 8, block)

    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    pooled.copy_(torch.randn(n, generator=g, device="cuda"))
    calls()                                          # eager warm-up
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        calls()
    for _ in range(3):
        pooled.copy_(torch.randn(n, generator=g, device="cuda"))   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (I.clone(), permuted.clone(), shuffled.clone())
        I.zero_(); permuted.zero_(); shuffled.zero_()
        calls()
        torch.cuda.synchronize()
        for a, b in zip(got, (I, permuted, shuffled)):
            assert torch.equal(a, b)
        assert float(I.diagonal().min()) > 0.99
