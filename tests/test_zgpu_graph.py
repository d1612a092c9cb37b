"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset nodes), so a
caller can capture the path in a HIP graph.  Each graph is replayed several times with new inputs and ordinary eager work
and synchronisations in between, and every replay is checked against the eager result."""
import numpy as np
import pytest
import torch

import paper_2604_10597_amd as corey
from gpu_util import to_dev, upload
from paper_2604_10597_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[case] {msg}", flush=True)


def test_producer_routing_and_scan_replayed_from_a_graph():
    cfg = wl.scaled(wl.CONFIGS["c4_mamba2p8b"], D=256, L=4096, seqlens=None)
    _say(f"graph: conv -> route -> scan {cfg.name} D{cfg.D} L{cfg.L}")
    w = wl.make(cfg, a_kind="random")
    d = upload(w)
    conv = wl.make_conv(cfg, 4)
    xs = [to_dev(conv["dev"]["x"], cfg.dtype)]
    for k in (1, 2):                                   # two more inputs with other ranges, hence other entropies
        xs.append((xs[0].float() * (1.0 + 3.0 * k) * (torch.rand_like(xs[0].float()) < 0.5 / k)).to(xs[0].dtype))
    wt, bs = torch.from_numpy(conv["dev"]["weight"]).cuda(), torch.from_numpy(conv["dev"]["bias"]).cuda()
    pol = corey.policy_default()

    x = xs[0].clone()
    u = torch.empty_like(x)
    y = torch.empty_like(x)
    last = torch.empty((cfg.B, cfg.D, cfg.N), dtype=torch.float32, device="cuda")
    parts = torch.empty(corey.binding.HANDOFF_BYTES, dtype=torch.uint8, device="cuda")
    ent = corey.corey_route_device(u, cfg.K, pol)      # allocates the outputs and the workspace once, outside the graph
    ws = torch.empty(corey.selective_scan_fwd_workspace(cfg.B, cfg.N, cfg.L), dtype=torch.uint8, device="cuda")

    def path():
        corey.causal_conv1d_silu_fwd(x, wt, bs, u=u, range_parts=parts)
        corey.corey_route_device(u, cfg.K, pol, out=ent, workspace=ent["workspace"], range_parts=parts)
        corey.selective_scan_fwd(u, d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"], delta_bias=d["delta_bias"],
                                 chunk=256, chunks_dev=ent["chunks"], y=y, last_state=last, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        path()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        path()

    seen = set()
    for rep in range(4):
        src = xs[rep % 3]
        x.copy_(src)
        path()                                          # eager
        torch.cuda.synchronize()
        want = (u.clone(), y.clone(), last.clone(), ent["chunks"].clone(), ent["counts"].clone(), ent["H"].clone())
        for t in (u, y, last, ent["chunks"], ent["counts"]):
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = (u, y, last, ent["chunks"], ent["counts"], ent["H"])
        for name, a, b in zip(("u", "y", "last", "chunks", "counts", "H"), got, want):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {rep}: {name} differs from the eager run"
        seen.add(int(ent["chunks"][0].item()))
    assert len(seen) >= 2, f"the inputs were meant to route to different chunks, saw {seen}"


def test_generation_steps_replayed_from_a_graph():
    T = 5
    cfg = wl.Config(name="dec_graph", B=3, D=640, N=16, L=1, dtype=wl.BF16, K=16, chunks=(64,), seed=77)
    _say(f"graph: {T} decode steps B{cfg.B} D{cfg.D}")
    c = wl.make_decode(cfg, a_kind="random")
    g = {k: to_dev(v, cfg.dtype) for k, v in c["dev"].items()}
    toks = [{k: (g[k].float() * (0.5 + 0.25 * t)).to(g[k].dtype) for k in ("x", "delta", "z", "Bt", "Ct")} for t in range(T)]
    state = g["state"].clone()
    ys = [torch.empty_like(g["x"]) for _ in range(T)]

    def steps():
        for t in range(T):
            k = toks[t]
            corey.selective_state_update(state, k["x"], k["delta"], g["A"], k["Bt"], k["Ct"], Dv=g["D"], z=k["z"],
                                         delta_bias=g["delta_bias"], y=ys[t])

    steps()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        steps()
    for rep in range(3):
        state.copy_(g["state"] * (1.0 + rep))
        steps()
        torch.cuda.synchronize()
        want = [state.clone()] + [t.clone() for t in ys]
        state.copy_(g["state"] * (1.0 + rep))
        for t in ys:
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip([state] + ys, want)):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {rep}: tensor {i} differs from the eager run"
