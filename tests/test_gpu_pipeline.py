"""End to end on the GPU against the oracle chained the same way: producer -> statistic and rule -> scan at the routed
chunk -> one generated token from the carried states."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_10597_amd as corey
from gpu_util import assert_close, counts_u32, fp32_rtol, to_dev, upload
from paper_2604_10597_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
def test_layer_prefill_then_one_token(dtype):
    cfg = wl.scaled(wl.CONFIGS["c1_mamba130m"], D=40, L=1200, dtype=dtype, seqlens=None)
    print(f"[case] pipeline {cfg.name} B{cfg.B} D{cfg.D} L{cfg.L} {dtype}", flush=True)
    w = wl.make(cfg, a_kind="random")
    d = upload(w)
    conv = wl.make_conv(cfg, 4)
    x = to_dev(conv["dev"]["x"], dtype)
    cw, cb = torch.from_numpy(conv["dev"]["weight"]).cuda(), torch.from_numpy(conv["dev"]["bias"]).cuda()
    P = cfg.L - 1                                         # the last position is generated as one token

    # ---- GPU
    cut = lambda t: t[:, :, :P].contiguous()
    u, conv_state, parts = corey.causal_conv1d_silu_fwd(cut(x), cw, cb, want_state=True)
    route = corey.corey_route_device(u, cfg.K, corey.policy_default(), range_parts=parts)
    y, state = corey.selective_scan_fwd(u, cut(d["delta"]), d["A"], cut(d["B"]), cut(d["C"]), Dv=d["D"], z=cut(d["z"]),
                                        delta_bias=d["delta_bias"], chunk=512, chunks_dev=route["chunks"])
    u1, conv_state, _ = corey.causal_conv1d_silu_fwd(x[:, :, P:].contiguous(), cw, cb, state_in=conv_state, want_state=True)
    col = lambda t: t[:, :, P].contiguous()
    y1 = corey.selective_state_update(state, u1[:, :, 0].contiguous(), col(d["delta"]), d["A"], col(d["B"]), col(d["C"]),
                                      Dv=d["D"], z=col(d["z"]), delta_bias=d["delta_bias"])
    torch.cuda.synchronize()

    # ---- oracle, fed with the stored u of the GPU producer where the next stage reads it (each stage is held to its own
    # tolerance; the producer's own parity is checked first)
    xv = conv["val"]["x"]
    ref_u, ref_cs = oracle.causal_conv1d_silu(xv, conv["val"]["weight"], conv["val"]["bias"])
    u_all = torch.cat([u, u1], dim=2).float().cpu().numpy()
    bits = {wl.F32: 24, wl.BF16: 8}[dtype]
    assert np.all(np.abs(u_all - ref_u) <= 1e-5 * (1 + np.abs(ref_u)) + 2.0 ** -bits * np.abs(ref_u))
    assert np.array_equal(conv_state.float().cpu().numpy(), ref_cs)
    ent = oracle.entropy_hist(u_all[:, :, :P], cfg.K)
    assert np.array_equal(counts_u32(route["counts"]), ent["counts"])
    st, chunk, _ = oracle.select_chunk(float(ent["r"][0]), P, oracle.policy())
    assert st == oracle.OK and int(route["chunks"][0].item()) == chunk
    v = w.val
    st, y_ref, s_ref = oracle.selective_scan(u_all, v["delta"], v["A"], v["B"], v["C"], Dv=v["D"], z=v["z"],
                                             delta_bias=v["delta_bias"], chunk=chunk)
    assert st == oracle.OK
    rt = fp32_rtol(cfg.L) if dtype == wl.F32 else 3e-3
    sb = {wl.F32: 0, wl.BF16: 8}[dtype]
    assert_close(y.float().cpu().numpy(), y_ref[:, :, :P], rt, "y of the prompt", stored_bf16=sb)
    assert_close(y1.float().cpu().numpy(), y_ref[:, :, P], rt, "y of the generated token", stored_bf16=sb)
    assert_close(state.cpu().numpy(), s_ref, fp32_rtol(cfg.L), "state after the generated token")


def _scan_args(d):
    return dict(Dv=d["D"], z=d["z"], delta_bias=d["delta_bias"], seqlens=d["seqlens"])


@pytest.mark.parametrize("case", ["whole_tensor_batch", "per_sequence", "producer_exact", "producer_sampled"])
def test_deferred_route_equals_the_separate_reduction(case):
    """corey_route_device_deferred + selective_scan_fwd_routed (the statistic's reduction and the chunk rule inside the
    scan's first kernel) against corey_route_device + selective_scan_fwd: every output bit for bit, several calls in a
    row on the same buffers (the hand-over buffer's partial histograms must come back cleared each time)."""
    print(f"[case] deferred route: {case}", flush=True)
    pol = corey.policy_default()
    calls_a = torch.zeros(12, dtype=torch.int32, device="cuda")
    calls_b = torch.zeros(12, dtype=torch.int32, device="cuda")
    if case in ("whole_tensor_batch", "per_sequence"):
        lens = (1536, 40, 900) if case == "per_sequence" else None
        import dataclasses
        cfg = dataclasses.replace(wl.scaled(wl.CONFIGS["c3_mamba1p4b"], D=48, L=1536, B=3), seqlens=lens)
        pol.mode = 1 if lens else 0
        w = wl.make(cfg, a_kind="random")
        d = upload(w)
        u, parts, kw = d["u"], None, {}
        stat_seqlens = d["seqlens"]
    else:
        cfg = wl.scaled(wl.CONFIGS["c4_mamba2p8b"], D=320, L=2048, seqlens=None)
        w = wl.make(cfg, a_kind="random")
        d = upload(w)
        conv = wl.make_conv(cfg, 4)
        x = to_dev(conv["dev"]["x"], cfg.dtype)
        cw, cb = torch.from_numpy(conv["dev"]["weight"]).cuda(), torch.from_numpy(conv["dev"]["bias"]).cuda()
        u, _, parts = corey.causal_conv1d_silu_fwd(x, cw, cb)
        kw = dict(stride=8, block=512) if case == "producer_sampled" else {}
        stat_seqlens = None
    for rep in range(3):
        if parts is not None and rep == 2:                         # a fresh hand-over from the producer in between
            corey.causal_conv1d_silu_fwd(x, cw, cb, u=u, range_parts=parts)
        a = corey.corey_route_device(u, cfg.K, pol, seqlens=stat_seqlens, range_parts=parts, chunk_calls=calls_a, **kw)
        ya, sa = corey.selective_scan_fwd(u, d["delta"], d["A"], d["B"], d["C"], chunk=256, chunks_dev=a["chunks"], **_scan_args(d))
        b = corey.corey_route_device_deferred(u, cfg.K, pol, seqlens=stat_seqlens, range_parts=parts, chunk_calls=calls_b, **kw)
        yb, sb = corey.selective_scan_fwd(u, d["delta"], d["A"], d["B"], d["C"], chunk=256, route=b["route"], **_scan_args(d))
        torch.cuda.synchronize()
        for k in ("counts", "chunks", "range"):
            assert torch.equal(a[k], b[k]), (case, rep, k)
        for k in ("H", "r"):
            assert torch.equal(a[k].view(torch.int64), b[k].view(torch.int64)), (case, rep, k)
        assert torch.equal(ya.view(torch.int16), yb.view(torch.int16)) and torch.equal(sa, sb), (case, rep)
        assert int(a["counts"].sum()) > 0 and torch.equal(calls_a, calls_b)
    # and against the oracle once
    ref = oracle.entropy_hist(u.float().cpu().numpy(), cfg.K, seqlens=w.seqlens if case == "per_sequence" else None,
                              range_all=(case == "producer_sampled"), **kw)
    assert np.array_equal(counts_u32(b["counts"]).reshape(ref["counts"].shape), ref["counts"])
    nh = b["chunks"].numel()
    for h in range(nh):
        Lh = int(w.seqlens[h]) if case == "per_sequence" else cfg.L
        st, c, margin = oracle.select_chunk(float(ref["r"][h]), Lh, oracle.policy(mode=pol.mode))
        assert st == oracle.OK and (margin < 1e-9 and margin >= 0 or int(b["chunks"][h].item()) == c)


def test_deferred_route_argument_errors():
    x = torch.randn(2, 4, 64, device="cuda").bfloat16()
    out = corey.corey_route_device_deferred(x, 16)
    lib, ptr = corey.binding.lib(), corey.binding._ptr
    ws = torch.empty(corey.selective_scan_fwd_workspace(3, 16, 64), dtype=torch.uint8, device="cuda")
    t = torch.empty(8, device="cuda")
    # a route taken for a whole-tensor statistic or a batch of 2 does not fit a batch of 3 with per-sequence chunks: nh is 1: fine;
    # an empty ticket is refused
    empty = corey.binding.DeferredRoute()
    st = lib.selective_scan_fwd_routed(ptr(t), ptr(t), ptr(t), ptr(t), ptr(t), None, None, None, 1, None, None, 256, empty, ptr(t), ptr(t),
                                       1, 3, 4, 16, 64, 0, ptr(ws), ws.numel(), None)
    assert st == 1
    st = lib.selective_scan_fwd_routed(ptr(t), ptr(t), ptr(t), ptr(t), ptr(t), None, None, None, 1, None, None, 256, None, ptr(t), ptr(t),
                                       1, 3, 4, 16, 64, 0, ptr(ws), ws.numel(), None)
    assert st == 2
    st = lib.selective_scan_fwd_routed(ptr(t), ptr(t), ptr(t), ptr(t), ptr(t), None, None, None, 1, None, None, 256, out["route"], ptr(t),
                                       ptr(t), 1, 3, 4, 16, 64, 2, ptr(ws), ws.numel(), None)
    assert st == 1                                                # COREY_SCAN_ONE_CHUNK is not the caller's to set here
    torch.cuda.synchronize()
