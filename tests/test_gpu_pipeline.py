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
