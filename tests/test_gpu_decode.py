"""GPU parity: selective_state_update (one generated token) against the CPU oracle, alone and after a prompt."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_10597_amd as corey
from gpu_util import assert_close, fp32_rtol, store_bits, to_dev, upload
from paper_2604_10597_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[case] {msg}", flush=True)


def _step(cfg, a_kind="mamba", use_z=True, use_bias=True, use_D=True, softplus=True):
    c = wl.make_decode(cfg, a_kind=a_kind)
    dev, val = c["dev"], c["val"]
    if not softplus:                       # the raw value is the step size then: keep it positive (clearing a sign is exact)
        use_bias = False
        dev["delta"] = dev["delta"] & np.uint16(0x7FFF) if dev["delta"].dtype == np.uint16 else np.abs(dev["delta"])
        val["delta"] = np.abs(val["delta"])
    g = {k: to_dev(v, cfg.dtype) for k, v in dev.items()}
    state = g["state"].clone()
    y = corey.selective_state_update(state, g["x"], g["delta"], g["A"], g["Bt"], g["Ct"], Dv=g["D"] if use_D else None,
                                     z=g["z"] if use_z else None, delta_bias=g["delta_bias"] if use_bias else None,
                                     delta_softplus=softplus)
    torch.cuda.synchronize()
    ref_s, ref_y = oracle.selective_state_update(val["state"], val["x"], val["delta"], val["A"], val["Bt"], val["Ct"],
                                                 Dv=val["D"] if use_D else None, z=val["z"] if use_z else None,
                                                 delta_bias=val["delta_bias"] if use_bias else None, delta_softplus=softplus)
    # one step in binary32: the tolerance of the scan's shortest configuration
    assert_close(state.cpu().numpy(), ref_s, fp32_rtol(1), "state")
    assert_close(y.float().cpu().numpy(), ref_y, fp32_rtol(1), "y", stored_bf16=store_bits(cfg))


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16, wl.F16])
@pytest.mark.parametrize("N", [1, 3, 4, 16, 23, 64, 100, 256])
def test_parity_over_state_sizes_and_types(dtype, N):
    for B, D in ((1, 1), (2, 37), (3, 300)):
        _say(f"decode B{B} D{D} N{N} {dtype}")
        cfg = wl.Config(name="dec", B=B, D=D, N=N, L=1, dtype=dtype, K=16, chunks=(64,), seed=31 * N + B)
        _step(cfg, a_kind="random" if N % 2 else "mamba")


def test_optional_arguments():
    cfg = wl.Config(name="dec", B=2, D=65, N=16, L=1, dtype=wl.BF16, K=16, chunks=(64,), seed=9)
    for kw in ({"use_z": False}, {"use_bias": False}, {"use_D": False}, {"softplus": False}):
        _say(f"decode options {kw}")
        _step(cfg, **kw)


def test_batched_decode_at_the_benchmark_size():
    cfg = wl.scaled(wl.CONFIGS["c4_mamba2p8b"], B=64, L=1, seqlens=None)
    _say(f"decode full B{cfg.B} D{cfg.D} N{cfg.N}")
    _step(cfg)


def test_generation_continues_a_prompt():
    """Prompt through selective_scan_fwd, then 6 tokens one at a time from its last_state: the outputs and the final state
    are those of the oracle's scan over the whole sequence."""
    T = 6
    cfg = wl.scaled(wl.CONFIGS["c1_mamba130m"], D=48, L=300 + T, seqlens=None)
    _say(f"prompt + generation {cfg.name} D{cfg.D} L{cfg.L}")
    w = wl.make(cfg, a_kind="random")
    st, y_ref, last_ref = oracle.selective_scan(w.val["u"], w.val["delta"], w.val["A"], w.val["B"], w.val["C"], Dv=w.val["D"],
                                                z=w.val["z"], delta_bias=w.val["delta_bias"], chunk=64, threads=8)
    assert st == oracle.OK
    d = upload(w)
    P = cfg.L - T
    cut = lambda t: t[:, :, :P].contiguous()
    y, last = corey.selective_scan_fwd(cut(d["u"]), cut(d["delta"]), d["A"], cut(d["B"]), cut(d["C"]), Dv=d["D"], z=cut(d["z"]),
                                       delta_bias=d["delta_bias"], chunk=64)
    ys = [y.float()]
    for t in range(P, cfg.L):
        col = lambda a: a[:, :, t].contiguous()
        yt = corey.selective_state_update(last, col(d["u"]), col(d["delta"]), d["A"], col(d["B"]), col(d["C"]), Dv=d["D"],
                                          z=col(d["z"]), delta_bias=d["delta_bias"])
        ys.append(yt.float().unsqueeze(2))
    torch.cuda.synchronize()
    got = torch.cat(ys, dim=2).cpu().numpy()
    assert_close(got, y_ref, fp32_rtol(cfg.L) if cfg.dtype == wl.F32 else 3e-3, "y over prompt and generated tokens",
                 stored_bf16=store_bits(cfg))
    assert_close(last.cpu().numpy(), last_ref, fp32_rtol(cfg.L), "state after the last generated token")
