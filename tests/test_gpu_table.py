"""GPU parity: the one-sweep statistic of a 16-bit tensor (bit-pattern table) against the CPU oracle's two-pass
histogram: counts bit for bit, H and r to summation rounding, range exactly; also with the table filled by the
producer of u (no pass over u at all)."""
import dataclasses
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2604_10597_amd as corey
from gpu_util import counts_u32, to_dev
from paper_2604_10597_amd import workloads as wl

pytestmark = pytest.mark.gpu
_WS = {}


def _say(msg):
    print(f"[case] {msg}", flush=True)


def _ws():
    if "t" not in _WS:
        _WS["t"] = torch.empty(corey.corey_pattern_table_workspace(), dtype=torch.uint8, device="cuda")
    return _WS["t"]


def _compare(out, ref, K):
    assert np.array_equal(counts_u32(out["counts"]).reshape(-1), ref["counts"].reshape(-1)), "bin counts differ"
    H, r, rng = out["H"].item(), out["r"].item(), out["range"].cpu().numpy().reshape(-1)
    if math.isnan(ref["H"][0]):
        assert math.isnan(H) and math.isnan(r)
    else:
        assert H == pytest.approx(ref["H"][0], rel=1e-12, abs=1e-14) and r == pytest.approx(ref["r"][0], rel=1e-12, abs=1e-14)
        assert rng[0] == ref["lo"][0] and rng[1] == ref["hi"][0]


def _check(x_store, x_val, dtype, K, eps=1e-8, xd=None):
    xd = to_dev(x_store, dtype) if xd is None else xd
    out = corey.corey_entropy_hist_onesweep(xd, K, eps=eps, table_ws=_ws())
    torch.cuda.synchronize()
    ref = oracle.entropy_hist(x_val, K, eps=eps)
    _compare(out, ref, K)
    return out, ref


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
@pytest.mark.parametrize("name,D,L", [("c1_mamba130m", 96, 2048), ("c2_mamba370m", 64, 1000), ("c3_mamba1p4b", 48, 1024),
                                       ("c4_mamba2p8b", 300, 512), ("paper_w1_fp16", 64, 777)])
def test_configs_at_oracle_size(name, D, L, dtype):
    cfg = dataclasses.replace(wl.scaled(wl.CONFIGS[name], D=D, L=L, dtype=dtype), seqlens=None)
    _say(f"one-sweep {cfg.name} B{cfg.B} D{D} L{L} {dtype}")
    w = wl.make(cfg, with_z=False)
    for K in (cfg.K, 2, 17, 4096):
        _check(w.dev["u"], w.val["u"], dtype, K)


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 3, 7), (2, 5, 37), (3, 4, 2049), (1, 2, 4104)])
def test_ragged_and_unaligned(dtype, shape):
    _say(f"one-sweep ragged {shape} {dtype}")
    rng = np.random.default_rng(sum(shape))
    store, val = wl.store(rng.standard_normal(shape).astype(np.float32), dtype)
    _check(store, val, dtype, 16)
    # the same values at every 2-byte offset inside a 16-byte word: single elements before and after the aligned body
    n = store.size
    for off in (1, 3, 7):
        buf = torch.zeros(n + 8, dtype=torch.int16, device="cuda")
        buf[off:off + n] = torch.from_numpy(store.reshape(-1).view(np.int16)).cuda()
        view = buf[off:off + n].view(torch.bfloat16 if dtype == wl.BF16 else torch.float16).reshape(shape)
        assert view.data_ptr() % 16 == (2 * off) % 16
        out = corey.corey_entropy_hist_onesweep(view, 16, table_ws=_ws())
        torch.cuda.synchronize()
        _compare(out, oracle.entropy_hist(val, 16), 16)


def test_sparse_constant_and_nonfinite_inputs():
    """Patterns that occur more often than a 15-bit counter holds (the overflow list), a tensor of zeros with a few
    values (the zero pattern's own counter), constant tensors, signed zeros, NaN and infinity."""
    rng = np.random.default_rng(5)
    _say("one-sweep sparse 2 % non-zero")
    x = np.where(rng.random((2, 64, 8192)) < 0.02, rng.standard_normal((2, 64, 8192)), 0.0).astype(np.float32)
    for dtype in (wl.BF16, wl.F16):
        store, val = wl.store(x, dtype)
        _check(store, val, dtype, 256)
    _say("one-sweep three values, 1.3 M elements")                  # each pattern overflows a counter many times over
    x = rng.choice(np.array([-1.5, 0.25, 3.0], dtype=np.float32), size=(1, 160, 8192), p=[0.7, 0.2, 0.1])
    store, val = wl.store(x, wl.BF16)
    out, ref = _check(store, val, wl.BF16, 64)
    assert ref["counts"].max() > 65536 * 8
    _say("one-sweep constant")
    const = np.full((1, 40, 4096), 2.5, dtype=np.float32)
    store, val = wl.store(const, wl.BF16)
    out, _ = _check(store, val, wl.BF16, 8)
    assert counts_u32(out["counts"])[0, 0] == const.size
    zeros = np.zeros((1, 8, 1024), dtype=np.float32)
    zeros[0, 3, 5] = -0.0
    store, val = wl.store(zeros, wl.F16)
    out, _ = _check(store, val, wl.F16, 8)
    assert counts_u32(out["counts"])[0, 0] == zeros.size
    _say("one-sweep non-finite")
    for bad in (np.nan, np.inf, -np.inf):
        x = np.linspace(-1, 1, 4 * 960, dtype=np.float32).reshape(1, 4, 960).copy()
        x[0, 2, 17] = bad
        for dtype in (wl.BF16, wl.F16):
            store, val = wl.store(x, dtype)
            out, ref = _check(store, val, dtype, 8)
            assert ref["status"] == oracle.ENONFINITE and counts_u32(out["counts"]).sum() == 0


def test_routing_and_errors():
    cfg = wl.scaled(wl.CONFIGS["c4_mamba2p8b"], D=256, L=2048)
    w = wl.make(cfg, with_z=False)
    xd = to_dev(w.dev["u"], cfg.dtype)
    for mode in (0, 2, 4):
        pol = corey.policy_default()
        pol.mode = mode
        one = corey.corey_entropy_hist_onesweep(xd, 256, policy=pol, table_ws=_ws())
        two = corey.corey_route_device(xd, 256, pol)
        torch.cuda.synchronize()
        assert torch.equal(one["chunks"], two["chunks"]) and torch.equal(one["counts"], two["counts"])
        assert torch.equal(one["H"], two["H"]) and torch.equal(one["r"], two["r"]) and torch.equal(one["range"], two["range"])
    with pytest.raises(corey.CoreyError) as e:
        corey.corey_entropy_hist_onesweep(xd.float(), 256, table_ws=_ws())
    assert e.value.code == 5                                        # fp32 storage: unsupported
    with pytest.raises(corey.CoreyError) as e:
        corey.corey_entropy_hist_onesweep(xd, 256, table_ws=torch.empty(1024, dtype=torch.uint8, device="cuda"))
    assert e.value.code == 7


@pytest.mark.parametrize("name", ["c1_mamba130m", "c2_mamba370m", "c3_mamba1p4b", "c4_mamba2p8b", "paper_w1_fp16"])
def test_full_size(name):
    cfg = dataclasses.replace(wl.CONFIGS[name], seqlens=None)
    _say(f"one-sweep full size {name}")
    w = wl.make(cfg, with_z=False)
    _check(w.dev["u"], w.val["u"], cfg.dtype, cfg.K)


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
@pytest.mark.parametrize("shape,W", [((1, 1, 1), 4), ((2, 3, 7), 2), ((2, 5, 37), 3), ((3, 4, 2049), 4), ((1, 2, 4104), 1),
                                     ((2, 6, 4096), 4), ((1, 40, 8192), 4), ((3, 300, 1000), 4)])
def test_table_filled_by_the_producer(dtype, shape, W):
    """causal_conv1d_silu_fwd with a pattern table: u, the carried state and the partial ranges are those of the plain
    launch bit for bit, and corey_entropy_hist_from_table gives the statistic of u that the oracle computes from u."""
    B, D, L = shape
    _say(f"producer table {shape} W{W} {dtype}")
    cfg = wl.Config(name="conv_t", B=B, D=D, N=16, L=L, dtype=dtype, K=64, chunks=(64,), seed=300 + W + L)
    c = wl.make_conv(cfg, W, with_state=(L % 2 == 1))
    xd, wd, bd = to_dev(c["dev"]["x"], dtype), to_dev(c["dev"]["weight"], wl.F32), to_dev(c["dev"]["bias"], wl.F32)
    sd = None if c["dev"].get("state_in") is None else to_dev(c["dev"]["state_in"], dtype)
    u0, so0, parts0 = corey.causal_conv1d_silu_fwd(xd, wd, bd, sd, want_state=True)
    u1, so1, parts1 = corey.causal_conv1d_silu_fwd(xd, wd, bd, sd, want_state=True, pattern_table=_ws())
    tdt = torch.bfloat16 if dtype == wl.BF16 else torch.float16
    pol = corey.policy_default()
    for K in (64, 1000, 64):                                     # the table serves any number of statistics
        out = corey.corey_entropy_hist_from_table(_ws(), tdt, L, K, policy=pol)
        two = corey.corey_route_device(u0, K, pol, range_parts=parts0)
        torch.cuda.synchronize()
        assert torch.equal(u0.view(torch.int16), u1.view(torch.int16)) and torch.equal(so0.view(torch.int16), so1.view(torch.int16))
        ref = oracle.entropy_hist(u0.float().cpu().numpy(), K)
        _compare(out, ref, K)
        assert torch.equal(out["chunks"], two["chunks"]) and torch.equal(out["counts"], two["counts"]) and torch.equal(out["H"], two["H"])
    # the partial ranges fold to the same range whichever launch wrote them
    e0 = corey.corey_entropy_hist(u0, 16, range_parts=parts0)
    e1 = corey.corey_entropy_hist(u0, 16, range_parts=parts1)
    torch.cuda.synchronize()
    assert torch.equal(e0["range"], e1["range"]) and torch.equal(e0["counts"], e1["counts"])


def test_producer_table_at_full_size():
    cfg = wl.CONFIGS["c4_mamba2p8b"]
    _say("producer table full size c4")
    c = wl.make_conv(cfg, 4)
    xd, wd, bd = to_dev(c["dev"]["x"], cfg.dtype), to_dev(c["dev"]["weight"], wl.F32), to_dev(c["dev"]["bias"], wl.F32)
    u, _, parts = corey.causal_conv1d_silu_fwd(xd, wd, bd, pattern_table=_ws())
    out = corey.corey_entropy_hist_from_table(_ws(), torch.bfloat16, cfg.L, cfg.K)
    torch.cuda.synchronize()
    ref = oracle.entropy_hist(u.float().cpu().numpy(), cfg.K)
    _compare(out, ref, cfg.K)
