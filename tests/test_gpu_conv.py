"""GPU parity: causal_conv1d_silu_fwd against the CPU oracle, and its fused range against the histogram's own sweep."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_10597_amd as corey
from gpu_util import counts_u32, to_dev
from paper_2604_10597_amd import workloads as wl

pytestmark = pytest.mark.gpu

SIG_BITS = {wl.F32: 24, wl.BF16: 8, wl.F16: 11}


def _say(msg):
    print(f"[case] {msg}", flush=True)


def _widen(t):
    return t.float().cpu().numpy()


def _tolerance(ref_u, val, W, dtype):
    """binary32 accumulation of W fused multiply-adds, a hardware exp2 and reciprocal (about 1 ulp each) and the
    gate's slope (< 1.1): 8 * 2^-24 of the magnitude of the accumulated terms; then one rounding to the storage
    type (half an ulp: 2^-p of the value, p its significand bits; fp16 subnormals: 2^-25 absolute)."""
    x, w, b = val["x"].astype(np.float64), np.abs(val["weight"].astype(np.float64)), np.abs(val["bias"].astype(np.float64))
    B, D, L = x.shape
    xp = np.concatenate([np.zeros((B, D, W - 1)) if val["state_in"] is None else np.abs(val["state_in"].astype(np.float64)),
                         np.abs(x)], axis=2)
    mag = np.broadcast_to(b[None, :, None], (B, D, L)).copy()
    for k in range(W):
        mag += w[None, :, k, None] * xp[:, :, k:k + L]
    tol = 8 * 2.0 ** -24 * mag + 2.0 ** -SIG_BITS[dtype] * np.abs(ref_u) * (1 + 1e-6)
    if dtype == wl.F16:
        tol += 2.0 ** -25
    return tol


def _run(cfg, W, with_state=False, want_state=True, bias=True):
    c = wl.make_conv(cfg, W, with_state=with_state)
    dev, val = c["dev"], c["val"]
    xd = to_dev(dev["x"], cfg.dtype)
    wd = torch.from_numpy(dev["weight"]).cuda()
    bd = torch.from_numpy(dev["bias"]).cuda() if bias else None
    sd = to_dev(dev["state_in"], cfg.dtype)
    u, so, parts = corey.causal_conv1d_silu_fwd(xd, wd, bd, sd, want_state=want_state)
    torch.cuda.synchronize()
    if not bias:
        val = dict(val, bias=np.zeros_like(val["bias"]))
    ref_u, ref_so = oracle.causal_conv1d_silu(val["x"], val["weight"], val["bias"], val["state_in"])
    got = _widen(u).astype(np.float64)
    err = np.abs(got - ref_u)
    tol = _tolerance(ref_u, val, W, cfg.dtype)
    bad = err > tol
    assert not bad.any(), f"{int(bad.sum())} of {bad.size} outside tolerance, worst {float((err / tol).max()):.2f}x"
    if want_state and W > 1:
        assert np.array_equal(_widen(so), ref_so)
    return u, parts, xd, wd, bd


def _parts_range(parts):
    """Reduce the partial ranges the producer left (host side, from their documented layout: lo_key, hi_key, saw_nan,
    pad as uint32; keys order floats as unsigned integers), and check that the partial histograms behind them are clear."""
    raw = parts.cpu().numpy().view(np.uint32)
    p = raw[:1024 * 4].reshape(-1, 4)                              # COREY_RANGE_PARTS records of 16 bytes ...
    assert raw.size == 1024 * 4 + 16 * 4096 and not raw[1024 * 4:].any()     # ... then the cleared partial histograms
    def unkey(k):
        k = np.uint32(k)
        bits = (k ^ np.uint32(0x80000000)) if (k & np.uint32(0x80000000)) else ~k
        return np.array([bits], dtype=np.uint32).view(np.float32)[0]
    return unkey(p[:, 0].min()), unkey(p[:, 1].max()), bool(p[:, 2].any())


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16, wl.F16])
@pytest.mark.parametrize("W", [1, 2, 3, 4])
@pytest.mark.parametrize("shape", [(1, 1, 1), (2, 3, 2), (1, 3, 7), (2, 5, 37), (3, 4, 2049), (1, 2, 4104), (2, 6, 4096)])
def test_parity_over_shapes_widths_and_types(dtype, W, shape):
    _say(f"conv {shape} W{W} {dtype}")
    B, D, L = shape
    cfg = wl.Config(name="conv_t", B=B, D=D, N=16, L=L, dtype=dtype, K=16, chunks=(64,), seed=100 + W + L)
    _run(cfg, W, with_state=(L % 2 == 1))


@pytest.mark.parametrize("name,D,L", [("c1_mamba130m", 96, 2048), ("c2_mamba370m", 64, 1000), ("c4_mamba2p8b", 300, 512)])
def test_fused_range_feeds_the_histogram(name, D, L):
    cfg = wl.scaled(wl.CONFIGS[name], D=D, L=L, seqlens=None)
    _say(f"conv+hist {cfg.name} B{cfg.B} D{cfg.D} L{cfg.L} {cfg.dtype}")
    u, parts, *_ = _run(cfg, 4, bias=(name != "c2_mamba370m"))
    uf = u.float()
    lo, hi, nan = _parts_range(parts)
    assert lo == uf.min().item() and hi == uf.max().item() and not nan
    plain = corey.corey_entropy_hist(u, cfg.K)
    fused = corey.corey_entropy_hist(u, cfg.K, range_parts=parts)
    torch.cuda.synchronize()
    assert np.array_equal(counts_u32(plain["counts"]), counts_u32(fused["counts"]))
    assert plain["H"].item() == fused["H"].item() and torch.equal(plain["range"], fused["range"])
    # and the statistic of that u is the oracle's
    ref = oracle.entropy_hist(uf.cpu().numpy(), cfg.K)
    assert np.array_equal(counts_u32(fused["counts"]), ref["counts"])
    routed = corey.corey_route_device(u, cfg.K, range_parts=parts)
    plain_routed = corey.corey_route_device(u, cfg.K)
    torch.cuda.synchronize()
    assert torch.equal(routed["chunks"], plain_routed["chunks"]) and routed["H"].item() == plain["H"].item()


def test_unaligned_views_and_nan_inputs():
    _say("conv unaligned / NaN")
    cfg = wl.Config(name="conv_u", B=2, D=3, N=16, L=1029, dtype=wl.BF16, K=16, chunks=(64,), seed=5)
    c = wl.make_conv(cfg, 4)
    base = torch.zeros(cfg.B * cfg.D * cfg.L + 1, dtype=torch.bfloat16, device="cuda")
    xd = base[1:].view(cfg.B, cfg.D, cfg.L)                     # 2 bytes off a 16-byte boundary
    xd.copy_(to_dev(c["dev"]["x"], cfg.dtype))
    wd, bd = torch.from_numpy(c["dev"]["weight"]).cuda(), torch.from_numpy(c["dev"]["bias"]).cuda()
    u, _, parts = corey.causal_conv1d_silu_fwd(xd, wd, bd)
    u2, _, _ = corey.causal_conv1d_silu_fwd(to_dev(c["dev"]["x"], cfg.dtype), wd, bd)
    torch.cuda.synchronize()
    assert torch.equal(u.view(torch.int16), u2.view(torch.int16))
    fused = corey.corey_entropy_hist(u, 16, range_parts=parts)
    plain = corey.corey_entropy_hist(u, 16)
    assert torch.equal(fused["counts"], plain["counts"])

    x = torch.randn(1, 2, 300, device="cuda")
    x[0, 1, 100] = float("nan")
    w = torch.full((2, 4), 0.5, device="cuda")
    u, _, parts = corey.causal_conv1d_silu_fwd(x, w)
    torch.cuda.synchronize()
    assert torch.isnan(u[0, 1, 100:104]).all() and not torch.isnan(u[0, 0]).any() and not torch.isnan(u[0, 1, 104:]).any()
    lo, hi, nan = _parts_range(parts)
    finite = u[~torch.isnan(u)]
    assert nan and lo == finite.min().item() and hi == finite.max().item()
    fused = corey.corey_entropy_hist(u, 16, range_parts=parts)
    plain = corey.corey_entropy_hist(u, 16)
    torch.cuda.synchronize()
    assert torch.equal(fused["counts"], plain["counts"])
    assert torch.equal(fused["H"].isnan(), plain["H"].isnan())


@pytest.mark.parametrize("name,D,L,stride,block", [("c1_mamba130m", 96, 2048, 8, 512), ("c4_mamba2p8b", 300, 512, 8, 1),
                                                    ("c2_mamba370m", 64, 1000, 3, 64), ("paper_w1_fp16", 40, 4096, 8, 512),
                                                    ("c0_tiny_f32", 33, 1001, 5, 24), ("c1_mamba130m", 7, 333, 4, 40)])
def test_fused_range_with_the_sampled_count(name, D, L, stride, block):
    """Range from the producer (all values), counts over every stride-th block: the oracle's range_all reading."""
    cfg = wl.scaled(wl.CONFIGS[name], D=D, L=L, seqlens=None)
    _say(f"conv + sampled hist {cfg.name} D{D} L{L} stride {stride} block {block}")
    u, parts, *_ = _run(cfg, 4)
    uf = u.float()
    got = corey.corey_entropy_hist(u, cfg.K, stride=stride, block=block, range_parts=parts)
    routed = corey.corey_route_device(u, cfg.K, stride=stride, block=block, range_parts=parts)
    torch.cuda.synchronize()
    ref = oracle.entropy_hist(uf.cpu().numpy(), cfg.K, stride=stride, block=block, range_all=True)
    assert np.array_equal(counts_u32(got["counts"]), ref["counts"]) and np.array_equal(counts_u32(routed["counts"]), ref["counts"])
    assert got["H"].item() == pytest.approx(ref["H"][0], rel=1e-12) and got["r"].item() == pytest.approx(ref["r"][0], rel=1e-12)
    assert got["range"].cpu().reshape(-1).tolist() == [uf.min().item(), uf.max().item()]
    st, c_ref, margin = oracle.select_chunk(float(ref["r"][0]), cfg.L, oracle.policy())
    if margin > 1e-9:
        assert routed["chunks"].item() == c_ref
    # the sampled statistic on its own range is a different (narrower-binned) histogram of the same values
    plain = oracle.entropy_hist(uf.cpu().numpy(), cfg.K, stride=stride, block=block)
    assert plain["counts"].sum() == ref["counts"].sum()


def test_given_range_is_rejected_for_per_sequence_statistics():
    x = torch.randn(2, 4, 64, device="cuda")
    w = torch.ones(4, 2, device="cuda")
    u, _, parts = corey.causal_conv1d_silu_fwd(x, w)
    with pytest.raises(corey.CoreyError):
        corey.corey_entropy_hist(u, 16, seqlens=torch.tensor([64, 10], dtype=torch.int32, device="cuda"), range_parts=parts)
    with pytest.raises(corey.CoreyError):
        corey.causal_conv1d_silu_fwd(x, torch.ones(4, 5, device="cuda"))


@pytest.mark.parametrize("name", ["c2_mamba370m", "c4_mamba2p8b", "paper_w1_fp16"])
def test_full_size_sampled_channels_and_whole_range(name):
    """The benchmark's launch configuration at full size: the oracle recomputes sampled channels, the fused range is
    checked against a plain reduction of the stored output, and the histogram it feeds against the oracle's."""
    cfg = wl.scaled(wl.CONFIGS[name], seqlens=None) if wl.CONFIGS[name].seqlens else wl.CONFIGS[name]
    _say(f"conv full size {name} B{cfg.B} D{cfg.D} L{cfg.L} {cfg.dtype}")
    c = wl.make_conv(cfg, 4, with_state=True)
    dev, val = c["dev"], c["val"]
    xd = to_dev(dev["x"], cfg.dtype)
    wd, bd = torch.from_numpy(dev["weight"]).cuda(), torch.from_numpy(dev["bias"]).cuda()
    sd = to_dev(dev["state_in"], cfg.dtype)
    u, so, parts = corey.causal_conv1d_silu_fwd(xd, wd, bd, sd, want_state=True)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 1, cfg.D // 2, cfg.D - 1], np.random.default_rng(5).integers(0, cfg.D, 12)]))
    sub = {"x": val["x"][:, rows, :], "weight": val["weight"][rows], "bias": val["bias"][rows], "state_in": val["state_in"][:, rows, :]}
    ref_u, ref_so = oracle.causal_conv1d_silu(sub["x"], sub["weight"], sub["bias"], sub["state_in"])
    got = _widen(u[:, torch.from_numpy(rows).cuda(), :]).astype(np.float64)
    err, tol = np.abs(got - ref_u), _tolerance(ref_u, sub, 4, cfg.dtype)
    assert not (err > tol).any(), f"worst {float((err / tol).max()):.2f}x the tolerance"
    assert np.array_equal(_widen(so)[:, rows, :], ref_so)
    uf = u.float()
    lo, hi, nan = _parts_range(parts)
    assert lo == uf.min().item() and hi == uf.max().item() and not nan
    fused = corey.corey_entropy_hist(u, cfg.K, range_parts=parts)
    torch.cuda.synchronize()
    ref = oracle.entropy_hist(uf.cpu().numpy(), cfg.K)
    assert np.array_equal(counts_u32(fused["counts"]), ref["counts"])
    assert fused["H"].item() == pytest.approx(ref["H"][0], rel=1e-12)


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32])
def test_generation_steps_continue_the_prompt_bit_for_bit(dtype):
    """A prompt through the vector path, then single steps from the carried state (the one-lane-per-row path): the same
    bits as one call over the whole sequence, and the same carried state."""
    P, T = 4096, 5
    cfg = wl.Config(name="conv_gen", B=2, D=70, N=16, L=P + T, dtype=dtype, K=16, chunks=(64,), seed=21)
    _say(f"conv prompt {P} + {T} steps {dtype}")
    c = wl.make_conv(cfg, 4)
    xd = to_dev(c["dev"]["x"], cfg.dtype)
    wd, bd = torch.from_numpy(c["dev"]["weight"]).cuda(), torch.from_numpy(c["dev"]["bias"]).cuda()
    whole, s_whole, _ = corey.causal_conv1d_silu_fwd(xd, wd, bd, want_state=True)
    u0, state, _ = corey.causal_conv1d_silu_fwd(xd[:, :, :P].contiguous(), wd, bd, want_state=True)
    outs = [u0]
    for t in range(P, P + T):
        ut, state, parts = corey.causal_conv1d_silu_fwd(xd[:, :, t:t + 1].contiguous(), wd, bd, state_in=state, want_state=True)
        outs.append(ut)
        lo, hi, nan = _parts_range(parts)
        assert lo == ut.float().min().item() and hi == ut.float().max().item() and not nan
    torch.cuda.synchronize()
    view = torch.int16 if dtype == wl.BF16 else torch.int32
    assert torch.equal(torch.cat(outs, dim=2).view(view), whole.view(view))
    assert torch.equal(state.view(view), s_whole.view(view))


def test_more_than_two_to_the_31_elements():
    """x and u of 2.2e9 elements each: 64-bit indexing in the producer and in the count sweep that takes its range.
    Inputs drawn on the GPU (seeded); the oracle recomputes three channels."""
    B, D, L, W, K = 1, 2100, (1 << 20) + 8, 4, 256
    _say(f"conv on {B * D * L} elements")
    g = torch.Generator(device="cuda").manual_seed(78)
    x = torch.empty((B, D, L), dtype=torch.bfloat16, device="cuda")
    for d0 in range(0, D, 300):
        x[:, d0:d0 + 300] = torch.randn(B, min(300, D - d0), L, generator=g, device="cuda").to(torch.bfloat16)
    wt = torch.rand(D, W, generator=g, device="cuda") - 0.5
    bs = torch.rand(D, generator=g, device="cuda") - 0.5
    st_in = torch.randn(B, D, W - 1, generator=g, device="cuda").to(torch.bfloat16)
    u, st_out, parts = corey.causal_conv1d_silu_fwd(x, wt, bs, st_in, want_state=True)
    torch.cuda.synchronize()
    rows = [0, D // 2 + 1, D - 1]
    val = {"x": _widen(x[:, rows]), "weight": _widen(wt[rows]), "bias": _widen(bs[rows]), "state_in": _widen(st_in[:, rows])}
    ref_u, ref_so = oracle.causal_conv1d_silu(val["x"], val["weight"], val["bias"], val["state_in"])
    err = np.abs(_widen(u[:, rows]).astype(np.float64) - ref_u)
    assert not (err > _tolerance(ref_u, val, W, wl.BF16)).any()
    assert np.array_equal(_widen(st_out[:, rows]), ref_so)
    lo, hi, nan = _parts_range(parts)
    assert not nan and lo == min(u[:, d0:d0 + 300].min().item() for d0 in range(0, D, 300))
    assert hi == max(u[:, d0:d0 + 300].max().item() for d0 in range(0, D, 300))
    fused = corey.corey_entropy_hist(u, K, range_parts=parts)
    plain = corey.corey_entropy_hist(u, K)
    sampled = corey.corey_entropy_hist(u, K, range_parts=parts, stride=8, block=512)
    torch.cuda.synchronize()
    assert torch.equal(fused["counts"], plain["counts"]) and int(counts_u32(fused["counts"]).astype(np.int64).sum()) == B * D * L
    nblocks = -(-B * D * L // 512)
    assert int(counts_u32(sampled["counts"]).astype(np.int64).sum()) == sum(min(512, B * D * L - i * 512) for i in range(0, nblocks, 8))
