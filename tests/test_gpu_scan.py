"""GPU parity: selective_scan_fwd against the CPU oracle, element by element, plus the invariants of the method.

Tolerance (written out in gpu_util.assert_close): |got - ref| <= rtol * (|ref| + rms(ref row)), with rtol = 1e-5 for
fp32 storage at the stated configuration (growing with sqrt(L/256) for longer sequences, see gpu_util.fp32_rtol)
and 3e-3 for bf16 storage with fp32 state, plus the bf16 store's own half ulp; the fp32 state is held to the fp32
bound for both storage types.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
import paper_2604_10597_amd as corey
from gpu_util import assert_close, chain_rtol, check_y, fp32_rtol, oracle_scan, store_bits, upload, y_rtol, y_to_f64
from paper_2604_10597_amd import workloads as wl

pytestmark = pytest.mark.gpu
ALL_CHUNKS = (16, 32, 64, 128, 256, 512, 1024, 2048)


def _say(msg):
    print(f"[case] {msg}", flush=True)


def _run(d, chunk, use_z=True, use_h0=True, chunks_dev=None, softplus=True, general_a=False, whole_rows=False):
    y, last = corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"] if use_z else None,
                                       delta_bias=d["delta_bias"], delta_softplus=softplus,
                                       h0=d.get("h0") if use_h0 else None, seqlens=d["seqlens"], chunk=chunk,
                                       chunks_dev=chunks_dev, general_a=general_a, whole_rows=whole_rows)
    torch.cuda.synchronize()
    return y_to_f64(y), last.cpu().numpy().astype(np.float64)


def _parity(cfg, chunks, a_kind="mamba", with_h0=False, use_z=True):
    w = wl.make(cfg, a_kind=a_kind, with_h0=with_h0)
    d = upload(w)
    y_ref, s_ref = oracle_scan(w, use_z=use_z)
    worst = 0.0
    # a structured A takes the power-chain path by default: run the general path on it as well (the benchmark's figures
    # are measured on the general path)
    for general_a in ((False, True) if a_kind == "mamba" and cfg.dtype != wl.F32 else (False,)):
        for chunk in chunks:
            # a launch this small gives every channel two rows of lanes with half of the states each: the launch shape of
            # large layers (one row per channel) is run on it as well
            split = corey.selective_scan_fwd_plan_split(cfg.B, cfg.D, cfg.N, chunk) == 1
            for whole_rows in ((False, True) if split else (False,)):
                what = f"chunk {chunk} general_a={general_a} whole_rows={whole_rows}"
                _say(f"scan {cfg.name} B{cfg.B} D{cfg.D} N{cfg.N} L{cfg.L} {cfg.dtype} A={a_kind} z={use_z} h0={with_h0} {what}")
                y, s = _run(d, chunk, use_z=use_z, general_a=general_a, whole_rows=whole_rows)
                worst = max(worst, check_y(y, y_ref, cfg, f"y {what}")[0])
                assert_close(s, s_ref, fp32_rtol(cfg.L), f"last_state {what}")
    return worst


def test_config0_fp32_every_chunk():
    _parity(wl.CONFIGS["c0_tiny_f32"], ALL_CHUNKS)
    _parity(wl.CONFIGS["c0_tiny_f32"], (64, 128, 256), a_kind="random", with_h0=True)


@pytest.mark.parametrize("name,D,L,seqlens", [
    ("c1_mamba130m", 40, 2048, None),
    ("c2_mamba370m", 24, 1280, None),
    ("c3_mamba1p4b", 20, 2304, (2304, 700)),
    ("c4_mamba2p8b", 200, 1100, None),
])
def test_configs_at_oracle_size_every_chunk(name, D, L, seqlens):
    cfg = wl.scaled(wl.CONFIGS[name], D=D, L=L, seqlens=seqlens)
    _parity(cfg, ALL_CHUNKS)


@pytest.mark.parametrize("name,D,L", [("paper_w1_fp16", 48, 2048), ("c2_mamba370m", 24, 1100)])
def test_fp16_storage(name, D, L):
    """IEEE binary16 storage (the paper's kernel-level precision): fp32 computation bound plus the fp16 store."""
    cfg = wl.scaled(wl.CONFIGS[name], D=D, L=L, dtype=wl.F16)
    _parity(cfg, (64, 256, 512, 2048))
    _parity(wl.scaled(cfg, L=333), (64, 512), a_kind="random", with_h0=True)


def test_unstructured_A_initial_state_and_no_gate():
    cfg = wl.scaled(wl.CONFIGS["c2_mamba370m"], D=36, L=777)
    _parity(cfg, (64, 512, 2048), a_kind="random", with_h0=True)
    _parity(cfg, (128, 1024), a_kind="random", use_z=False)
    cfg32 = wl.scaled(wl.CONFIGS["c2_mamba370m"], D=20, L=1500, dtype=wl.F32)
    _parity(cfg32, (64, 256, 2048), a_kind="random", with_h0=True)


@pytest.mark.parametrize("N", [1, 3, 16, 40, 64, 256])
def test_state_sizes(N):
    cfg = wl.scaled(wl.CONFIGS["c1_mamba130m"], D=12, L=300, N=N, B=2)
    _parity(cfg, (64, 2048), a_kind="random", with_h0=True)


@pytest.mark.parametrize("L", [1, 15, 16, 17, 63, 65, 1023, 2049])
def test_ragged_lengths(L):
    for dtype in (wl.F32, wl.BF16, wl.F16):
        cfg = wl.scaled(wl.CONFIGS["c0_tiny_f32"], D=7, L=L, B=2, dtype=dtype)
        _parity(cfg, (16, 64, 2048), a_kind="random")


def test_padded_batches_and_empty_sequence():
    for lens in ((512, 2048), (2048, 512), (1, 2048), (0, 100), (2048, 2048)):
        cfg = wl.scaled(wl.CONFIGS["c3_mamba1p4b"], D=16, L=2048, seqlens=lens)
        w = wl.make(cfg, with_h0=True)
        d = upload(w)
        y_ref, s_ref = oracle_scan(w)
        for chunk, whole_rows in ((64, False), (64, True), (256, False), (256, True), (2048, False)):
            _say(f"scan padded lens={lens} chunk={chunk} whole_rows={whole_rows}")
            y, s = _run(d, chunk, whole_rows=whole_rows)
            assert_close(y, y_ref, y_rtol(cfg), f"y lens {lens}", True)
            assert_close(s, s_ref, fp32_rtol(cfg.L), f"state lens {lens}")
            for b, n in enumerate(lens):
                assert not y[b, :, n:].any()                 # padded positions are exactly zero
        if lens[0] == 0:
            assert np.array_equal(s[0], w.val["h0"][0].astype(np.float64))


def test_per_sequence_device_chunks():
    cfg = wl.scaled(wl.CONFIGS["c3_mamba1p4b"], D=24, L=1536, B=4, seqlens=(1536, 40, 900, 1536))
    w = wl.make(cfg)
    d = upload(w)
    y_ref, s_ref = oracle_scan(w)
    chunks = torch.tensor([2048, 64, 512, 100], dtype=torch.int32, device="cuda")   # 100 is invalid -> host value
    _say("scan per-sequence device chunks")
    y, s = _run(d, 256, chunks_dev=chunks)
    assert_close(y, y_ref, y_rtol(cfg), "y device chunks", True)
    # each sequence must equal a uniform launch with its own chunk, bit for bit
    for b, c in enumerate((2048, 64, 512, 256)):
        yb, sb = _run(d, c)
        assert np.array_equal(yb[b], y[b]) and np.array_equal(sb[b], s[b])
    # one routed chunk for the whole batch (COREY_SCAN_ONE_CHUNK): equal to a uniform launch with that chunk
    y1, s1 = _run(d, 2048, chunks_dev=torch.tensor([128], dtype=torch.int32, device="cuda"))
    yu, su = _run(d, 128)
    assert np.array_equal(y1, yu) and np.array_equal(s1, su)
    with pytest.raises(TypeError):
        _run(d, 256, chunks_dev=torch.tensor([128, 128], dtype=torch.int32, device="cuda"))     # neither one entry nor B
    with pytest.raises(TypeError):
        _run(d, 256, chunks_dev=torch.tensor([128, 128, 128, 128], device="cuda"))              # int64


def test_device_side_routing_matches_the_oracle_rule():
    import math
    import oracle
    _say("device chunk rule")
    rs = np.concatenate([np.linspace(0.0, 1.0, 801), [float("nan"), -0.5, 1.5]])
    r_dev = torch.from_numpy(rs).cuda()
    for mode in (0, 1, 2, 3, 4):
        for cmin, cmax in ((64, 2048), (32, 512)):
            for scale in (1.0, math.log(256) / 8.0):
                for L in (25, 50, 51, 300, 16384):
                    pol, opol = corey.policy_default(), oracle.policy(mode=mode, c_min=cmin, c_max=cmax, h_ref_scale=scale)
                    pol.mode, pol.c_min, pol.c_max, pol.h_ref_scale = mode, cmin, cmax, scale
                    got = corey.corey_select_chunk_device(r_dev, L, pol).cpu().numpy()
                    for r, g in zip(rs, got):
                        st, c, margin = oracle.select_chunk(float(r), L, opol)
                        if st == oracle.ENONFINITE:
                            assert g == 0
                        elif margin < 0 or margin > 1e-12:          # away from a rounding tie of Eq. 2
                            assert g == c, (mode, cmin, cmax, scale, L, r, g, c)
    # per-sequence lengths
    lens = torch.tensor([25, 50, 51, 4096], dtype=torch.int32, device="cuda")
    pol = corey.policy_default()
    pol.mode = 2
    got = corey.corey_select_chunk_device(torch.zeros(4, dtype=torch.float64, device="cuda"), 1, pol, seqlens=lens)
    assert got.cpu().tolist() == [128, 128, 512, 512]


def test_routed_scan_without_host_round_trip():
    cfg = wl.scaled(wl.CONFIGS["c3_mamba1p4b"], D=32, L=2048, B=3, seqlens=(2048, 40, 700))
    w = wl.make(cfg)
    d = upload(w)
    _say("scan routed on device")
    ent = corey.corey_entropy_hist(d["u"], cfg.K, seqlens=d["seqlens"])
    pol = corey.policy_default()
    pol.mode = 1                                              # sequence-length gate, then the entropy rule
    chunks = corey.corey_select_chunk_device(ent["r"], cfg.L, pol, seqlens=d["seqlens"])
    y, s = _run(d, 512, chunks_dev=chunks)                    # no synchronisation between the three calls
    import oracle
    ref = oracle.entropy_hist(w.val["u"], cfg.K, seqlens=w.seqlens)
    expect = [oracle.select_chunk(float(ref["r"][b]), int(w.seqlens[b]), oracle.policy(mode=1))[1] for b in range(3)]
    assert chunks.cpu().tolist() == expect and expect[1] == 128
    y_ref, s_ref = oracle_scan(w)
    assert_close(y, y_ref, y_rtol(cfg), "routed y", True)
    assert_close(s, s_ref, fp32_rtol(cfg.L), "routed state")
    for b, c in enumerate(expect):                            # each sequence ran with its own chunk
        yb, _ = _run(d, c)
        assert np.array_equal(yb[b], y[b])


def test_route_device_equals_the_two_calls():
    """corey_route_device = corey_entropy_hist then corey_select_chunk_device, bit for bit, for every mode."""
    cfg = wl.scaled(wl.CONFIGS["c3_mamba1p4b"], D=32, L=2048, B=3, seqlens=(2048, 40, 700))
    w = wl.make(cfg)
    d = upload(w)
    _say("route_device")
    for seqlens in (d["seqlens"], None):
        for mode in (0, 1, 2, 3, 4):
            for stride, block in ((1, 1), (8, 512)):
                pol = corey.policy_default()
                pol.mode = mode
                ent = corey.corey_entropy_hist(d["u"], cfg.K, seqlens=seqlens, stride=stride, block=block)
                two = corey.corey_select_chunk_device(ent["r"], cfg.L, pol, seqlens=seqlens)
                one = corey.corey_route_device(d["u"], cfg.K, pol, seqlens=seqlens, stride=stride, block=block)
                torch.cuda.synchronize()
                assert torch.equal(one["chunks"], two) and torch.equal(one["counts"], ent["counts"])
                assert torch.equal(one["r"], ent["r"]) and torch.equal(one["H"], ent["H"])
    bad = corey.policy_default()
    bad.c_min = 48
    with pytest.raises(corey.CoreyError):
        corey.corey_route_device(d["u"], cfg.K, bad)


def test_route_device_with_ema_and_chunk_counters():
    """The smoothed entropy across calls and the chunk-distribution counters, against the oracle's EMA and rule."""
    import math
    import oracle
    K = 256
    rng = np.random.default_rng(11)
    pol, opol = corey.policy_default(), oracle.policy()
    ema = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda")
    calls = torch.zeros(12, dtype=torch.int32, device="cuda")
    s_ref = float("nan")
    expect_calls = np.zeros(12, dtype=np.int64)
    _say("route_device EMA")
    for it, scale in enumerate((1.0, 1.0, 30.0, 1.0, 0.2, 1.0, 8.0, 1.0)):
        x = rng.standard_normal((1, 8, 2048)).astype(np.float32)
        x[0, 0, :16] *= scale                                  # a few outliers stretch the range: entropy moves call to call
        store, val = wl.store(x, wl.BF16)
        out = corey.corey_route_device(upload_one(store), K, pol, ema_lambda=0.85, ema_state=ema, chunk_calls=calls)
        torch.cuda.synchronize()
        ref = oracle.entropy_hist(val, K)
        s_ref = oracle.ema_update(0.85, s_ref, float(ref["H"][0]))
        assert out["H"].item() == pytest.approx(ref["H"][0], rel=1e-12)          # raw value of this call
        assert ema.item() == pytest.approx(s_ref, rel=1e-12)
        r_s = min(max(s_ref / math.log(K), 0.0), 1.0)
        st, c, margin = oracle.select_chunk(r_s, 2048, opol)
        assert margin > 1e-9 and out["chunks"].item() == c
        expect_calls[int(math.log2(c))] += 1
    assert np.array_equal(calls.cpu().numpy(), expect_calls) and expect_calls.sum() == 8
    with pytest.raises(corey.CoreyError):
        corey.corey_route_device(upload_one(store), K, pol, ema_lambda=1.0, ema_state=ema)


def upload_one(store):
    from gpu_util import to_dev
    return to_dev(store, wl.BF16)


def test_structured_A_fast_path():
    """A[d, n] = (n + 1) A[d, 0] with 16-bit storage takes the power-chain path unless COREY_SCAN_GENERAL_A is given: it
    must meet the same bounds as the general path, differ from it only by the chain's roundings (gpu_util.chain_rtol),
    and leave every other A untouched."""
    for name, dtype in (("c2_mamba370m", wl.BF16), ("paper_w1_fp16", wl.F16)):
        cfg = wl.scaled(wl.CONFIGS[name], D=40, L=1300, dtype=dtype)
        w = wl.make(cfg, a_kind="mamba", with_h0=True)
        d = upload(w)
        y_ref, s_ref = oracle_scan(w)
        for chunk in (64, 512, 1024, 2048):
            _say(f"scan structured A {name} {dtype} chunk={chunk}")
            y1, s1 = _run(d, chunk)
            y0, s0 = _run(d, chunk, general_a=True)
            for y, s in ((y1, s1), (y0, s0)):
                check_y(y, y_ref, cfg, f"y chunk {chunk}")
                assert_close(s, s_ref, fp32_rtol(cfg.L), f"state chunk {chunk}")
            assert not np.array_equal(s1, s0)             # the two paths really are different code
            assert_close(s1, s0, chain_rtol(cfg.N), "structured against general state")
        # an unstructured A takes the general path whatever the flag
        wr = wl.make(cfg, a_kind="random")
        dr = upload(wr)
        ya, sa = _run(dr, 512)
        yb, sb = _run(dr, 512, general_a=True)
        assert np.array_equal(ya, yb) and np.array_equal(sa, sb)
    # fp32 storage never takes it
    cfg = wl.scaled(wl.CONFIGS["c0_tiny_f32"], D=16, L=512)
    w = wl.make(cfg)
    d = upload(w)
    ya, sa = _run(d, 256)
    yb, sb = _run(d, 256, general_a=True)
    assert np.array_equal(ya, yb) and np.array_equal(sa, sb)
    # an unknown flag bit is an error, found before any launch
    lib, ptr = corey.binding.lib(), corey.binding._ptr
    ws = torch.empty(corey.selective_scan_fwd_workspace(cfg.B, cfg.N, cfg.L), dtype=torch.uint8, device="cuda")
    y, last = torch.empty_like(d["u"]), torch.empty((cfg.B, cfg.D, cfg.N), dtype=torch.float32, device="cuda")
    st = lib.selective_scan_fwd(ptr(d["u"]), ptr(d["delta"]), ptr(d["A"]), ptr(d["B"]), ptr(d["C"]), None, None, None, 1, None, None, 256,
                                None, ptr(y), ptr(last), 0, cfg.B, cfg.D, cfg.N, cfg.L, 8, ptr(ws), ws.numel(), None)
    assert st == 1


def test_invariants_on_the_gpu_path():
    cfg = wl.scaled(wl.CONFIGS["c2_mamba370m"], D=32, L=1024)
    w = wl.make(cfg, a_kind="random")
    d = upload(w)
    _say("scan invariants")
    y1, s1 = _run(d, 256)
    # linearity in u: scaling by a power of two scales y and the state exactly
    d2 = dict(d)
    d2["u"] = (d["u"].to(torch.float32) * 4).to(d["u"].dtype)
    y4, s4 = _run(d2, 256)
    assert np.array_equal(y4, 4 * y1) and np.array_equal(s4, 4 * s1)
    # continuation: scanning the tail from the returned state reproduces the full scan
    cut = 384
    head = {k: (v[..., :cut].contiguous() if k in ("u", "delta", "z", "B", "C") else v) for k, v in d.items()}
    tail = {k: (v[..., cut:].contiguous() if k in ("u", "delta", "z", "B", "C") else v) for k, v in d.items()}
    yh, sh = _run(head, 128)
    tail["h0"] = torch.from_numpy(sh.astype(np.float32)).cuda()
    yt, st = _run(tail, 128)
    assert_close(np.concatenate([yh, yt], axis=-1), y1, y_rtol(cfg), "split scan", True)
    assert_close(st, s1, fp32_rtol(cfg.L), "split scan state")
    # gate: z = 0 gives y = 0; no gate equals gated / silu
    d0 = dict(d)
    d0["z"] = torch.zeros_like(d["z"])
    y0, _ = _run(d0, 256)
    assert not y0.any()
    # repeat runs are bit-identical
    y1b, s1b = _run(d, 256)
    assert np.array_equal(y1, y1b) and np.array_equal(s1, s1b)


def test_closed_form_on_gpu_without_softplus():
    # constant inputs: geometric series (decay strong enough that binary32 rounding of exp() stays below tolerance)
    B, D, N, L = 1, 8, 16, 600
    dl, uu, bb, cc = 0.25, 1.5, -0.75, 2.0
    A = -np.broadcast_to(np.arange(1, N + 1, dtype=np.float32), (D, N)).copy()
    full = lambda v, shape: torch.full(shape, v, dtype=torch.float32, device="cuda")
    y, last = corey.selective_scan_fwd(full(uu, (B, D, L)), full(dl, (B, D, L)), torch.from_numpy(A).cuda(),
                                       full(bb, (B, N, L)), full(cc, (B, N, L)), delta_softplus=False, chunk=128)
    abar = np.exp(dl * A[0].astype(np.float64))
    t = np.arange(1, L + 1)[:, None]
    h = dl * bb * uu * (1 - abar ** t) / (1 - abar)
    assert_close(y.cpu().numpy()[0, 0], cc * h.sum(1), fp32_rtol(L), "geometric series y")
    assert_close(last.cpu().numpy()[0, 0], h[-1], fp32_rtol(L), "geometric series state")


@pytest.mark.parametrize("B,D,chunk,N", [(1, 4160, 512, 16), (1, 6200, 512, 16), (2, 2100, 512, 16), (1, 8300, 256, 16),
                                          (3, 1500, 512, 16), (1, 4200, 512, 128), (3, 3000, 256, 200)])
def test_launches_that_mix_both_lane_geometries(B, D, chunk, N):
    """Channel counts beyond one resident wave per row: most channels run with 16 steps per lane, the remainder with 8, in
    one launch (host chunk and device chunk).  Sampled channels from both parts and around the split against the oracle."""
    cfg = wl.scaled(wl.CONFIGS["c2_mamba370m"], B=B, D=D, L=1536 if N == 16 else 600, seqlens=None, N=N)
    _say(f"mixed geometries B{B} D{D} N{N} chunk {chunk}")
    w = wl.make(cfg, a_kind="random")
    d = upload(w)
    split = corey.selective_scan_fwd_plan(B, D, N, chunk)
    if N == 16:
        layer = 256 * (4096 // chunk) // B // 32 * 32
        assert split == D // layer * layer
    assert 0 < split < D
    rows = np.unique(np.clip(np.concatenate([[0, 1, split - 2, split - 1, split, split + 1, D - 1],
                                             np.random.default_rng(D).integers(0, D, 10)]), 0, D - 1))
    y_ref, s_ref = oracle_scan(w, rows=rows)
    chunks_dev = torch.full((B,), chunk, dtype=torch.int32, device="cuda")
    for routed in (False, True):
        y, last = corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"],
                                           delta_bias=d["delta_bias"], chunk=chunk if not routed else 64,
                                           chunks_dev=chunks_dev if routed else None)
        torch.cuda.synchronize()
        ys = y[:, torch.from_numpy(rows).cuda(), :]
        assert_close(y_to_f64(ys), y_ref, y_rtol(cfg), f"y routed={routed}", store_bits(cfg))
        assert_close(last.cpu().numpy()[:, rows, :], s_ref, fp32_rtol(cfg.L), f"state routed={routed}")
        assert torch.isfinite(y.float()).all()


@pytest.mark.parametrize("D,chunk,L", [(13000, 64, 600), (26000, 32, 200), (50000, 16, 100), (1536, 256, 1100), (640, 64, 1100)])
def test_short_tiles_and_few_channels(D, chunk, L):
    """Launches short of waves take 4 time steps per lane, the same chunks with many channels 8: both against the oracle
    on sampled channels, host chunk and device chunk, bit for bit the same."""
    cfg = wl.scaled(wl.CONFIGS["c2_mamba370m"], B=1, D=D, L=L, seqlens=None)
    steps = corey.selective_scan_fwd_plan_steps(1, D, cfg.N, chunk)
    assert steps == (8 if D >= 13000 else 4) and corey.selective_scan_fwd_plan(1, D, cfg.N, chunk) == 0
    _say(f"short tiles D{D} chunk {chunk}: {steps} steps per lane")
    w = wl.make(cfg, a_kind="random")
    d = upload(w)
    rows = np.unique(np.concatenate([[0, 1, D // 2, D - 2, D - 1], np.random.default_rng(D).integers(0, D, 8)]))
    y_ref, s_ref = oracle_scan(w, rows=rows)
    outs = []
    for chunks_dev in (None, torch.full((1,), chunk, dtype=torch.int32, device="cuda")):
        y, last = corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"], delta_bias=d["delta_bias"],
                                           chunk=chunk if chunks_dev is None else 512, chunks_dev=chunks_dev)
        torch.cuda.synchronize()
        ys = y[:, torch.from_numpy(rows).cuda(), :]
        assert_close(y_to_f64(ys), y_ref, y_rtol(cfg), "y", store_bits(cfg))
        assert_close(last.cpu().numpy()[:, rows, :], s_ref, fp32_rtol(cfg.L), "state")
        assert torch.isfinite(y.float()).all()
        outs.append((y, last))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


@pytest.mark.parametrize("B,D,N,L,chunk,steps", [(1, 1024, 16, 4096, 1024, 16), (1, 1536, 16, 2048, 512, 8), (2, 300, 64, 1500, 256, 4),
                                                  (1, 5120, 16, 700, 64, 4), (3, 257, 24, 333, 16, 4), (1, 1537, 16, 2048, 1024, 16)])
def test_two_rows_per_channel_against_whole_rows(B, D, N, L, chunk, steps):
    """Launches short of waves give a channel two rows of lanes with half of the states each.  Per (channel, state) both
    launch shapes do the same arithmetic in the same order, so on the general path the final state is the same bit for bit;
    y adds the two halves' sums in another order and is held to the oracle (sampled channels) and to the other shape."""
    expect = 0 if D == 1537 else 1                        # 1537 channels of 64 lanes: one wave more than the rule's 1536
    assert corey.selective_scan_fwd_plan_split(B, D, N, chunk) == expect
    d16 = corey.selective_scan_fwd_plan(B, D, N, chunk)
    assert (16 if d16 == D else corey.selective_scan_fwd_plan_steps(B, D, N, chunk)) == steps and d16 in (0, D)
    lens = None if B == 1 else tuple(L - 37 * b for b in range(B))
    cfg = dataclasses.replace(wl.scaled(wl.CONFIGS["c2_mamba370m"], B=B, D=D, N=N, L=L), seqlens=lens)
    _say(f"two rows per channel B{B} D{D} N{N} L{L} chunk {chunk} ({steps} steps per lane) split={expect}")
    w = wl.make(cfg, a_kind="random", with_h0=True)
    d = upload(w)
    rows = np.unique(np.concatenate([[0, 1, D // 2, D - 2, D - 1], np.random.default_rng(D).integers(0, D, 8)]))
    y_ref, s_ref = oracle_scan(w, rows=rows)
    idx = torch.from_numpy(rows).cuda()
    outs = {}
    for whole_rows in (False, True):
        for routed in (False, True):
            cd = torch.full((B,), chunk, dtype=torch.int32, device="cuda") if routed else None
            y, last = corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"], delta_bias=d["delta_bias"],
                                               h0=d["h0"], seqlens=d["seqlens"], chunk=2048 if routed else chunk, chunks_dev=cd,
                                               general_a=True, whole_rows=whole_rows)
            torch.cuda.synchronize()
            check_y(y_to_f64(y[:, idx, :]), y_ref, cfg, f"y whole_rows={whole_rows} routed={routed}")
            assert_close(last.cpu().numpy()[:, rows, :], s_ref, fp32_rtol(cfg.L), f"state whole_rows={whole_rows} routed={routed}")
            outs[(whole_rows, routed)] = (y, last)
        # the chunk read from device memory picks the same launch shape as the host's
        assert torch.equal(outs[(whole_rows, False)][0], outs[(whole_rows, True)][0])
        assert torch.equal(outs[(whole_rows, False)][1], outs[(whole_rows, True)][1])
    assert torch.equal(outs[(False, False)][1], outs[(True, False)][1])            # the state, bit for bit
    ya, yb = y_to_f64(outs[(False, False)][0]), y_to_f64(outs[(True, False)][0])
    if expect:
        if ya.size >= 2_000_000:                          # (enough values for a sum in another order to cross a 16-bit rounding)
            assert not np.array_equal(ya, yb)             # the two shapes really are different code
    else:
        assert np.array_equal(ya, yb)                     # no split planned: the flag changes nothing
    scale = np.sqrt((yb ** 2).mean(-1, keepdims=True)) + np.abs(yb)
    store = {wl.BF16: 2.0 ** -8, wl.F16: 2.0 ** -11, wl.F32: 0.0}[cfg.dtype]
    assert np.all(np.abs(ya - yb) <= 4e-6 * scale + 2 * store * np.abs(yb))


@pytest.mark.parametrize("chunk", [128, 512, 2048])
def test_structured_path_on_every_row_at_full_size(chunk):
    """Every channel of the benchmark layer, structured path against general path: a workgroup that read A before it was
    in place (a missing barrier once let that happen on a few workgroups per launch) shows up as a row that disagrees."""
    cfg = wl.CONFIGS["c4_mamba2p8b"]
    w = wl.make(cfg)
    d = upload(w)
    _say(f"structured against general, every row, chunk {chunk}")
    res = []
    for general_a in (False, True):
        y, last = corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"],
                                           delta_bias=d["delta_bias"], chunk=chunk, general_a=general_a)
        torch.cuda.synchronize()
        res.append((y.float(), last))
    (y1, s1), (y0, s0) = res
    assert torch.isfinite(y1).all() and torch.isfinite(y0).all()
    tol = 0.01 * (y0.abs() + y0.pow(2).mean(-1, keepdim=True).sqrt())          # a bf16 ulp is 0.4 to 0.8 % of the value
    assert int(((y1 - y0).abs() > tol).sum()) == 0
    assert int(((s1 - s0).abs() > 1e-4 * (s0.abs() + s0.pow(2).mean(-1, keepdim=True).sqrt())).sum()) == 0


def test_mixed_launch_with_padded_sequences_and_a_chunk_per_sequence():
    """Two padded sequences routed to different chunks on the device: one of them splits its channels between both lane
    geometries, the other does not; the grid comes from a third chunk given as the host's hint."""
    B, D = 2, 2100
    cfg = wl.scaled(wl.CONFIGS["c3_mamba1p4b"], B=B, D=D, L=1536, seqlens=(1536, 700))
    _say(f"mixed geometries, padded, per-sequence chunks B{B} D{D}")
    assert corey.selective_scan_fwd_plan(B, D, cfg.N, 512) == 2048 and corey.selective_scan_fwd_plan(B, D, cfg.N, 256) == 0
    w = wl.make(cfg, a_kind="random")
    d = upload(w)
    rows = np.unique(np.concatenate([[0, 1, 2046, 2047, 2048, 2049, D - 1], np.random.default_rng(8).integers(0, D, 10)]))
    y_ref, s_ref = oracle_scan(w, rows=rows)
    chunks_dev = torch.tensor([512, 256], dtype=torch.int32, device="cuda")
    y, last = corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"], delta_bias=d["delta_bias"],
                                       seqlens=d["seqlens"], chunk=128, chunks_dev=chunks_dev)
    torch.cuda.synchronize()
    ys = y[:, torch.from_numpy(rows).cuda(), :]
    assert_close(y_to_f64(ys), y_ref, y_rtol(cfg), "y", store_bits(cfg))
    assert_close(last.cpu().numpy()[:, rows, :], s_ref, fp32_rtol(cfg.L), "state")
    assert (y[1, :, 700:] == 0).all()


@pytest.mark.parametrize("name", ["c1_mamba130m", "c2_mamba370m", "c3_mamba1p4b", "c4_mamba2p8b", "paper_w1_fp16"])
def test_full_size_sampled_rows(name):
    """The benchmark's launch configuration at full size; the oracle recomputes sampled channels one by one.  Every
    launch runs twice: on the general path (COREY_SCAN_GENERAL_A, the path every headline figure is measured on) and with
    the fast path for the layers' structured A left on."""
    cfg = wl.CONFIGS[name]
    w = wl.make(cfg)
    d = upload(w)
    rows = np.unique(np.concatenate([[0, 1, cfg.D // 2, cfg.D - 1], np.random.default_rng(3).integers(0, cfg.D, 12)]))
    y_ref, s_ref = oracle_scan(w, rows=rows)
    ent = corey.corey_entropy_hist(d["u"], cfg.K)
    chunk = corey.corey_select_chunk(ent["r"].item(), cfg.L)
    idx = torch.from_numpy(rows).cuda()
    worst = [0.0, 0.0, 0.0]

    def check(y, last, what):
        assert torch.isfinite(y.to(torch.float32)).all()
        a, b = check_y(y_to_f64(y[:, idx, :]), y_ref, cfg, f"{name} y {what}")
        c = assert_close(last.cpu().numpy()[:, rows, :], s_ref, fp32_rtol(cfg.L), f"{name} state {what}")
        worst[:] = max(worst[0], a), max(worst[1], b), max(worst[2], c)

    for general_a in (True, False):
        for c in sorted({chunk, 64, 512, 1024, 2048}):      # (small layers: two rows per channel up to 1024, one beyond)
            _say(f"scan full size {name} chunk={c} (routed={chunk}) general_a={general_a}")
            y, last = corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"],
                                               delta_bias=d["delta_bias"], seqlens=d["seqlens"], chunk=c, general_a=general_a)
            torch.cuda.synchronize()
            check(y, last, f"chunk {c} general_a={general_a}")
        # the launch the benchmark times: statistic and rule on the GPU, the scan reading the chunk from device memory
        _say(f"scan full size {name} device-routed general_a={general_a}")
        route = corey.corey_route_device(d["u"], cfg.K, corey.policy_default(), seqlens=d["seqlens"])
        y, last = corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"], delta_bias=d["delta_bias"],
                                           seqlens=d["seqlens"], chunk=chunk, chunks_dev=route["chunks"], general_a=general_a)
        torch.cuda.synchronize()
        check(y, last, f"device-routed general_a={general_a}")
    print(f"[worst] {name}: y error / stated bound {worst[0]:.3f}, / fp32 computation bound {worst[1]:.3f}, state / bound {worst[2]:.3f}",
          flush=True)


@pytest.mark.parametrize("general_a", [True, False])
@pytest.mark.parametrize("lens", [(8192, 512), (8192, 2048), (2048, 512), (8192, 8192)])
def test_padded_pairs_of_the_mixed_regime_layer_at_full_size(lens, general_a):
    """The mixed-regime layer (two sequences of a 1.4B-shaped layer, right-padded to 8192) with the other pairs of its
    three prompt lengths: per-sequence statistic and rule on the GPU, the scan reading each sequence's chunk from device
    memory.  Counts against the oracle on everything, y and state on sampled channels."""
    import oracle
    cfg = wl.scaled(wl.CONFIGS["c3_mamba1p4b"], seqlens=lens)
    _say(f"mixed-regime pair {lens} at full size general_a={general_a}")
    w = wl.make(cfg)
    d = upload(w)
    rows = np.unique(np.concatenate([[0, 1, cfg.D - 1], np.random.default_rng(sum(lens)).integers(0, cfg.D, 9)]))
    y_ref, s_ref = oracle_scan(w, rows=rows)
    pol = corey.policy_default()
    pol.mode = 1                                                  # sequence-length gate, then the entropy rule
    route = corey.corey_route_device(d["u"], cfg.K, pol, seqlens=d["seqlens"])
    y, last = corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"], delta_bias=d["delta_bias"],
                                       seqlens=d["seqlens"], chunk=512, chunks_dev=route["chunks"], general_a=general_a)
    torch.cuda.synchronize()
    ref = oracle.entropy_hist(w.val["u"], cfg.K, seqlens=w.seqlens)
    assert np.array_equal(route["counts"].cpu().numpy().view(np.uint32).reshape(ref["counts"].shape), ref["counts"])
    opol = oracle.policy(mode=1)
    for b, n in enumerate(lens):
        st, c, margin = oracle.select_chunk(float(ref["r"][b]), n, opol)
        assert st == oracle.OK and (margin < 1e-9 or route["chunks"][b].item() == c)
    ys = y[:, torch.from_numpy(rows).cuda(), :]
    check_y(y_to_f64(ys), y_ref, cfg, "y")
    assert_close(last.cpu().numpy()[:, rows, :], s_ref, fp32_rtol(cfg.L), "state")
    for b, n in enumerate(lens):
        assert (y[b, :, n:] == 0).all()


@pytest.mark.parametrize("chunk", [64, 512, 2048])
def test_very_long_sequence(chunk):
    """262144 steps on a few channels (hundreds to thousands of tiles per row, a ragged last tile, B and C of 16 MB): the
    carried state and the tile bookkeeping over a long run; the tolerance on the fp32 state grows with sqrt(L)."""
    cfg = wl.scaled(wl.CONFIGS["c1_mamba130m"], D=6, L=262144 - 24)
    _say(f"scan L={cfg.L} chunk {chunk}")
    w = wl.make(cfg, a_kind="random", with_h0=True)
    d = upload(w)
    y_ref, s_ref = oracle_scan(w)
    y, s = _run(d, chunk)
    assert_close(y, y_ref, y_rtol(cfg), "y", store_bits(cfg))
    assert_close(s, s_ref, fp32_rtol(cfg.L), "state")
    ent = corey.corey_entropy_hist(d["u"], 4096)
    ref = oracle.entropy_hist(w.val["u"], 4096)
    assert np.array_equal(ent["counts"].cpu().numpy().view(np.uint32).reshape(ref["counts"].shape), ref["counts"])


def test_more_than_two_to_the_31_elements():
    """One tensor of 2.2e9 elements (4.4 GB in bf16): every index that is a product of sizes has to be 64-bit.  Inputs are
    drawn on the GPU (seeded); the oracle recomputes three channels, the histogram is checked against plain torch
    operations that follow the stated binary32 bin arithmetic."""
    B, D, N, L, K = 1, 2100, 16, (1 << 20) + 8, 256
    assert B * D * L > (1 << 31)
    _say(f"scan and histogram on {B * D * L} elements")
    g = torch.Generator(device="cuda").manual_seed(77)
    rnd = lambda *shape, scale=1.0: (torch.randn(*shape, generator=g, device="cuda", dtype=torch.float32) * scale)
    u = torch.empty((B, D, L), dtype=torch.bfloat16, device="cuda")
    delta, z = torch.empty_like(u), torch.empty_like(u)
    for t in (u, delta, z):                                      # row blocks: no 8.8 GB fp32 temporary
        for d0 in range(0, D, 300):
            t[:, d0:d0 + 300] = rnd(B, min(300, D - d0), L, scale=0.5 if t is delta else 1.0).to(torch.bfloat16)
    Bm, Cm = rnd(B, N, L).to(torch.bfloat16), rnd(B, N, L).to(torch.bfloat16)
    A = -torch.exp(rnd(D, N))
    Dv, bias = rnd(D), torch.log(torch.rand(D, generator=g, device="cuda") * 0.099 + 0.001)
    y, last = corey.selective_scan_fwd(u, delta, A, Bm, Cm, Dv=Dv, z=z, delta_bias=bias, chunk=1024)
    torch.cuda.synchronize()
    rows = [0, D // 2 + 1, D - 1]
    f = lambda t: t.float().cpu().numpy()
    st, y_ref, s_ref = oracle.selective_scan(f(u[:, rows]), f(delta[:, rows]), f(A[rows]), f(Bm), f(Cm), Dv=f(Dv[rows]), z=f(z[:, rows]),
                                             delta_bias=f(bias[rows]), chunk=256, threads=3)
    assert st == oracle.OK
    assert_close(f(y[:, rows]).astype(np.float64), y_ref, 3e-3, "y", True)
    assert_close(last[:, rows].cpu().numpy().astype(np.float64), s_ref, fp32_rtol(L), "state")
    assert bool(torch.isfinite(last).all())

    ent = corey.corey_entropy_hist(u, K)
    torch.cuda.synchronize()
    lo, hi = ent["range"].reshape(-1).tolist()
    assert lo == min(u[:, d0:d0 + 300].min().item() for d0 in range(0, D, 300))
    assert hi == max(u[:, d0:d0 + 300].max().item() for d0 in range(0, D, 300))
    scale = torch.tensor(np.float32(np.float64(K) / (np.float64(hi) - np.float64(lo))), device="cuda")
    counts = torch.zeros(K, dtype=torch.int64, device="cuda")
    for d0 in range(0, D, 100):
        q = (u[:, d0:d0 + 100].float() - lo) * scale             # two separate binary32 operations
        counts += torch.bincount(q.to(torch.int32).clamp_(max=K - 1).reshape(-1), minlength=K)
    got = ent["counts"].reshape(-1).to(torch.int64) & 0xFFFFFFFF
    assert torch.equal(got, counts) and int(counts.sum()) == B * D * L
