"""GPU parity: corey_entropy_hist against the CPU oracle (bit-exact counts; H and r to summation rounding)."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2604_10597_amd as corey
from gpu_util import counts_u32, to_dev
from paper_2604_10597_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[case] {msg}", flush=True)


def _check(x_store, x_val, dtype, K, eps=1e-8, stride=1, seqlens=None, block=1):
    xd = to_dev(x_store, dtype)
    sl = None if seqlens is None else torch.from_numpy(np.asarray(seqlens, dtype=np.int32)).cuda()
    out = corey.corey_entropy_hist(xd, K, eps=eps, stride=stride, seqlens=sl, block=block)
    torch.cuda.synchronize()
    ref = oracle.entropy_hist(x_val, K, eps=eps, stride=stride, seqlens=seqlens, block=block)
    got_counts = counts_u32(out["counts"])
    assert np.array_equal(got_counts, ref["counts"]), "bin counts differ"
    H, r, rng = out["H"].cpu().numpy(), out["r"].cpu().numpy(), out["range"].cpu().numpy()
    for h in range(ref["H"].size):
        if math.isnan(ref["H"][h]):
            assert math.isnan(H[h]) and math.isnan(r[h])
        else:
            assert H[h] == pytest.approx(ref["H"][h], rel=1e-12, abs=1e-14)
            assert r[h] == pytest.approx(ref["r"][h], rel=1e-12, abs=1e-14)
            assert rng[h, 0] == ref["lo"][h] and rng[h, 1] == ref["hi"][h]
    return out, ref


@pytest.mark.parametrize("name,D,L", [("c0_tiny_f32", None, None), ("c1_mamba130m", 96, 2048), ("c2_mamba370m", 64, 1000),
                                       ("c3_mamba1p4b", 48, 1024), ("c4_mamba2p8b", 300, 512)])
def test_configs_at_oracle_size(name, D, L):
    cfg = wl.CONFIGS[name]
    if D:
        sl = None if cfg.seqlens is None else tuple(min(s, L) // (1 if i == 0 else 3) for i, s in enumerate(cfg.seqlens))
        cfg = wl.scaled(cfg, D=D, L=L, seqlens=sl)
    _say(f"entropy {cfg.name} B{cfg.B} D{cfg.D} L{cfg.L} {cfg.dtype} K{cfg.K}")
    w = wl.make(cfg)
    _check(w.dev["u"], w.val["u"], cfg.dtype, cfg.K, seqlens=None if w.seqlens is None else w.seqlens)
    if w.seqlens is not None:                       # the same tensor as one whole-tensor histogram
        _check(w.dev["u"], w.val["u"], cfg.dtype, cfg.K)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16, wl.F16])
@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 3, 7), (2, 5, 37), (3, 4, 2049), (1, 2, 4104)])
def test_ragged_shapes_and_unaligned_rows(dtype, shape):
    _say(f"entropy ragged {shape} {dtype}")
    rng = np.random.default_rng(sum(shape))
    store, val = wl.store(rng.standard_normal(shape).astype(np.float32), dtype)
    for K in (2, 16, 257):
        _check(store, val, dtype, K)
    B, D, L = shape
    lens = np.array([(L * (b + 1)) // (B + 1) for b in range(B)], dtype=np.int32)
    _check(store, val, dtype, 16, seqlens=lens)
    if B > 1:
        lens[0] = 0                                  # an empty sequence: its H and r are NaN, counts zero
        out, ref = _check(store, val, dtype, 16, seqlens=lens)
        assert math.isnan(ref["H"][0])


@pytest.mark.parametrize("stride", [2, 8, 13])
def test_sampled_histogram(stride):
    _say(f"entropy stride {stride}")
    cfg = wl.scaled(wl.CONFIGS["c2_mamba370m"], D=40, L=520)
    w = wl.make(cfg)
    _check(w.dev["u"], w.val["u"], cfg.dtype, 256, stride=stride)
    _check(w.dev["u"], w.val["u"], cfg.dtype, 256, stride=stride, seqlens=np.array([520, 100, 7, 333], np.int32))


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16, wl.F32])
def test_block_sampled_histogram(dtype):
    """Every stride-th block of consecutive values: the flat path (power-of-two blocks of whole 16-byte words, which
    fetches only the sampled runs) and the general path (any block, per-sequence histograms, ragged ends)."""
    cfg = wl.scaled(wl.CONFIGS["c2_mamba370m"], D=40, L=520, dtype=dtype)          # 83200 values: ragged against every block below
    w = wl.make(cfg)
    for stride, block in ((8, 512), (8, 8), (3, 64), (2, 4096), (5, 32768), (8, 262144), (4, 24), (8, 100), (7, 1)):
        _say(f"entropy {dtype} stride {stride} block {block}")
        _check(w.dev["u"], w.val["u"], cfg.dtype, 256, stride=stride, block=block)
    _check(w.dev["u"], w.val["u"], cfg.dtype, 256, stride=4, block=16, seqlens=np.array([520, 100, 7, 333], np.int32))
    cfg = wl.scaled(wl.CONFIGS["c4_mamba2p8b"], D=512, L=4096, dtype=dtype)       # large enough for every workgroup to loop
    w = wl.make(cfg)
    _say(f"entropy {dtype} 2M values stride 8 block 512")
    _check(w.dev["u"], w.val["u"], cfg.dtype, 256, stride=8, block=512)
    # per-sequence histograms over long rows: turns of whole slabs that cross rows, rows with a ragged last slab, and the
    # sampled sweep that skips the vectors of unsampled blocks without fetching them
    cfg = wl.scaled(wl.CONFIGS["c3_mamba1p4b"], B=3, D=6, L=6144, dtype=dtype, seqlens=(6144, 4096, 2056))
    w = wl.make(cfg)
    lens = np.array(cfg.seqlens, np.int32)
    for stride, block in ((1, 1), (8, 512), (2, 8), (4, 2048), (8, 16384), (3, 64), (8, 4)):
        _say(f"entropy {dtype} per sequence, long rows, stride {stride} block {block}")
        _check(w.dev["u"], w.val["u"], cfg.dtype, 64, stride=stride, block=block, seqlens=lens)
    _check(w.dev["u"], w.val["u"], cfg.dtype, 64, stride=8, block=512, seqlens=np.array([6144, 0, 6144], np.int32))


def test_bin_limits_and_eps():
    _say("entropy K limits")
    rng = np.random.default_rng(1)
    store, val = wl.store(rng.laplace(0, 3, (2, 64, 512)).astype(np.float32), wl.BF16)
    for K in (2, 1024, 1025, 4096):
        out, ref = _check(store, val, wl.BF16, K, eps=0.0)
        # 65536 values in up to 4096 bins of a Laplace tail: many bins are empty, and H stays finite without eps
        assert (ref["counts"] == 0).any() or K == 2
        assert np.isfinite(ref["H"]).all() and torch.isfinite(out["H"]).all() and torch.isfinite(out["r"]).all()
    _check(store, val, wl.BF16, 64, eps=1e-12)


def test_degenerate_inputs():
    _say("entropy degenerate")
    const = np.full((1, 4, 96), 2.5, dtype=np.float32)
    out, _ = _check(const, const, wl.F32, 8)
    assert counts_u32(out["counts"])[0, 0] == const.size
    for bad in (np.nan, np.inf, -np.inf):
        x = np.linspace(-1, 1, 4 * 96, dtype=np.float32).reshape(1, 4, 96).copy()
        x[0, 2, 17] = bad
        out, ref = _check(x, x, wl.F32, 8)
        assert ref["status"] == oracle.ENONFINITE and counts_u32(out["counts"]).sum() == 0
    # heavy collisions: almost everything in one bin
    x = np.zeros((1, 64, 1024), dtype=np.float32)
    x[0, 0, 0], x[0, 1, 5] = -90.0, 90.0
    _check(x, x, wl.F32, 256)


def test_uniform_histogram_gives_log_K():
    K = 256
    x = np.tile(np.arange(K, dtype=np.float32), 64).reshape(1, 64, K)
    out = corey.corey_entropy_hist(torch.from_numpy(x).cuda(), K, eps=0.0)
    assert (counts_u32(out["counts"]) == 64).all()
    assert out["H"].item() == pytest.approx(math.log(K), rel=1e-14) and out["r"].item() == pytest.approx(1.0, abs=1e-14)


def test_repeat_runs_are_identical_and_outputs_reusable():
    cfg = wl.scaled(wl.CONFIGS["c4_mamba2p8b"], D=256, L=2048)
    w = wl.make(cfg)
    xd = to_dev(w.dev["u"], cfg.dtype)
    out = corey.corey_entropy_hist(xd, 256)
    first = (counts_u32(out["counts"]).copy(), out["H"].item())
    for _ in range(3):                               # same output and workspace buffers, back to back
        corey.corey_entropy_hist(xd, 256, out=out, workspace=out["workspace"])
    torch.cuda.synchronize()
    assert np.array_equal(counts_u32(out["counts"]), first[0]) and out["H"].item() == first[1]


def test_fp16_whole_tensor_fast_path_and_nan():
    _say("entropy fp16")
    rng = np.random.default_rng(4)
    store, val = wl.store(rng.standard_normal((2, 96, 2048)).astype(np.float32) * 3, wl.F16)
    _check(store, val, wl.F16, 256)
    _check(store, val, wl.F16, 256, stride=8)
    bad = store.copy()
    bad[1, 5, 100] = np.float16(np.nan)
    out, ref = _check(bad, bad.astype(np.float32), wl.F16, 64)
    assert ref["status"] == oracle.ENONFINITE


@pytest.mark.parametrize("name", ["c1_mamba130m", "c2_mamba370m", "c3_mamba1p4b", "c4_mamba2p8b", "paper_w1_fp16"])
def test_full_size_counts_and_routed_chunk(name):
    cfg = wl.CONFIGS[name]
    _say(f"entropy full size {name}")
    w = wl.make(cfg, with_z=False)
    out, ref = _check(w.dev["u"], w.val["u"], cfg.dtype, cfg.K, seqlens=w.seqlens)
    pol, opol = corey.policy_default(), oracle.policy()
    for h in range(ref["r"].size):
        L = int(w.seqlens[h]) if w.seqlens is not None else cfg.L
        st, c_ref, margin = oracle.select_chunk(float(ref["r"][h]), L, opol)
        assert margin > 1e-9, "decision sits on a rounding tie"
        assert corey.corey_select_chunk(out["r"][h].item(), L, pol) == c_ref
