"""The seeded input generators: storage rounding agrees with a library conversion, draws are reproducible,
and the named configurations have the shapes the benchmark states."""
import numpy as np
import torch

from paper_2604_10597_amd import workloads as wl


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 37,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, np.inf, -np.inf],
                                 dtype=np.float32)])
    bits = wl.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(wl.bf16_bits_to_f32(bits), ref.to(torch.float32).numpy())


def test_fp16_rounding_matches_torch():
    rng = np.random.default_rng(1)
    a = (rng.standard_normal(50000) * 50).astype(np.float32)
    store, val = wl.store(a, wl.F16)
    ref = torch.from_numpy(a).to(torch.float16)
    assert np.array_equal(store.view(np.uint16), ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(val, ref.to(torch.float32).numpy())


def test_shapes_and_reproducibility():
    cfg = wl.scaled(wl.CONFIGS["c2_mamba370m"], D=8, L=64)
    a, b = wl.make(cfg), wl.make(cfg)
    for k in a.dev:
        assert (a.dev[k] is None and b.dev[k] is None) or np.array_equal(a.dev[k], b.dev[k])
    assert a.dev["u"].dtype == np.uint16 and a.dev["u"].shape == (4, 8, 64)
    assert a.val["u"].dtype == np.float32 and a.dev["A"].shape == (8, 16) and a.dev["B"].shape == (4, 16, 64)
    assert np.array_equal(a.val["A"][3], -np.arange(1, 17, dtype=np.float32))
    c0 = wl.make(wl.CONFIGS["c0_tiny_f32"])
    assert c0.dev["u"].dtype == np.float32 and c0.dev["u"].shape == (1, 64, 256)
    c4 = wl.CONFIGS["c4_mamba2p8b"]
    assert (c4.B, c4.D, c4.N, c4.L) == (1, 5120, 16, 16384)
    assert abs(wl.scan_bytes(c4) / 1e6 - 672.8) < 0.5          # the stated algorithmic traffic at that shape
    w = wl.make(wl.scaled(c4, D=200, L=128))
    hot = np.abs(w.val["u"][0]).max(axis=1) > 10
    assert hot.sum() == 2                                       # 1 % of 200 channels scaled x20
