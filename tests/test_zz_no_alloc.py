"""corey_entropy_hist_static (the entry point for callers that cannot allocate) against corey_entropy_hist, through the
C ABI: same counts, H, r and range on two calls in a row that share the library's built-in scratch buffer, the second
on a smaller input; sizes beyond the buffer are refused before any launch."""
import ctypes

import numpy as np
import pytest
import torch

from gpu_util import to_dev
from paper_2604_10597_amd import binding
from paper_2604_10597_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _outs(nh, K):
    return dict(counts=torch.full((nh, K), -1, dtype=torch.int32, device="cuda"),
                H=torch.full((nh,), -1.0, dtype=torch.float64, device="cuda"),
                r=torch.full((nh,), -1.0, dtype=torch.float64, device="cuda"),
                range=torch.full((nh, 2), -1.0, dtype=torch.float32, device="cuda"))


def _both(x, K, seqlens=None, stride=1, block=1, eps=1e-8):
    """One call of each entry point through the raw C ABI; returns their outputs."""
    lib, ptr = binding.lib(), binding._ptr
    B, D, L = x.shape
    nh = B if seqlens is not None else 1
    ws = torch.empty(lib.corey_entropy_hist_workspace(B, K), dtype=torch.uint8, device="cuda")
    a, b = _outs(nh, K), _outs(nh, K)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    st = lib.corey_entropy_hist(ptr(x), binding._dtype_code(x), B, D, L, ptr(seqlens), K, eps, stride, block, ptr(a["counts"]), ptr(a["H"]),
                                ptr(a["r"]), ptr(a["range"]), None, ptr(ws), ws.numel(), stream)
    assert st == 0, lib.corey_last_error()
    st = lib.corey_entropy_hist_static(ptr(x), binding._dtype_code(x), B, D, L, ptr(seqlens), K, eps, stride, block, ptr(b["counts"]),
                                       ptr(b["H"]), ptr(b["r"]), ptr(b["range"]), None, stream)
    assert st == 0, lib.corey_last_error()
    torch.cuda.synchronize()
    return a, b


def _same(a, b, what):
    for k in ("counts", "range"):
        assert torch.equal(a[k], b[k]), (what, k)
    for k in ("H", "r"):                                         # NaN (an empty sequence) on both sides counts as equal
        assert torch.equal(a[k].view(torch.int64), b[k].view(torch.int64)), (what, k)
    assert int(a["counts"].sum()) > 0 or bool(torch.isnan(a["H"]).all())


def test_static_scratch_entry_point_equals_the_workspace_one():
    cases = [
        # (config, D, L, seqlens, K, stride, block): a large call first, then smaller ones on the same built-in buffer
        ("c4_mamba2p8b", 512, 4096, None, 256, 1, 1),
        ("c2_mamba370m", 24, 1000, None, 64, 1, 1),              # fewer bins, fewer values: stale partial counts would show
        ("c3_mamba1p4b", 16, 1024, (1024, 300), 256, 1, 1),      # per-sequence histograms (the general kernels)
        ("c4_mamba2p8b", 64, 2048, None, 4096, 8, 512),          # most bins, sampled
        ("c1_mamba130m", 3, 7, None, 16, 1, 1),                  # a handful of values, unaligned rows
    ]
    for name, D, L, lens, K, stride, block in cases:
        cfg = wl.scaled(wl.CONFIGS[name], D=D, L=L, seqlens=lens)
        print(f"[case] static scratch {name} D{D} L{L} lens {lens} K{K} stride {stride} block {block}", flush=True)
        w = wl.make(cfg, with_z=False)
        x = to_dev(w.dev["u"], cfg.dtype)
        sl = None if w.seqlens is None else torch.from_numpy(w.seqlens).cuda()
        a, b = _both(x, K, sl, stride, block)
        _same(a, b, name)
    # the binding's wrapper goes through the same entry point
    out = binding.corey_entropy_hist_static(x, 16, _outs(1, 16))
    ref = binding.corey_entropy_hist(x, 16)
    torch.cuda.synchronize()
    _same(ref, out, "binding")


def test_static_scratch_limit_is_enforced_on_the_host():
    lib = binding.lib()
    fake, none = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    call = lambda B, K, x=fake: lib.corey_entropy_hist_static(x, 1, B, 4, 8, none, K, 1e-8, 1, 1, fake, fake, fake, none, none, none)
    assert lib.corey_entropy_hist_workspace(1, 4096) <= binding.STATIC_SCRATCH_BYTES
    assert lib.corey_entropy_hist_workspace(64, 256) > binding.STATIC_SCRATCH_BYTES
    assert call(64, 256) == 7 and b"built-in" in lib.corey_last_error()        # COREY_EWORKSPACE, nothing launched
    assert call(8, 4096) == 7
    assert call(1, 1) == 1 and call(0, 16) == 3 and call(1, 16, none) == 2     # the common argument checks still apply
