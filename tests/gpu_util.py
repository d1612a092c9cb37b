"""Helpers for the GPU parity tests: upload a workload, run the oracle on it (or on sampled rows), compare."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2604_10597_amd import workloads as wl

RTOL = {wl.F32: 1e-5, wl.BF16: 3e-3}


def fp32_rtol(L: int) -> float:
    """Tolerance on quantities kept in fp32 end to end (y for fp32 storage, the carried state always).

    1e-5 is the bound stated for the fp32 configuration (L = 256).  Every step rounds the decay exp(dl A) and the
    state update to binary32 (relative 2^-24 each); a state whose decay is close to 1 remembers up to L steps, so
    these independent roundings add up like a random walk, ~ sqrt(L) * 6e-8 of the state's scale (1.5e-6 at
    L = 256 typical, several times that in the tail of many thousand elements).  The bound therefore grows with
    sqrt(L / 256) for sequences longer than the stated configuration.
    """
    return 1e-5 * max(1.0, (L / 256.0) ** 0.5)


def y_rtol(cfg) -> float:
    """fp32 and fp16 storage: the fp32 computation bound (the fp16 store's half ulp is granted separately);
    bf16 storage: the stated 3e-3."""
    return RTOL[wl.BF16] if cfg.dtype == wl.BF16 else fp32_rtol(cfg.L)


def store_bits(cfg) -> int:
    """Significand bits of the storage type of y (0: fp32, no store rounding to grant)."""
    return {wl.F32: 0, wl.BF16: 8, wl.F16: 11}[cfg.dtype]


def to_dev(arr, dtype):
    """Storage array from workloads.store -> GPU tensor of that storage type."""
    if arr is None:
        return None
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).cuda().view(torch.bfloat16)
    if arr.dtype == np.float16:
        return torch.from_numpy(arr).cuda()
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def upload(w: wl.Workload):
    d = {k: to_dev(v, w.cfg.dtype) for k, v in w.dev.items()}
    d["seqlens"] = None if w.seqlens is None else torch.from_numpy(w.seqlens).cuda()
    return d


def y_to_f64(y: torch.Tensor) -> np.ndarray:
    return y.to(torch.float32).cpu().numpy().astype(np.float64)


def counts_u32(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def oracle_scan(w: wl.Workload, rows=None, chunk=256, use_z=True, use_h0=True, threads=8):
    """Oracle on all rows, or on the channel subset `rows` (same B, C and parameters)."""
    v = w.val
    sel = slice(None) if rows is None else np.asarray(rows)
    pick3 = lambda a: None if a is None else np.ascontiguousarray(a[:, sel, :])
    pick1 = lambda a: None if a is None else np.ascontiguousarray(a[sel])
    st, y, last = oracle.selective_scan(
        pick3(v["u"]), pick3(v["delta"]), pick1(v["A"]), v["B"], v["C"], Dv=pick1(v["D"]),
        z=pick3(v["z"]) if use_z else None, delta_bias=pick1(v["delta_bias"]), delta_softplus=True,
        h0=pick3(v["h0"]) if (use_h0 and v.get("h0") is not None) else None,
        seqlens=w.seqlens, chunk=chunk, threads=threads)
    assert st == oracle.OK
    return y, last


def assert_close(got: np.ndarray, ref: np.ndarray, rtol: float, what: str, stored_bf16=False, terms=None):
    """|got - ref| <= rtol * (|ref| + rms of the reference row)  [+ 2^-22 * terms]  [+ half an ulp of the storage type of y].

    `stored_bf16`: False / 0 (fp32 result), True / 8 (bfloat16: 8 significand bits) or 11 (binary16).

    The first term is the tolerance on the fp32 computation, relative to the value and to the row's scale (a sum
    over states that cancels is not held to a relative bound on its own tiny value).  When the result is stored
    as bfloat16 the store itself rounds by up to half an ulp (2^-8 relative just above a power of two, i.e. more
    than 3e-3), so that rounding is granted on top: the value before the store must lie within rtol.

    `terms` (the oracle's sum of the absolute values of the terms every y is made of): the row's rms stands in for the size
    of those terms, which it cannot when a row has one or two valid steps (rms of the row = the value itself) and the sum
    over states happens to cancel.  Each binary32 term carries a few roundings of its own (the decay's exponential, two
    products, the fused update: about four times 2^-24 relative), so the sum is off by up to 2^-22 times the sum of the
    absolute terms whatever the sum's own value; given `terms`, that much is granted on top (about a twentieth of the first
    term for an ordinary row)."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    bound = rtol * (np.abs(ref) + rms) + 1e-30
    if terms is not None:
        bound = bound + 2.0 ** -22 * np.asarray(terms, dtype=np.float64)
    bits = 8 if stored_bf16 is True else int(stored_bf16)
    if bits:
        with np.errstate(divide="ignore"):
            e = np.floor(np.log2(np.abs(ref) + bound))
        e = np.maximum(e, -14.0) if bits == 11 else e           # binary16 spacing stops shrinking below 2^-14
        bound = bound + np.where(ref != 0, 2.0 ** (e - bits), 0.0)
    err = np.abs(got - ref)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err / bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} outside tolerance {rtol}; worst at {i}: "
                             f"got {got[i]!r} ref {ref[i]!r} err {err[i]:.3e} bound {bound[i]:.3e}")
    return float((err / bound).max())


def check_y(got, ref, cfg, what):
    """y against the oracle: the stated bound (1e-5 fp32 / 3e-3 for bf16 inputs, plus the store's half ulp), and for
    16-bit storage also a tighter one that bites: the inputs are the same bits on both sides and all arithmetic is
    binary32, so the value *before* the store must meet the fp32 computation bound; only the one rounding of the store
    (half an ulp of the storage type) comes on top.  Returns (error / stated bound, error / tight bound), worst element."""
    stated = assert_close(got, ref, y_rtol(cfg), what, store_bits(cfg))
    tight = stated
    if cfg.dtype != wl.F32:
        tight = assert_close(got, ref, fp32_rtol(cfg.L), what + " (fp32 computation bound + store rounding)", store_bits(cfg))
    return stated, tight


def chain_rtol(N: int) -> float:
    """Bound on the difference between the structured-A path and the general path (both on the GPU), relative to the
    state's value and its row's scale.  The structured path forms the decay of state n as the (n+1)-th power of state 0's
    by n multiplications, i.e. n roundings more than the general path's single exponential: independent relative errors of
    about 0.29 * 2^-24 each (uniform rounding), sqrt(n) * 1.7e-8 per factor.  A state with |A_n| = n + 1 remembers about
    m = 1 / (dl (n + 1)) steps whose factor errors add like a random walk, so the state differs by about
    sqrt(m n) * 1.7e-8 <= sqrt(1 / dl_min) * 1.7e-8; the benchmark recipe's smallest step sizes are about 2.5e-4
    (softplus of a -1.5 sigma draw plus the lowest bias), giving 1.1e-6 rms, and 3.6 sigma over the few ten thousand
    state values of a test is 4e-6.  It does not grow with N: deeper chains belong to faster-decaying states."""
    del N
    return 4e-6
