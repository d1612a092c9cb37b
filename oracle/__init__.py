"""CPU oracle for the COREY hot path (test infrastructure only).

Thin ctypes loader around ``corey_oracle.c``.  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product package never does, and this package
never imports the product.  All arithmetic lives in the C file; this module only marshals numpy
arrays into it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "corey_oracle.c")
_LIB = os.path.join(_HERE, "libcorey_oracle.so")

OK, EINVAL, ENONFINITE = 0, 1, 4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (double precision, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fopenmp",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class Policy(ctypes.Structure):
    """Mirror of ``oracle_policy`` (scheduler family around Eq. 2)."""
    _fields_ = [("mode", ctypes.c_int32), ("c_min", ctypes.c_int32), ("c_max", ctypes.c_int32),
                ("h_ref_scale", ctypes.c_double), ("short_len", ctypes.c_int32),
                ("short_chunk", ctypes.c_int32), ("long_chunk", ctypes.c_int32),
                ("static_chunk", ctypes.c_int32), ("safe_chunk", ctypes.c_int32),
                ("guard_buckets", ctypes.c_int32)]


def policy(mode=0, c_min=64, c_max=2048, h_ref_scale=1.0, short_len=50, short_chunk=128,
           long_chunk=512, static_chunk=512, safe_chunk=512, guard_buckets=2) -> Policy:
    return Policy(mode, c_min, c_max, h_ref_scale, short_len, short_chunk, long_chunk,
                  static_chunk, safe_chunk, guard_buckets)


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_entropy_hist.restype = ctypes.c_int
        _lib.oracle_select_chunk.restype = ctypes.c_int
        _lib.oracle_selective_scan.restype = ctypes.c_int
        _lib.oracle_max_threads.restype = ctypes.c_int
    return _lib


def _f32(a):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _i32(a):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def entropy_hist(x, K, eps=1e-8, stride=1, seqlens=None, block=1, range_all=False):
    """x: float array [B, D, L] (already widened).  Returns dict(status, counts, H, r, lo, hi).
    range_all: bins bounded by the minimum / maximum of all values rather than of the sampled ones."""
    x = np.asarray(x)
    if x.ndim != 3:
        raise ValueError("x must be [B, D, L]")
    B, D, L = x.shape
    xk, xp = _f32(x)
    sk, sp = _i32(seqlens)
    nh = B if seqlens is not None else 1
    counts = np.zeros((nh, K), dtype=np.uint32)
    H = np.zeros(nh, dtype=np.float64)
    r = np.zeros(nh, dtype=np.float64)
    lo = np.zeros(nh, dtype=np.float32)
    hi = np.zeros(nh, dtype=np.float32)
    st = lib().oracle_entropy_hist(
        xp, ctypes.c_int64(B), ctypes.c_int64(D), ctypes.c_int64(L), sp, ctypes.c_int32(K),
        ctypes.c_double(eps), ctypes.c_int64(stride), ctypes.c_int64(block), ctypes.c_int32(1 if range_all else 0),
        counts.ctypes.data_as(ctypes.c_void_p), H.ctypes.data_as(ctypes.c_void_p),
        r.ctypes.data_as(ctypes.c_void_p), lo.ctypes.data_as(ctypes.c_void_p),
        hi.ctypes.data_as(ctypes.c_void_p))
    return dict(status=st, counts=counts, H=H, r=r, lo=lo, hi=hi)


def ema_update(lam, prev, H):
    """One step of the entropy EMA; prev = NaN means no estimate yet."""
    f = lib().oracle_ema_update
    f.restype = ctypes.c_double
    return f(ctypes.c_double(lam), ctypes.c_double(prev), ctypes.c_double(H))


def selective_state_update(state, x, delta, A, Bt, Ct, Dv=None, z=None, delta_bias=None, delta_softplus=True):
    """One decode step.  state [B, D, N], x/delta/z [B, D], A [D, N], Bt/Ct [B, N].  Returns (state_out float64
    [B, D, N], y float64 [B, D])."""
    state = np.asarray(state)
    B, D, N = state.shape
    keep = [_f32(a) for a in (state, x, delta, A, Bt, Ct, Dv, z, delta_bias)]
    so = np.zeros((B, D, N), dtype=np.float64)
    y = np.zeros((B, D), dtype=np.float64)
    f = lib().oracle_selective_state_update
    f.restype = ctypes.c_int
    st = f(*[k[1] for k in keep], ctypes.c_int(1 if delta_softplus else 0), ctypes.c_int64(B), ctypes.c_int64(D),
           ctypes.c_int64(N), so.ctypes.data_as(ctypes.c_void_p), y.ctypes.data_as(ctypes.c_void_p))
    assert st == OK
    return so, y


def causal_conv1d_silu(x, weight, bias=None, state_in=None):
    """x [B, D, L], weight [D, W], bias [D], state_in [B, D, W-1] (float arrays).  Returns (u float64 [B, D, L],
    state_out float32 [B, D, W-1])."""
    x = np.asarray(x)
    B, D, L = x.shape
    W = np.asarray(weight).shape[1]
    xk, xp = _f32(x)
    wk, wp = _f32(weight)
    bk, bp = _f32(bias)
    sk, sp = _f32(state_in)
    u = np.zeros((B, D, L), dtype=np.float64)
    so = np.zeros((B, D, max(W - 1, 0)), dtype=np.float32)
    f = lib().oracle_causal_conv1d_silu
    f.restype = ctypes.c_int
    st = f(xp, wp, bp, sp, ctypes.c_int64(B), ctypes.c_int64(D), ctypes.c_int64(L), ctypes.c_int32(W),
           u.ctypes.data_as(ctypes.c_void_p), so.ctypes.data_as(ctypes.c_void_p))
    assert st == OK
    return u, so


def select_chunk(r, L, pol: Policy | None = None):
    """Returns (status, chunk, margin)."""
    pol = pol or policy()
    chunk = ctypes.c_int32(0)
    margin = ctypes.c_double(0.0)
    st = lib().oracle_select_chunk(ctypes.c_double(r), ctypes.c_int64(L), ctypes.byref(pol),
                                   ctypes.byref(chunk), ctypes.byref(margin))
    return st, chunk.value, margin.value


def selective_scan(u, delta, A, Bm, Cm, Dv=None, z=None, delta_bias=None, delta_softplus=True,
                   h0=None, seqlens=None, chunk=256, threads=1, want_terms=False):
    """All inputs float arrays (widened).  Returns (status, y float64 [B,D,L], last float64 [B,D,N]); with `want_terms`
    also the sum of the absolute values of the terms each y is made of (for a checker's rounding bound)."""
    u = np.asarray(u)
    B, D, L = u.shape
    A = np.asarray(A)
    N = A.shape[1]
    assert A.shape == (D, N)
    assert np.asarray(Bm).shape == (B, N, L) and np.asarray(Cm).shape == (B, N, L)
    keep = []
    ptrs = []
    for a in (u, delta, A, Bm, Cm, Dv, z, delta_bias):
        k, p = _f32(a)
        keep.append(k)
        ptrs.append(p)
    hk, hp = _f32(h0)
    sk, sp = _i32(seqlens)
    y = np.zeros((B, D, L), dtype=np.float64)
    last = np.zeros((B, D, N), dtype=np.float64)
    terms = np.zeros((B, D, L), dtype=np.float64) if want_terms else None
    st = lib().oracle_selective_scan(
        ptrs[0], ptrs[1], ptrs[2], ptrs[3], ptrs[4], ptrs[5], ptrs[6], ptrs[7],
        ctypes.c_int(1 if delta_softplus else 0), hp, sp, ctypes.c_int64(chunk),
        ctypes.c_int64(B), ctypes.c_int64(D), ctypes.c_int64(N), ctypes.c_int64(L),
        y.ctypes.data_as(ctypes.c_void_p), last.ctypes.data_as(ctypes.c_void_p),
        ctypes.c_int(threads), terms.ctypes.data_as(ctypes.c_void_p) if want_terms else None)
    if want_terms:
        return st, y, last, terms
    return st, y, last


def max_threads() -> int:
    return lib().oracle_max_threads()
