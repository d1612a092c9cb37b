"""Seeded synthetic inputs for the COREY hot path (numpy only; none of the method's arithmetic).

Both the HIP path and the CPU oracle are fed from here so that they see the same bit patterns.  The
module draws random tensors, rounds them to the storage type of the configuration and hands back
(i) the storage bits for upload and (ii) the exactly-widened float32 values for the oracle.  It knows
nothing about histograms, chunks or recurrences.

The five named configurations are the benchmark's: Mamba-shaped layers whose scan input ``u`` has the
layout [batch, d_inner, L] (the post-convolution tensor the paper's entropy hook reads, see its
"Real-Checkpoint Entropy Validation"), with the value distributions of the paper's perturbation sweep
(normal, Laplace-tailed, outlier-scaled) standing in for its real-prompt workloads, which are not
available offline.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

F32 = "f32"
BF16 = "bf16"
F16 = "f16"


# ----------------------------------------------------------------------------- storage helpers
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round to nearest, ties to even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    w = a.view(np.uint32).astype(np.uint64)
    nan = (w & 0x7FFFFFFF) > 0x7F800000
    r = (w + 0x7FFF + ((w >> 16) & 1)) >> 16
    r = np.where(nan, (w >> 16) | 0x40, r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def store(a: np.ndarray, dtype: str):
    """Return (storage array for upload, float32 values that storage represents)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == F32:
        return a, a
    if dtype == F16:
        h = a.astype(np.float16)                  # IEEE round to nearest even
        return h, h.astype(np.float32)
    bits = f32_to_bf16_bits(a)
    return bits, bf16_bits_to_f32(bits)


# ----------------------------------------------------------------------------- configurations
@dataclass(frozen=True)
class Config:
    name: str
    B: int
    D: int
    N: int
    L: int
    dtype: str
    K: int
    chunks: tuple
    u_kind: str = "normal"         # normal | mixture | outlier_channels
    seqlens: tuple | None = None   # per-sequence valid lengths (right padded to L)
    seed: int = 0


_SWEEP = (64, 128, 256, 512, 1024, 2048)

CONFIGS = {
    "c0_tiny_f32": Config("c0_tiny_f32", 1, 64, 16, 256, F32, 16, (64, 128, 256), seed=1000),
    "c1_mamba130m": Config("c1_mamba130m", 1, 1536, 16, 2048, BF16, 256, _SWEEP, seed=1001),
    "c2_mamba370m": Config("c2_mamba370m", 4, 2048, 16, 4096, BF16, 256, _SWEEP, "mixture", seed=1002),
    "c3_mamba1p4b": Config("c3_mamba1p4b", 2, 4096, 16, 8192, BF16, 256, _SWEEP, seqlens=(8192, 2048),
                           seed=1003),
    "c4_mamba2p8b": Config("c4_mamba2p8b", 1, 5120, 16, 16384, BF16, 256, _SWEEP, "outlier_channels",
                           seed=1004),
    # the shape of the paper's own kernel-level benchmark (batch 1, d 1024, L 4096, d_state 16, FP16 standard-normal
    # activations, K = 256): reported beside the build's configurations for context
    "paper_w1_fp16": Config("paper_w1_fp16", 1, 1024, 16, 4096, F16, 256, _SWEEP, seed=1005),
}
# The mixed-regime configuration lists three lengths for a batch of two: these are the pairs it is run on.
C3_LENGTH_PAIRS = ((8192, 512), (8192, 2048), (2048, 512), (8192, 8192))


def scaled(cfg: Config, D: int | None = None, L: int | None = None, B: int | None = None,
           seqlens: tuple | None = None, dtype: str | None = None, N: int | None = None) -> Config:
    """Same recipe at another size (parity cases the oracle finishes in seconds)."""
    return Config(cfg.name + "_scaled", B or cfg.B, D or cfg.D, N or cfg.N, L or cfg.L,
                  dtype or cfg.dtype, cfg.K, cfg.chunks, cfg.u_kind,
                  seqlens if seqlens is not None else cfg.seqlens, cfg.seed)


@dataclass
class Workload:
    cfg: Config
    # storage arrays (what is uploaded): float32 for F32 configs, uint16 bf16 bits otherwise
    dev: dict = field(default_factory=dict)
    # float32 values those storage arrays represent (what the oracle reads)
    val: dict = field(default_factory=dict)
    seqlens: np.ndarray | None = None


def make(cfg: Config, a_kind: str = "mamba", with_z: bool = True, with_h0: bool = False) -> Workload:
    """Draw one workload.  Order of draws is fixed: u, delta, delta_bias, B, C, D, z, (h0).

    u        normal: N(0,1).  mixture: each element N(0,1) w.p. 0.7 else Laplace(0, b=3).
             outlier_channels: N(0,1) with 1 % of the channels (chosen by the generator) scaled x20.
    delta    N(0, sigma=0.5) -- the raw value; the scan adds delta_bias and applies softplus.
    delta_bias[d] ~ U(ln 1e-3, ln 1e-1).
    A[d,n]   "mamba": -(n+1) (the S4D-real initialisation every benchmark configuration uses);
             "random": -exp(N(0,1)) per element (no structure across n; used by tests).
    B, C     [B, N, L] ~ N(0,1).   D[d], z ~ N(0,1).
    """
    rng = np.random.default_rng(cfg.seed)
    B, D, N, L = cfg.B, cfg.D, cfg.N, cfg.L
    f = np.float32

    u = rng.standard_normal((B, D, L), dtype=f)
    if cfg.u_kind == "mixture":
        pick = rng.random((B, D, L), dtype=f) < f(0.3)
        lap = rng.laplace(0.0, 3.0, size=(B, D, L)).astype(f)
        u = np.where(pick, lap, u)
        del pick, lap
    elif cfg.u_kind == "outlier_channels":
        n_out = max(1, int(round(0.01 * D)))
        ch = rng.choice(D, size=n_out, replace=False)
        u[:, ch, :] *= f(20.0)
    delta = (rng.standard_normal((B, D, L), dtype=f) * f(0.5)).astype(f)
    delta_bias = rng.uniform(np.log(1e-3), np.log(1e-1), size=D).astype(f)
    Bm = rng.standard_normal((B, N, L), dtype=f)
    Cm = rng.standard_normal((B, N, L), dtype=f)
    Dv = rng.standard_normal(D, dtype=f)
    z = rng.standard_normal((B, D, L), dtype=f) if with_z else None
    h0 = rng.standard_normal((B, D, N), dtype=f) if with_h0 else None
    if a_kind == "mamba":
        A = -np.broadcast_to(np.arange(1, N + 1, dtype=f), (D, N)).copy()
    elif a_kind == "random":
        A = -np.exp(rng.standard_normal((D, N), dtype=f)).astype(f)
    else:
        raise ValueError(a_kind)

    w = Workload(cfg)
    for name, arr in (("u", u), ("delta", delta), ("B", Bm), ("C", Cm), ("z", z)):
        if arr is None:
            w.dev[name] = w.val[name] = None
        else:
            w.dev[name], w.val[name] = store(arr, cfg.dtype)
    for name, arr in (("A", A), ("D", Dv), ("delta_bias", delta_bias), ("h0", h0)):
        w.dev[name] = w.val[name] = arr          # parameters and state stay float32
    if cfg.seqlens is not None:
        w.seqlens = np.asarray(cfg.seqlens, dtype=np.int32)
        assert w.seqlens.shape == (B,) and int(w.seqlens.max()) <= L
    return w


def make_conv(cfg: Config, W: int = 4, with_state: bool = False, seed_offset: int = 7919) -> dict:
    """Inputs of the convolution that produces u: x [B, D, L] ~ N(0,1) (1 % of the channels scaled x20 when the
    configuration's u has such outlier channels) rounded to cfg.dtype, weight [D, W] and bias [D]
    ~ U(-1/sqrt(W), 1/sqrt(W)) (the default initialisation of a depthwise Conv1d with W taps), optional
    state_in [B, D, W-1] ~ N(0,1) in the storage type.  Returns {"dev": storage arrays, "val": float32 values}."""
    rng = np.random.default_rng(cfg.seed + seed_offset)
    f = np.float32
    x = rng.standard_normal((cfg.B, cfg.D, cfg.L), dtype=f)
    if cfg.u_kind == "outlier_channels":          # the layer's outlier channels are outliers of its input as well
        ch = rng.choice(cfg.D, size=max(1, int(round(0.01 * cfg.D))), replace=False)
        x[:, ch, :] *= f(20.0)
    k = f(1.0 / np.sqrt(W))
    weight = rng.uniform(-k, k, size=(cfg.D, W)).astype(f)
    bias = rng.uniform(-k, k, size=cfg.D).astype(f)
    out = {"dev": {}, "val": {}}
    out["dev"]["x"], out["val"]["x"] = store(x, cfg.dtype)
    if with_state and W > 1:
        st = rng.standard_normal((cfg.B, cfg.D, W - 1), dtype=f)
        out["dev"]["state_in"], out["val"]["state_in"] = store(st, cfg.dtype)
    else:
        out["dev"]["state_in"] = out["val"]["state_in"] = None
    for name, arr in (("weight", weight), ("bias", bias)):
        out["dev"][name] = out["val"][name] = arr
    return out


def make_decode(cfg: Config, a_kind: str = "mamba", seed_offset: int = 104729) -> dict:
    """Inputs of one generated token for cfg.B sequences (cfg.L is not used): state [B, D, N] float32 ~ N(0,1); x, z
    [B, D] ~ N(0,1) and delta [B, D] ~ N(0, 0.5) in cfg.dtype; Bt, Ct [B, N] ~ N(0,1) in cfg.dtype; A, D, delta_bias as in
    make().  Returns {"dev": storage arrays, "val": float32 values}."""
    rng = np.random.default_rng(cfg.seed + seed_offset)
    f = np.float32
    B, D, N = cfg.B, cfg.D, cfg.N
    out = {"dev": {}, "val": {}}
    state = rng.standard_normal((B, D, N), dtype=f)
    for name, arr in (("x", rng.standard_normal((B, D), dtype=f)), ("delta", rng.standard_normal((B, D), dtype=f) * f(0.5)),
                      ("z", rng.standard_normal((B, D), dtype=f)), ("Bt", rng.standard_normal((B, N), dtype=f)),
                      ("Ct", rng.standard_normal((B, N), dtype=f))):
        out["dev"][name], out["val"][name] = store(arr, cfg.dtype)
    if a_kind == "mamba":
        A = -np.broadcast_to(np.arange(1, N + 1, dtype=f), (D, N)).copy()
    else:
        A = -np.exp(rng.standard_normal((D, N), dtype=f)).astype(f)
    for name, arr in (("state", state), ("A", A), ("D", rng.standard_normal(D, dtype=f)),
                      ("delta_bias", rng.uniform(np.log(1e-3), np.log(1e-1), size=D).astype(f))):
        out["dev"][name] = out["val"][name] = arr
    return out


def decode_bytes(cfg: Config) -> int:
    """Bytes one decode step must move: the state read and written, A once, the per-row scalars and y."""
    s = 4 if cfg.dtype == F32 else 2
    return 8 * cfg.B * cfg.D * cfg.N + 4 * cfg.D * cfg.N + 4 * cfg.B * cfg.D * s + 2 * cfg.B * cfg.N * s + 8 * cfg.D


def conv_bytes(cfg: Config) -> int:
    """Bytes the convolution must move once: x in, u out (parameters are negligible)."""
    s = 4 if cfg.dtype == F32 else 2
    return 2 * cfg.B * cfg.D * cfg.L * s


def scan_bytes(cfg: Config, with_z: bool = True, with_h0: bool = False) -> int:
    """Bytes the scan must move once: u, delta, (z) in over the valid tokens, B and C once over the valid tokens, y out
    over all B*L positions (padded positions are written as zero), parameters, final state."""
    s = 4 if cfg.dtype == F32 else 2
    valid = sum(cfg.seqlens) if cfg.seqlens is not None else cfg.B * cfg.L
    n = ((3 if with_z else 2) * cfg.D * valid + cfg.B * cfg.D * cfg.L) * s + 2 * cfg.N * valid * s
    n += 4 * cfg.D * cfg.N + 8 * cfg.D + 4 * cfg.B * cfg.D * cfg.N * (2 if with_h0 else 1)
    return n


def entropy_bytes(cfg: Config, passes: int = 2) -> int:
    """Bytes the exact statistic reads: `passes` sweeps over u plus the K counters."""
    s = 4 if cfg.dtype == F32 else 2
    return passes * cfg.B * cfg.D * cfg.L * s + 4 * cfg.K
