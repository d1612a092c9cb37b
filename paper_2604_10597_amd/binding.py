"""ctypes binding of libcorey.so: argument marshalling only.

Functions carry the names of the C entry points (include/corey.h).  Device buffers are torch tensors
(torch is used for GPU memory and streams, nothing else); every step of the path runs in the library's
HIP kernels.  There is no fallback: if the library is missing or fails to load, calls raise.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("COREY_LIB") or os.path.join(_HERE, "libcorey.so")   # COREY_LIB: another build of the same library

COREY_F32, COREY_BF16, COREY_F16 = 0, 1, 2
STATUS = {0: "COREY_OK", 1: "COREY_EINVAL", 2: "COREY_ENULL", 3: "COREY_ESHAPE", 4: "COREY_ENONFINITE",
          5: "COREY_EUNSUPPORTED", 6: "COREY_EHIP", 7: "COREY_EWORKSPACE"}
EXPORTS = ("corey_entropy_hist", "corey_entropy_hist_static", "corey_entropy_hist_workspace", "corey_pattern_table_workspace",
           "corey_entropy_hist_onesweep", "corey_entropy_hist_from_table", "corey_policy_default", "corey_select_chunk",
           "corey_select_chunk_device", "corey_route_device", "corey_route_device_deferred", "selective_scan_fwd_routed", "corey_ema_update", "causal_conv1d_silu_fwd", "selective_state_update",
           "selective_scan_fwd", "selective_scan_fwd_workspace", "selective_scan_fwd_plan", "selective_scan_fwd_plan_steps", "selective_scan_fwd_plan_split", "corey_last_error", "corey_version")


class CoreyError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code


class Policy(ctypes.Structure):
    """corey_policy"""
    _fields_ = [("mode", ctypes.c_int32), ("c_min", ctypes.c_int32), ("c_max", ctypes.c_int32),
                ("h_ref_scale", ctypes.c_double), ("short_len", ctypes.c_int32), ("short_chunk", ctypes.c_int32),
                ("long_chunk", ctypes.c_int32), ("static_chunk", ctypes.c_int32), ("safe_chunk", ctypes.c_int32),
                ("guard_buckets", ctypes.c_int32)]


class DeferredRoute(ctypes.Structure):
    """corey_deferred_route: opaque, filled by corey_route_device_deferred, consumed by selective_scan_fwd_routed"""
    _fields_ = [("opaque", ctypes.c_uint64 * 40)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libcorey.so (built in-tree by build.py); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        i64, i32, vp, dbl = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_double
        L.corey_entropy_hist.restype = ctypes.c_int
        L.corey_entropy_hist.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, i32, dbl, i64, i64, vp, vp, vp, vp, vp, vp,
                                         ctypes.c_size_t, vp]
        L.corey_entropy_hist_static.restype = ctypes.c_int
        L.corey_entropy_hist_static.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, i32, dbl, i64, i64, vp, vp, vp, vp, vp, vp]
        L.corey_pattern_table_workspace.restype = ctypes.c_size_t
        L.corey_pattern_table_workspace.argtypes = []
        L.corey_entropy_hist_onesweep.restype = ctypes.c_int
        L.corey_entropy_hist_onesweep.argtypes = [vp, ctypes.c_int, i64, i64, i64, i32, dbl, ctypes.POINTER(Policy), vp, vp, vp, vp, vp, vp,
                                                  ctypes.c_size_t, vp]
        L.corey_entropy_hist_from_table.restype = ctypes.c_int
        L.corey_entropy_hist_from_table.argtypes = [ctypes.c_int, i64, i32, dbl, ctypes.POINTER(Policy), vp, vp, vp, vp, vp, vp,
                                                    ctypes.c_size_t, vp]
        L.selective_state_update.restype = ctypes.c_int
        L.selective_state_update.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, ctypes.c_int, i64, i64, i64, vp]
        L.causal_conv1d_silu_fwd.restype = ctypes.c_int
        L.causal_conv1d_silu_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, ctypes.c_int, i64, i64, i64, i32, vp]
        L.corey_route_device.restype = ctypes.c_int
        L.corey_route_device.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, i32, dbl, i64, i64, ctypes.POINTER(Policy), dbl, vp, vp,
                                         vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.corey_route_device_deferred.restype = ctypes.c_int
        L.corey_route_device_deferred.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, i32, dbl, i64, i64, ctypes.POINTER(Policy), vp,
                                                  vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, ctypes.POINTER(DeferredRoute), vp]
        L.selective_scan_fwd_routed.restype = ctypes.c_int
        L.selective_scan_fwd_routed.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp, i32, ctypes.POINTER(DeferredRoute),
                                                vp, vp, ctypes.c_int, i64, i64, i64, i64, ctypes.c_uint32, vp, ctypes.c_size_t, vp]
        L.corey_ema_update.restype = ctypes.c_int
        L.corey_ema_update.argtypes = [dbl, ctypes.POINTER(dbl), dbl]
        L.corey_entropy_hist_workspace.restype = ctypes.c_size_t
        L.corey_entropy_hist_workspace.argtypes = [i64, i32]
        L.corey_policy_default.restype = ctypes.c_int
        L.corey_policy_default.argtypes = [ctypes.POINTER(Policy)]
        L.corey_select_chunk.restype = ctypes.c_int
        L.corey_select_chunk.argtypes = [dbl, i64, ctypes.POINTER(Policy), ctypes.POINTER(i32)]
        L.corey_select_chunk_device.restype = ctypes.c_int
        L.corey_select_chunk_device.argtypes = [vp, vp, i64, i32, ctypes.POINTER(Policy), vp, vp]
        L.selective_scan_fwd.restype = ctypes.c_int
        L.selective_scan_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp, i32, vp, vp, vp,
                                         ctypes.c_int, i64, i64, i64, i64, ctypes.c_uint32, vp, ctypes.c_size_t, vp]
        L.selective_scan_fwd_plan.restype = ctypes.c_int64
        L.selective_scan_fwd_plan.argtypes = [i64, i64, i64, i32]
        L.selective_scan_fwd_plan_steps.restype = i32
        L.selective_scan_fwd_plan_steps.argtypes = [i64, i64, i64, i32]
        L.selective_scan_fwd_plan_split.restype = i32
        L.selective_scan_fwd_plan_split.argtypes = [i64, i64, i64, i32]
        L.selective_scan_fwd_workspace.restype = ctypes.c_size_t
        L.selective_scan_fwd_workspace.argtypes = [i64, i64, i64]
        L.corey_last_error.restype = ctypes.c_char_p
        L.corey_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(code: int):
    if code != 0:
        raise CoreyError(code, lib().corey_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return COREY_F32
    if t.dtype == torch.bfloat16:
        return COREY_BF16
    if t.dtype == torch.float16:
        return COREY_F16
    raise TypeError(f"unsupported storage type {t.dtype}")


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, name):
    if t is not None and (not t.is_cuda or not t.is_contiguous()):
        raise ValueError(f"{name} must be a contiguous GPU tensor")


def _want(t, name, dtype, shape):
    """Optional tensor `t` must have this dtype and shape (the library reads raw memory and cannot check either)."""
    if t is not None and (t.dtype != dtype or tuple(t.shape) != tuple(shape)):
        raise TypeError(f"{name} must be {dtype} of shape {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")


def policy_default() -> Policy:
    p = Policy()
    _check(lib().corey_policy_default(ctypes.byref(p)))
    return p


def corey_version() -> str:
    return lib().corey_version().decode()


def corey_entropy_hist_workspace(B: int, K: int) -> int:
    return int(lib().corey_entropy_hist_workspace(B, K))


def selective_state_update(state: torch.Tensor, x: torch.Tensor, delta: torch.Tensor, A: torch.Tensor, Bt: torch.Tensor,
                           Ct: torch.Tensor, Dv: torch.Tensor | None = None, z: torch.Tensor | None = None,
                           delta_bias: torch.Tensor | None = None, delta_softplus: bool = True, y: torch.Tensor | None = None):
    """One decode step: state float32 [B, D, N] is updated in place; x, delta, z [B, D]; Bt, Ct [B, N]; returns y [B, D]."""
    for name, t in (("state", state), ("x", x), ("delta", delta), ("A", A), ("Bt", Bt), ("Ct", Ct), ("Dv", Dv), ("z", z),
                    ("delta_bias", delta_bias), ("y", y)):
        _dev(t, name)
    B, D, N = state.shape
    if state.dtype != torch.float32 or A.dtype != torch.float32 or A.shape != (D, N):
        raise TypeError("state [B, D, N] and A [D, N] must be float32")
    for name, t, shape in (("x", x, (B, D)), ("delta", delta, (B, D)), ("z", z, (B, D)), ("Bt", Bt, (B, N)), ("Ct", Ct, (B, N))):
        if t is not None and (tuple(t.shape) != shape or t.dtype != x.dtype):
            raise TypeError(f"{name} must be {shape} in the dtype of x")
    for name, t in (("Dv", Dv), ("delta_bias", delta_bias)):
        if t is not None and (t.dtype != torch.float32 or tuple(t.shape) != (D,)):
            raise TypeError(f"{name} must be float32 [D]")
    if y is None:
        y = torch.empty_like(x)
    _check(lib().selective_state_update(_ptr(state), _ptr(x), _ptr(delta), _ptr(A), _ptr(Bt), _ptr(Ct), _ptr(Dv), _ptr(z),
                                        _ptr(delta_bias), 1 if delta_softplus else 0, _ptr(y), _dtype_code(x), B, D, N, _stream()))
    return y


HANDOFF_BYTES = 1024 * 16 + 16 * 4096 * 4      # COREY_HANDOFF_BYTES: partial ranges + partial histograms
RANGE_PARTS_BYTES = HANDOFF_BYTES
CHUNK_SLOTS = 12                   # COREY_CHUNK_SLOTS


def causal_conv1d_silu_fwd(x: torch.Tensor, weight: torch.Tensor, bias: torch.Tensor | None = None,
                           state_in: torch.Tensor | None = None, u: torch.Tensor | None = None, want_state: bool = False,
                           range_parts: torch.Tensor | None = None, pattern_table: torch.Tensor | None = None):
    """x [B, D, L] GPU tensor, weight float32 [D, W], bias float32 [D].  Returns (u, state_out or None, range_parts):
    range_parts (uint8 GPU tensor of HANDOFF_BYTES, allocated here if omitted) can be handed to
    corey_entropy_hist / corey_route_device on this u, which then skip their range sweep.  pattern_table: uint8 GPU
    tensor of corey_pattern_table_workspace() bytes; the kernel then also fills the bit-pattern table of u for
    corey_entropy_hist_from_table."""
    for name, t in (("x", x), ("weight", weight), ("bias", bias), ("state_in", state_in), ("u", u), ("range_parts", range_parts),
                    ("pattern_table", pattern_table)):
        _dev(t, name)
    B, D, L = x.shape
    W = weight.shape[1]
    if weight.shape[0] != D or weight.dtype != torch.float32 or (bias is not None and bias.dtype != torch.float32):
        raise TypeError("weight [D, W] and bias [D] must be float32")
    if u is None:
        u = torch.empty_like(x)
    state_out = torch.empty((B, D, W - 1), dtype=x.dtype, device=x.device) if want_state else None
    if range_parts is None:
        range_parts = torch.empty(HANDOFF_BYTES, dtype=torch.uint8, device=x.device)
    elif range_parts.numel() < HANDOFF_BYTES or range_parts.dtype != torch.uint8:
        raise TypeError(f"range_parts must be a uint8 tensor of {HANDOFF_BYTES} bytes")
    _check(lib().causal_conv1d_silu_fwd(_ptr(x), _ptr(weight), _ptr(bias), _ptr(state_in), _ptr(u), _ptr(state_out),
                                        _ptr(range_parts), _ptr(pattern_table), 0 if pattern_table is None else pattern_table.numel(),
                                        _dtype_code(x), B, D, L, W, _stream()))
    return u, state_out, range_parts


def corey_entropy_hist(x: torch.Tensor, K: int, eps: float = 1e-8, stride: int = 1, seqlens: torch.Tensor | None = None,
                       out: dict | None = None, workspace: torch.Tensor | None = None, block: int = 1,
                       range_parts: torch.Tensor | None = None):
    """x: [B, D, L] GPU tensor (float32 or bfloat16).  Returns dict(counts, H, r, range) of GPU tensors;
    nothing is copied to the host and the call does not synchronise."""
    _dev(x, "x"), _dev(seqlens, "seqlens")
    if x.dim() != 3:
        raise ValueError("x must be [B, D, L]")
    B, D, L = x.shape
    nh = B if seqlens is not None else 1
    _want(seqlens, "seqlens", torch.int32, (B,))
    if out is None:
        out = dict(counts=torch.empty((nh, K), dtype=torch.int32, device=x.device),   # uint32 bit patterns
                   H=torch.empty(nh, dtype=torch.float64, device=x.device),
                   r=torch.empty(nh, dtype=torch.float64, device=x.device),
                   range=torch.empty((nh, 2), dtype=torch.float32, device=x.device))
    need = corey_entropy_hist_workspace(B, K)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    _check(lib().corey_entropy_hist(_ptr(x), _dtype_code(x), B, D, L, _ptr(seqlens), K, eps, stride, block,
                                    _ptr(out["counts"]), _ptr(out["H"]), _ptr(out["r"]), _ptr(out.get("range")),
                                    _ptr(range_parts), _ptr(workspace), workspace.numel(), _stream()))
    out["workspace"] = workspace
    return out


def corey_pattern_table_workspace() -> int:
    return int(lib().corey_pattern_table_workspace())


def _table_out(K, device, policy, out):
    if out is None:
        out = dict(counts=torch.empty((1, K), dtype=torch.int32, device=device), H=torch.empty(1, dtype=torch.float64, device=device),
                   r=torch.empty(1, dtype=torch.float64, device=device), range=torch.empty((1, 2), dtype=torch.float32, device=device))
    if policy is not None and out.get("chunks") is None:
        out["chunks"] = torch.empty(1, dtype=torch.int32, device=device)
    return out


def corey_entropy_hist_onesweep(x: torch.Tensor, K: int, eps: float = 1e-8, policy: Policy | None = None, out: dict | None = None,
                                table_ws: torch.Tensor | None = None):
    """The statistic of a bfloat16 / float16 tensor from one pass over it (bit-pattern table).  Returns the dict of
    corey_entropy_hist (plus `chunks` when a policy is given, as corey_route_device) and `table_ws`."""
    _dev(x, "x"), _dev(table_ws, "table_ws")
    if x.dim() != 3:
        raise ValueError("x must be [B, D, L]")
    B, D, L = x.shape
    out = _table_out(K, x.device, policy, out)
    if table_ws is None:
        table_ws = torch.empty(corey_pattern_table_workspace(), dtype=torch.uint8, device=x.device)
    _check(lib().corey_entropy_hist_onesweep(_ptr(x), _dtype_code(x), B, D, L, K, eps, ctypes.byref(policy) if policy is not None else None,
                                             _ptr(out.get("chunks")) if policy is not None else None, _ptr(out["counts"]), _ptr(out["H"]),
                                             _ptr(out["r"]), _ptr(out.get("range")), _ptr(table_ws), table_ws.numel(), _stream()))
    out["table_ws"] = table_ws
    return out


def corey_entropy_hist_from_table(table_ws: torch.Tensor, dtype: torch.dtype, L: int, K: int, eps: float = 1e-8,
                                  policy: Policy | None = None, out: dict | None = None):
    """The statistic of the tensor whose producer (causal_conv1d_silu_fwd with pattern_table=table_ws) filled the table."""
    _dev(table_ws, "table_ws")
    out = _table_out(K, table_ws.device, policy, out)
    code = {torch.bfloat16: COREY_BF16, torch.float16: COREY_F16, torch.float32: COREY_F32}[dtype]
    _check(lib().corey_entropy_hist_from_table(code, L, K, eps, ctypes.byref(policy) if policy is not None else None,
                                               _ptr(out.get("chunks")) if policy is not None else None, _ptr(out["counts"]), _ptr(out["H"]),
                                               _ptr(out["r"]), _ptr(out.get("range")), _ptr(table_ws), table_ws.numel(), _stream()))
    return out


STATIC_SCRATCH_BYTES = 1 << 20     # COREY_STATIC_SCRATCH_BYTES


def corey_entropy_hist_static(x: torch.Tensor, K: int, out: dict, eps: float = 1e-8, stride: int = 1,
                              seqlens: torch.Tensor | None = None, block: int = 1, range_parts: torch.Tensor | None = None):
    """corey_entropy_hist on the library's built-in scratch buffer: nothing is allocated, here or in the library, so
    `out` (dict(counts, H, r[, range]) of GPU tensors, as corey_entropy_hist returns) must be given."""
    _dev(x, "x"), _dev(seqlens, "seqlens")
    if x.dim() != 3:
        raise ValueError("x must be [B, D, L]")
    B, D, L = x.shape
    nh = B if seqlens is not None else 1
    _want(seqlens, "seqlens", torch.int32, (B,))
    _want(out["counts"], "counts", torch.int32, (nh, K))
    _want(out["H"], "H", torch.float64, (nh,))
    _want(out["r"], "r", torch.float64, (nh,))
    _want(out.get("range"), "range", torch.float32, (nh, 2))
    _check(lib().corey_entropy_hist_static(_ptr(x), _dtype_code(x), B, D, L, _ptr(seqlens), K, eps, stride, block,
                                           _ptr(out["counts"]), _ptr(out["H"]), _ptr(out["r"]), _ptr(out.get("range")),
                                           _ptr(range_parts), _stream()))
    return out


def corey_ema_update(lam: float, state: float, H: float) -> float:
    """One step of the entropy EMA on the host; state = NaN means no estimate yet.  Returns the new state."""
    st = ctypes.c_double(state)
    _check(lib().corey_ema_update(float(lam), ctypes.byref(st), float(H)))
    return st.value


def corey_route_device(x: torch.Tensor, K: int, policy: Policy | None = None, eps: float = 1e-8, stride: int = 1, block: int = 1,
                       seqlens: torch.Tensor | None = None, out: dict | None = None, workspace: torch.Tensor | None = None,
                       ema_lambda: float = 0.0, ema_state: torch.Tensor | None = None, chunk_calls: torch.Tensor | None = None,
                       range_parts: torch.Tensor | None = None):
    """corey_entropy_hist and the chunk rule in one call.  Returns the dict of corey_entropy_hist plus `chunks`
    (int32 GPU tensor [nh], directly usable as `chunks_dev` of selective_scan_fwd); no synchronisation.
    ema_state: float64 GPU tensor [nh] (NaN = no estimate yet), updated in place; chunk_calls: int32 GPU tensor
    [COREY_CHUNK_SLOTS] of counters the caller clears."""
    _dev(ema_state, "ema_state"), _dev(chunk_calls, "chunk_calls")
    _dev(x, "x"), _dev(seqlens, "seqlens")
    if x.dim() != 3:
        raise ValueError("x must be [B, D, L]")
    B, D, L = x.shape
    nh = B if seqlens is not None else 1
    _want(seqlens, "seqlens", torch.int32, (B,))
    _want(ema_state, "ema_state", torch.float64, (nh,))
    _want(chunk_calls, "chunk_calls", torch.int32, (CHUNK_SLOTS,))
    p = policy if policy is not None else policy_default()
    if out is None:
        out = dict(counts=torch.empty((nh, K), dtype=torch.int32, device=x.device),
                   H=torch.empty(nh, dtype=torch.float64, device=x.device),
                   r=torch.empty(nh, dtype=torch.float64, device=x.device),
                   range=torch.empty((nh, 2), dtype=torch.float32, device=x.device),
                   chunks=torch.empty(nh, dtype=torch.int32, device=x.device))
    if workspace is None:
        workspace = out.get("workspace")
    if workspace is None:
        workspace = torch.empty(max(corey_entropy_hist_workspace(B, K), 256), dtype=torch.uint8, device=x.device)
    _check(lib().corey_route_device(_ptr(x), _dtype_code(x), B, D, L, _ptr(seqlens), K, eps, stride, block, ctypes.byref(p),
                                    float(ema_lambda), _ptr(ema_state), _ptr(chunk_calls), _ptr(out["counts"]), _ptr(out["H"]), _ptr(out["r"]), _ptr(out.get("range")),
                                    _ptr(range_parts), _ptr(out["chunks"]), _ptr(workspace), workspace.numel(), _stream()))
    out["workspace"] = workspace
    return out


def corey_route_device_deferred(x: torch.Tensor, K: int, policy: Policy | None = None, eps: float = 1e-8, stride: int = 1, block: int = 1,
                                seqlens: torch.Tensor | None = None, out: dict | None = None, workspace: torch.Tensor | None = None,
                                chunk_calls: torch.Tensor | None = None, range_parts: torch.Tensor | None = None):
    """The sweeps of corey_route_device without its reduction: returns the same dict (its tensors are written by the
    selective_scan_fwd_routed call that follows) with `route`, the ticket that call takes."""
    _dev(chunk_calls, "chunk_calls"), _dev(x, "x"), _dev(seqlens, "seqlens")
    if x.dim() != 3:
        raise ValueError("x must be [B, D, L]")
    B, D, L = x.shape
    nh = B if seqlens is not None else 1
    _want(seqlens, "seqlens", torch.int32, (B,))
    _want(chunk_calls, "chunk_calls", torch.int32, (CHUNK_SLOTS,))
    p = policy if policy is not None else policy_default()
    if out is None:
        out = dict(counts=torch.empty((nh, K), dtype=torch.int32, device=x.device),
                   H=torch.empty(nh, dtype=torch.float64, device=x.device),
                   r=torch.empty(nh, dtype=torch.float64, device=x.device),
                   range=torch.empty((nh, 2), dtype=torch.float32, device=x.device),
                   chunks=torch.empty(nh, dtype=torch.int32, device=x.device))
    if workspace is None:
        workspace = out.get("workspace")
    if workspace is None:
        workspace = torch.empty(max(corey_entropy_hist_workspace(B, K), 256), dtype=torch.uint8, device=x.device)
    route = out.get("route") or DeferredRoute()
    _check(lib().corey_route_device_deferred(_ptr(x), _dtype_code(x), B, D, L, _ptr(seqlens), K, eps, stride, block, ctypes.byref(p),
                                             _ptr(chunk_calls), _ptr(out["counts"]), _ptr(out["H"]), _ptr(out["r"]), _ptr(out.get("range")),
                                             _ptr(range_parts), _ptr(out["chunks"]), _ptr(workspace), workspace.numel(),
                                             ctypes.byref(route), _stream()))
    out["workspace"] = workspace
    out["route"] = route
    return out


def corey_select_chunk(r: float, L: int, policy: Policy | None = None) -> int:
    p = policy if policy is not None else policy_default()
    c = ctypes.c_int32(0)
    _check(lib().corey_select_chunk(float(r), int(L), ctypes.byref(p), ctypes.byref(c)))
    return c.value


def corey_select_chunk_device(r_dev: torch.Tensor, L: int, policy: Policy | None = None, seqlens: torch.Tensor | None = None,
                              out: torch.Tensor | None = None) -> torch.Tensor:
    """r_dev: float64 GPU tensor [nh].  Returns an int32 GPU tensor [nh] of chunks (no synchronisation)."""
    _dev(r_dev, "r_dev"), _dev(seqlens, "seqlens")
    if r_dev.dtype != torch.float64:
        raise TypeError("r_dev must be float64")
    p = policy if policy is not None else policy_default()
    nh = r_dev.numel()
    _want(seqlens, "seqlens", torch.int32, (nh,))
    if out is None:
        out = torch.empty(nh, dtype=torch.int32, device=r_dev.device)
    _check(lib().corey_select_chunk_device(_ptr(r_dev), _ptr(seqlens), int(L), nh, ctypes.byref(p), _ptr(out), _stream()))
    return out


def selective_scan_fwd_plan(B: int, D: int, N: int, chunk: int) -> int:
    return int(lib().selective_scan_fwd_plan(B, D, N, chunk))


def selective_scan_fwd_plan_steps(B: int, D: int, N: int, chunk: int) -> int:
    return int(lib().selective_scan_fwd_plan_steps(B, D, N, chunk))


def selective_scan_fwd_plan_split(B: int, D: int, N: int, chunk: int) -> int:
    return int(lib().selective_scan_fwd_plan_split(B, D, N, chunk))


def selective_scan_fwd_workspace(B: int, N: int, L: int) -> int:
    return int(lib().selective_scan_fwd_workspace(B, N, L))


COREY_SCAN_GENERAL_A = 1
COREY_SCAN_ONE_CHUNK = 2
COREY_SCAN_WHOLE_ROWS = 4


def selective_scan_fwd(u, delta, A, Bm, Cm, Dv=None, z=None, delta_bias=None, delta_softplus=True, h0=None,
                       seqlens=None, chunk: int = 512, chunks_dev=None, y=None, last_state=None, workspace=None,
                       general_a: bool = False, route: DeferredRoute | None = None, whole_rows: bool = False):
    """Tensors as in include/corey.h.  Returns (y, last_state); enqueues on torch's current stream.
    `workspace`: uint8 GPU tensor of selective_scan_fwd_workspace(B, N, L) bytes (allocated here if omitted).
    `general_a`: COREY_SCAN_GENERAL_A, i.e. never take the fast path for A[d, n] = (n + 1) A[d, 0].
    `chunks_dev` of one entry for a batch of several sequences is passed with COREY_SCAN_ONE_CHUNK.
    `whole_rows`: COREY_SCAN_WHOLE_ROWS, i.e. never share a channel's states between two rows of lanes.
    `route`: the ticket of corey_route_device_deferred; the call is then selective_scan_fwd_routed (no chunks_dev)."""
    for name, t in (("u", u), ("delta", delta), ("A", A), ("Bm", Bm), ("Cm", Cm), ("Dv", Dv), ("z", z),
                    ("delta_bias", delta_bias), ("h0", h0), ("seqlens", seqlens), ("chunks_dev", chunks_dev),
                    ("y", y), ("last_state", last_state), ("workspace", workspace)):
        _dev(t, name)
    if u.dim() != 3 or A.dim() != 2:
        raise ValueError("u must be [B, D, L] and A [D, N]")
    B, D, L = u.shape
    N = A.shape[1]
    if A.shape != (D, N) or Bm.shape != (B, N, L) or Cm.shape != (B, N, L) or delta.shape != u.shape:
        raise ValueError("inconsistent shapes")
    for name, t in (("delta", delta), ("z", z), ("y", y)):
        _want(t, name, u.dtype, (B, D, L))
    for name, t in (("Bm", Bm), ("Cm", Cm)):
        _want(t, name, u.dtype, (B, N, L))
    _want(A, "A", torch.float32, (D, N))
    for name, t in (("Dv", Dv), ("delta_bias", delta_bias)):
        _want(t, name, torch.float32, (D,))
    for name, t in (("h0", h0), ("last_state", last_state)):
        _want(t, name, torch.float32, (B, D, N))
    _want(seqlens, "seqlens", torch.int32, (B,))
    # a single routed chunk (the whole-tensor statistic of a batch) applies to every sequence
    one_chunk = chunks_dev is not None and B > 1 and tuple(chunks_dev.shape) == (1,)
    _want(chunks_dev, "chunks_dev", torch.int32, (1,) if one_chunk else (B,))
    if y is None:
        y = torch.empty_like(u)
    if last_state is None:
        last_state = torch.empty((B, D, N), dtype=torch.float32, device=u.device)
    if workspace is None:
        workspace = torch.empty(selective_scan_fwd_workspace(B, N, L), dtype=torch.uint8, device=u.device)
    flags = (COREY_SCAN_GENERAL_A if general_a else 0) | (COREY_SCAN_WHOLE_ROWS if whole_rows else 0)
    if route is not None:
        if chunks_dev is not None:
            raise ValueError("a route brings its own chunks")
        _check(lib().selective_scan_fwd_routed(_ptr(u), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm), _ptr(Dv), _ptr(z),
                                               _ptr(delta_bias), 1 if delta_softplus else 0, _ptr(h0), _ptr(seqlens), int(chunk),
                                               ctypes.byref(route), _ptr(y), _ptr(last_state), _dtype_code(u), B, D, N, L,
                                               flags, _ptr(workspace), workspace.numel(), _stream()))
        return y, last_state
    _check(lib().selective_scan_fwd(_ptr(u), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm), _ptr(Dv), _ptr(z),
                                    _ptr(delta_bias), 1 if delta_softplus else 0, _ptr(h0), _ptr(seqlens), int(chunk),
                                    _ptr(chunks_dev), _ptr(y), _ptr(last_state), _dtype_code(u), B, D, N, L,
                                    flags | (COREY_SCAN_ONE_CHUNK if one_chunk else 0), _ptr(workspace), workspace.numel(), _stream()))
    return y, last_state
