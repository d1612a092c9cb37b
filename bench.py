#!/usr/bin/env python3
"""Benchmark of the COREY hot path on one MI355X.

One step = one pass of the whole path over one batch that already sits in HBM: corey_route_device on u (the exact
full histogram, H, r and the chunk rule on the GPU), then selective_scan_fwd reading the routed chunk from device
memory (no host round trip inside a step).  Prints ONE JSON line.

  value      scan algorithmic bytes (u, delta, z in; y out; B, C, parameters, final state) per step time, GB/s
  roofline   for the dominant kernel (the scan): algorithmic bytes / its own launch duration, measured with
             events on the launch stream inside the timed region, against the 8 TB/s HBM peak; the `alu` block
             beside it prices the same launches against the fp32 vector peak, which is the bound that binds
  ceilings   a plain device copy of the same bytes on this machine, and the time the scan's own instruction count needs
             at one plain wave64 instruction per 4 cycles and one transcendental per 8 on each SIMD
  per_chunk  scan-only latency, GB/s and tokens/s for every chunk of the sweep
  producer   the causal convolution + SiLU that writes u and its range, and the statistic with and without that range
             (two sweeps, one sweep, one sweep over every 8th block), each also as a percentage of the scan
  decode     one generated token (selective_state_update), eager calls and replayed from a HIP graph
  paper_shape  the scan on the paper's kernel-benchmark shape (a small layer) per chunk, with two rows of lanes per channel where
             the launch plan gives them and with one row per channel (COREY_SCAN_WHOLE_ROWS)
  graph_replay  the same step replayed from a HIP graph (no faster than the eager launches here: the step is GPU-bound)
  overhead   entropy + routing cost relative to the scan alone at the routed chunk, for the exact statistic (the
             timed step) and for the sampled one (every 8th block of 512 values, the paper's stride-8 variant at
             cache-line granularity), and with the chunk rule on the host instead
  pipeline   whole steps of the layer's routed path, producer included (conv -> statistic and rule -> scan), against
             conv -> scan at the same chunk: exact and sampled statistic on the producer's range, with the reduction as a
             launch of its own and deferred into the scan's first kernel; this is where the <= 2 % goal is judged
  policies   which chunk each scheduler variant (entropy rule, guarded rule, sequence-length table) picks from the exact
             and from the sampled statistic, the distance of Eq. 2's argument from its nearest switch point, and the whole
             step each costs
  one_sweep  the bit-pattern-table statistic (one pass over u, or none when the producer filled the table)
  structured_A  the same scan with the library's fast path for A[d, n] = (n + 1) A[d, 0] left on (the benchmark
             layers have that A; trained weights in general do not, so every other figure here is measured with the
             fast path switched off, i.e. one exponential per (channel, state, step))
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload on this host's cores (and on one core),
             with the CPU model
  parity     this run's own outputs against what the oracle computed in that leg: histogram counts and routed chunk
             equal (when the sample was the whole workload), worst error of y and of the final state over the
             tolerance the parity tests use (below 1 passes)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X fp32 vector, published (256 CUs x 2.4 GHz x 256 flop/clk)
# HBM bytes per scan launch measured with `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE`, scaled by what the same counters
# read for a 256 MiB device copy (profiles/hot_path_c4_mamba2p8b_counters.txt); not re-measured by this script
MEASURED_TRAFFIC_BYTES = {"c4_mamba2p8b": 749_400_000}
TRAFFIC_FROM = "profiles/hot_path_c4_mamba2p8b_counters.txt"
# vector instructions per wave-level state update of the scan at the routed chunk, from SQ_INSTS_VALU and
# SQ_INSTS_VALU_TRANS_F32 of the same counter summary
COUNTED_INSTRUCTIONS = {"c4_mamba2p8b": {"plain": 7.42, "trans": 1.325, "from": "profiles/hot_path_c4_mamba2p8b_counters.txt"}}


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--ramp-seconds", type=float, default=1.0,
                    help="untimed: the whole step is repeated for this long before the warm-up steps, because the chip takes "
                         "some tens of milliseconds of this ALU-heavy load to settle its clocks (the first launches of a "
                         "process run up to a third slower than the steady state)")
    ap.add_argument("--config", default="c4_mamba2p8b")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 256 MiB device-to-device copy a few times: a dispatch of known traffic against which "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (rows are independent and would shard "
              "over channels); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2604_10597_amd as corey
    from paper_2604_10597_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    cfg = wl.CONFIGS[args.config]
    w = wl.make(cfg)

    def dev(a):
        if a is None:
            return None
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()          # float32 and float16 upload as they are

    d = {k: dev(v) for k, v in w.dev.items()}
    seqlens = None if w.seqlens is None else torch.from_numpy(w.seqlens).cuda()
    tokens = int(w.seqlens.sum()) if w.seqlens is not None else cfg.B * cfg.L
    scan_bytes = wl.scan_bytes(cfg)
    state_updates = cfg.D * cfg.N * tokens
    # algorithmic flops per state update: 2 mul + 2 fma (6 flop) + 1 exp counted as one
    scan_flop = 7.0 * state_updates

    scan_ws = torch.empty(corey.selective_scan_fwd_workspace(cfg.B, cfg.N, cfg.L), dtype=torch.uint8, device="cuda")
    y = torch.empty_like(d["u"])
    last = torch.empty((cfg.B, cfg.D, cfg.N), dtype=torch.float32, device="cuda")
    ent = corey.corey_entropy_hist(d["u"], cfg.K, seqlens=seqlens)
    pol = corey.policy_default()
    r_pinned = torch.empty(ent["r"].shape, dtype=torch.float64).pin_memory()

    # every headline figure is measured on the general path (COREY_SCAN_GENERAL_A): the benchmark layers' A = -(n + 1) would
    # otherwise take the library's power-chain path, which trained weights in general cannot
    def scan(chunk, general_a=True):
        corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"],
                                 delta_bias=d["delta_bias"], seqlens=seqlens, chunk=chunk, y=y, last_state=last, workspace=scan_ws,
                                 general_a=general_a)

    ent["chunks"] = torch.empty(ent["r"].numel(), dtype=torch.int32, device="cuda")
    chunks_dev = ent["chunks"]
    # the host's chunk is only the launch-shape hint of the device-routed scan: the chunk this workload routes to
    hint = max(corey.corey_select_chunk(float(v), int(n), pol) for v, n in
               zip(ent["r"].cpu().tolist(), (w.seqlens if w.seqlens is not None else [cfg.L] * ent["r"].numel())))

    def scan_routed(stride=1, block=1):
        """The whole path with no host round trip: statistic and chunk rule on the GPU -> scan that reads the chunk."""
        corey.corey_route_device(d["u"], cfg.K, pol, seqlens=seqlens, out=ent, stride=stride, block=block)
        corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"],
                                 delta_bias=d["delta_bias"], seqlens=seqlens, chunk=hint, chunks_dev=chunks_dev,
                                 y=y, last_state=last, workspace=scan_ws, general_a=True)

    def route_on_host():
        corey.corey_entropy_hist(d["u"], cfg.K, seqlens=seqlens, out=ent, workspace=ent["workspace"])
        r_pinned.copy_(ent["r"], non_blocking=True)
        torch.cuda.current_stream().synchronize()              # the host needs r to pick the launch shape
        Ls = w.seqlens if w.seqlens is not None else [cfg.L] * r_pinned.numel()
        return max(corey.corey_select_chunk(float(r_pinned[i]), int(Ls[i]), pol) for i in range(r_pinned.numel()))

    if args.calibrate_copy:
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- the timed region: K whole steps
    ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ev1 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < args.ramp_seconds:
        for _ in range(20):
            scan_routed()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        scan_routed()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        corey.corey_route_device(d["u"], cfg.K, pol, seqlens=seqlens, out=ent)
        ev0[i].record()
        corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"],
                                 delta_bias=d["delta_bias"], seqlens=seqlens, chunk=hint, chunks_dev=chunks_dev,
                                 y=y, last_state=last, workspace=scan_ws, general_a=True)
        ev1[i].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / args.steps
    scan_ms = float(np.mean([a.elapsed_time(b) for a, b in zip(ev0, ev1)]))
    chunk = int(chunks_dev.max().item())

    # the same step with the sampled statistic (every 8th block of 512 values: 1/8 of the bytes of u)
    def time_steps(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0s = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0s) * 1e3 / args.steps

    ms_step_sampled = time_steps(lambda: scan_routed(8, 512))
    r_sampled = [round(float(v), 6) for v in ent["r"].cpu().tolist()]
    chunk_sampled = int(chunks_dev.max().item())

    # the same step replayed from a HIP graph (ten steps per graph): what a serving loop pays once the launches are recorded
    torch.cuda.synchronize()
    step_graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(step_graph):
        for _ in range(10):
            scan_routed()
    step_graph.replay()
    torch.cuda.synchronize()
    t0g = time.perf_counter()
    for _ in range(max(1, args.steps // 10)):
        step_graph.replay()
    torch.cuda.synchronize()
    ms_step_graph = (time.perf_counter() - t0g) * 1e3 / (max(1, args.steps // 10) * 10)
    chunk_graph = int(chunks_dev.max().item())

    # the same step with the chunk rule on the host (one 8-byte read of r and a synchronisation per step)
    for _ in range(2):
        scan(route_on_host())
    torch.cuda.synchronize()
    t0h = time.perf_counter()
    for i in range(args.steps):
        scan(route_on_host())
    torch.cuda.synchronize()
    ms_step_host = (time.perf_counter() - t0h) * 1e3 / args.steps

    def time_scan(c, warm, reps, general_a=True):
        for _ in range(warm):
            scan(c, general_a)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            scan(c, general_a)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    # ---- scan alone at the routed chunk (for the overhead figure) and the chunk sweep
    scan_alone_ms = time_scan(chunk, 3, args.steps)
    # the sampled statistic can route to another chunk: its overhead is taken against the scan at that chunk
    scan_alone_sampled_ms = scan_alone_ms if chunk_sampled == chunk else time_scan(chunk_sampled, 3, args.steps)
    hist_a, hist_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    hist_a.record()
    for _ in range(args.steps):
        corey.corey_entropy_hist(d["u"], cfg.K, seqlens=seqlens, out=ent, workspace=ent["workspace"])
    hist_b.record()
    torch.cuda.synchronize()
    hist_ms = hist_a.elapsed_time(hist_b) / args.steps
    hist_a.record()
    for _ in range(args.steps):
        corey.corey_entropy_hist(d["u"], cfg.K, seqlens=seqlens, out=ent, workspace=ent["workspace"], stride=8, block=512)
    hist_b.record()
    torch.cuda.synchronize()
    hist_sampled_ms = hist_a.elapsed_time(hist_b) / args.steps
    per_chunk = {}
    if not args.no_sweep:
        for c in cfg.chunks:
            ms = time_scan(c, 2, 10)
            per_chunk[str(c)] = {"ms": round(ms, 4), "GBps": round(scan_bytes / ms * 1e-6, 1),
                                 "tokens_per_s": round(tokens / ms * 1e3, 1),
                                 "hbm_frac": round(scan_bytes / ms * 1e-6 / HBM_PEAK_GBPS, 4)}

    # ---- the structured-A fast path, reported separately
    structured = {"note": "A[d,n] = (n+1) A[d,0] detected on the GPU: exp(dl A[d,n]) formed as exp(dl A[d,0])^(n+1)",
                  "scan_ms": {}, "GBps": {}}
    for c in (sorted({chunk, 1024}) if args.no_sweep else cfg.chunks):
        ms = time_scan(c, 2, 10, general_a=False)
        structured["scan_ms"][str(c)] = round(ms, 4)
        structured["GBps"][str(c)] = round(scan_bytes / ms * 1e-6, 1)
    structured["hbm_frac_at_routed_chunk"] = round(structured["GBps"][str(chunk)] / HBM_PEAK_GBPS, 4)

    # ---- ceilings beside the HBM peak: what a plain device copy reaches on this machine, and the time the scan's own
    # instruction stream needs when every SIMD issues without a gap (counts per wave-level state update from the
    # committed counter summary; a SIMD issues one plain wave64 fp32 instruction per 4 cycles and one transcendental per
    # 8 -- packed fp32 instructions are not used -- as the same counters and register-only probes show)
    src = torch.empty(scan_bytes // 2, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    ca, cb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ca.record()
    for _ in range(20):
        dst.copy_(src)
    cb.record()
    torch.cuda.synchronize()
    copy_ms = ca.elapsed_time(cb) / 20
    del src, dst
    wave_updates = state_updates / 64.0
    counted = COUNTED_INSTRUCTIONS.get(cfg.name)
    ceilings = {"device_copy_GBps": round(scan_bytes / copy_ms * 1e-6, 1), "device_copy_ms_for_scan_bytes": round(copy_ms, 4),
                "floor_cycles_per_wave_update": 28.0,
                "floor_note": "the two-pass recurrence needs 5 plain vector instructions (4 cycles each on a SIMD) and one "
                              "exponential (8 cycles) per wave-level state update: 28 SIMD cycles"}
    if counted:
        issue_cycles = wave_updates / 1024.0 * (counted["plain"] * 4.0 + counted["trans"] * 8.0)          # per SIMD (256 CUs x 4)
        ceilings.update({"counted_plain_per_wave_update": counted["plain"], "counted_transcendental_per_wave_update": counted["trans"],
                         "counted_cycles_per_wave_update": round(counted["plain"] * 4.0 + counted["trans"] * 8.0, 2),
                         "counted_from": counted["from"],
                         "issue_model_ms_at_2p4GHz": round(issue_cycles / 2.4e9 * 1e3, 4)})

    # ---- the producer of u (causal convolution + SiLU) with the range of u taken in the same pass: the statistic then
    # needs one sweep over u instead of two
    cv = wl.make_conv(cfg, 4)
    xc, wc, bc = dev(cv["dev"]["x"]), dev(cv["dev"]["weight"]), dev(cv["dev"]["bias"])
    uc = torch.empty_like(xc)
    _, _, parts = corey.causal_conv1d_silu_fwd(xc, wc, bc, u=uc)

    def time_kernel(fn, reps):
        # a short untimed run first: after the ALU-bound scan the chip takes some milliseconds to settle on a bandwidth-bound
        # kernel's clocks (the first launches measured up to 15 % slower)
        t_r = time.perf_counter()
        while time.perf_counter() - t_r < 0.2:
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    conv_ms = time_kernel(lambda: corey.causal_conv1d_silu_fwd(xc, wc, bc, u=uc, range_parts=parts), args.steps)
    entc = corey.corey_route_device(uc, cfg.K, pol)
    hist2_ms = time_kernel(lambda: corey.corey_route_device(uc, cfg.K, pol, out=entc), args.steps)
    hist1_ms = time_kernel(lambda: corey.corey_route_device(uc, cfg.K, pol, out=entc, range_parts=parts), args.steps)
    hist18_ms = time_kernel(lambda: corey.corey_route_device(uc, cfg.K, pol, out=entc, range_parts=parts, stride=8, block=512), args.steps)
    conv_bytes = wl.conv_bytes(cfg)
    producer = {"note": "causal depthwise convolution (4 taps) + SiLU writing u and the partial ranges of u; "
                        "corey_route_device given those ranges skips its range sweep (whole-tensor statistic)",
                "conv_ms": round(conv_ms, 4), "conv_GBps": round(conv_bytes / conv_ms * 1e-6, 1),
                "conv_hbm_frac": round(conv_bytes / conv_ms * 1e-6 / HBM_PEAK_GBPS, 4),
                "route_two_sweeps_ms": round(hist2_ms, 4), "route_given_range_ms": round(hist1_ms, 4),
                "route_given_range_sampled_stride8_block512_ms": round(hist18_ms, 4),
                "pct_of_scan": {"two_sweeps": round(hist2_ms / scan_alone_ms * 100, 2),
                                "given_range": round(hist1_ms / scan_alone_ms * 100, 2),
                                "given_range_sampled": round(hist18_ms / scan_alone_ms * 100, 2)}}
    # ---- whole steps of the layer's routed path with the producer in front: conv -> [statistic, rule] -> scan
    # (the host's chunk of a device-routed launch only shapes the grid: the chunk this u routed to last time)
    hint_u = max(16, int(entc["chunks"].max().item())) if seqlens is None else hint

    def scan_u(chunk=None, chunks=None, route=None):
        corey.selective_scan_fwd(uc, d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"], delta_bias=d["delta_bias"],
                                 chunk=chunk or hint_u, chunks_dev=chunks, route=route, y=y, last_state=last, workspace=scan_ws, general_a=True)

    def conv_only():
        corey.causal_conv1d_silu_fwd(xc, wc, bc, u=uc, range_parts=parts)

    pipeline, policies, one_sweep = None, None, None
    if seqlens is None:
        entd = corey.corey_route_device_deferred(uc, cfg.K, pol, range_parts=parts)

        def step_static(chunk):
            conv_only()
            scan_u(chunk=chunk)

        def step_routed(stride, block, deferred, policy, hint_c):
            conv_only()
            if deferred:
                corey.corey_route_device_deferred(uc, cfg.K, policy, out=entd, range_parts=parts, stride=stride, block=block)
                scan_u(chunk=hint_c, route=entd["route"])
            else:
                corey.corey_route_device(uc, cfg.K, policy, out=entc, range_parts=parts, stride=stride, block=block)
                scan_u(chunk=hint_c, chunks=entc["chunks"])

        def routed_entry(stride, block, deferred, policy=pol):
            step_routed(stride, block, deferred, policy, hint_u)       # untimed: which chunk this variant routes to = its launch hint
            c = int((entd if deferred else entc)["chunks"].max().item())
            ms = time_steps(lambda: step_routed(stride, block, deferred, policy, c))
            base = static_ms.get(c)
            if base is None:
                base = static_ms[c] = time_steps(lambda: step_static(c))
            return {"ms_per_step": round(ms, 4), "chunk": c, "conv_plus_scan_ms_at_that_chunk": round(base, 4),
                    "overhead_pct": round((ms - base) / base * 100, 2), "overhead_us": round((ms - base) * 1e3, 1)}

        static_ms = {}
        pipeline = {"note": "one step = causal_conv1d_silu_fwd (writes u, its partial ranges and cleared partial histograms) -> "
                            "corey_route_device on that range -> selective_scan_fwd at the device-routed chunk; overhead against "
                            "conv -> scan at the chunk the variant routes to (general path, same buffers)",
                    "exact": routed_entry(1, 1, False), "exact_deferred_reduction": routed_entry(1, 1, True),
                    "sampled_stride8_block512": routed_entry(8, 512, False),
                    "sampled_stride8_block512_deferred_reduction": routed_entry(8, 512, True)}
        pipeline["conv_plus_scan_ms"] = {str(c): round(v, 4) for c, v in sorted(static_ms.items())}

        # ---- scheduler variants on the exact and on the sampled statistic: chunk, distance from the nearest switch point of
        # Eq. 2 (in log2 units of the rule's argument; 0.5 is the middle of a bucket), whole step
        import math

        def margin_of(r, policy):
            v = policy.c_min + min(max(r * policy.h_ref_scale, 0.0), 1.0) * (policy.c_max - policy.c_min)
            lg = math.log2(v)
            return round(abs(lg - (math.floor(lg) + 0.5)), 4)

        policies = {"note": "mode 0 = Eq. 2, mode 4 = guarded Eq. 2 (fallback to 512 unless two buckets away), mode 2 = sequence-length "
                            "table; statistic on the producer's range, reduction deferred into the scan"}
        for label, (stride, block) in (("exact", (1, 1)), ("sampled_stride8_block512", (8, 512))):
            for mode in (0, 4, 2):
                pm = corey.policy_default()
                pm.mode = mode
                e = routed_entry(stride, block, True, pm)
                r_now = float(entd["r"][0].item())
                e["r"] = round(r_now, 6)
                e["margin_log2"] = margin_of(r_now, pm) if mode in (0, 4) else None
                policies[f"{label}_mode{mode}"] = e
        # the same on the benchmark workload's own u (statistic on its own range, reduction deferred): here the exact and the
        # sampled r can fall on different sides of a switch point of Eq. 2
        entw = corey.corey_route_device_deferred(d["u"], cfg.K, pol)

        def step_workload(stride, block, policy, hint_c):
            corey.corey_route_device_deferred(d["u"], cfg.K, policy, out=entw, stride=stride, block=block)
            corey.selective_scan_fwd(d["u"], d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"], delta_bias=d["delta_bias"],
                                     chunk=hint_c, route=entw["route"], y=y, last_state=last, workspace=scan_ws, general_a=True)

        on_u = {}
        for label, (stride, block) in (("exact", (1, 1)), ("sampled_stride8_block512", (8, 512))):
            for mode in (0, 4):
                pm = corey.policy_default()
                pm.mode = mode
                step_workload(stride, block, pm, hint)
                c = int(entw["chunks"].max().item())
                r_now = float(entw["r"][0].item())
                ms = time_steps(lambda: step_workload(stride, block, pm, c))
                on_u[f"{label}_mode{mode}"] = {"ms_per_step": round(ms, 4), "chunk": c, "r": round(r_now, 6), "margin_log2": margin_of(r_now, pm)}
        policies["on_the_workloads_u"] = on_u
        policies["recommended"] = ("mode 4 (guarded) with the sampled statistic: it keeps the safe chunk unless the prediction is two "
                                   "buckets away, so a statistic that lands on the other side of a switch point cannot pick the slower "
                                   "neighbour; see the entries above for this workload")

        # ---- the bit-pattern-table statistic (16-bit storage): one pass over u, or none when the producer filled the table
        if cfg.dtype != "f32":
            tws = torch.empty(corey.corey_pattern_table_workspace(), dtype=torch.uint8, device="cuda")
            tout = corey.corey_entropy_hist_onesweep(uc, cfg.K, policy=pol, table_ws=tws)
            one_ms = time_kernel(lambda: corey.corey_entropy_hist_onesweep(uc, cfg.K, policy=pol, out=tout, table_ws=tws), args.steps)
            conv_t_ms = time_kernel(lambda: corey.causal_conv1d_silu_fwd(xc, wc, bc, u=uc, range_parts=parts, pattern_table=tws), args.steps)
            tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float16
            from_ms = time_kernel(lambda: corey.corey_entropy_hist_from_table(tws, tdt, cfg.L, cfg.K, policy=pol, out=tout), args.steps)
            one_sweep = {"note": "exact statistic from the table of the 65536 bit patterns: one pass over u (against two sweeps), or "
                                 "none when the producer fills the table (against producer + one count sweep)",
                         "one_sweep_ms": round(one_ms, 4), "two_sweeps_ms": round(hist2_ms, 4),
                         "conv_filling_table_ms": round(conv_t_ms, 4), "from_table_ms": round(from_ms, 4),
                         "conv_table_plus_statistic_ms": round(conv_t_ms + from_ms, 4),
                         "conv_plus_count_sweep_ms": round(conv_ms + hist1_ms, 4),
                         "counts_equal_two_sweeps": bool(torch.equal(tout["counts"], corey.corey_entropy_hist(uc, cfg.K)["counts"]))}
            del tws
    del xc, uc

    # ---- one generated token from the carried state (the recurrence at L = 1), single sequence and batches of 64 and 512
    # (back-to-back launches from Python: the small cases show the launch rate, about 12 us per call, not the kernel)
    decode = {"note": "selective_state_update on the benchmark's layer shape; bytes = state read + written, A, per-row scalars"}
    for Bd in (1, 64, 512):
        dc = wl.scaled(cfg, B=Bd, L=1, seqlens=None)
        dd = {k: dev(v) for k, v in wl.make_decode(dc)["dev"].items()}
        yd = torch.empty_like(dd["x"])
        ms = time_kernel(lambda: corey.selective_state_update(dd["state"], dd["x"], dd["delta"], dd["A"], dd["Bt"], dd["Ct"], Dv=dd["D"],
                                                              z=dd["z"], delta_bias=dd["delta_bias"], y=yd), args.steps)
        # the same step from a HIP graph of 32 launches (what a serving loop would replay): the kernel, not the call rate
        def one_token():
            corey.selective_state_update(dd["state"], dd["x"], dd["delta"], dd["A"], dd["Bt"], dd["Ct"], Dv=dd["D"], z=dd["z"],
                                         delta_bias=dd["delta_bias"], y=yd)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(32):
                one_token()
        ms_g = time_kernel(graph.replay, 20) / 32
        # with the convolution's own single step in front (its carried window in, u_t and the new window out)
        xt = dd["x"].unsqueeze(2).contiguous()
        ut = torch.empty_like(xt)
        cw, cb = torch.rand(cfg.D, 4, device="cuda") - 0.5, torch.rand(cfg.D, device="cuda") - 0.5
        win = [torch.zeros((Bd, cfg.D, 3), dtype=xt.dtype, device="cuda") for _ in range(2)]
        cparts = torch.empty(corey.binding.HANDOFF_BYTES, dtype=torch.uint8, device="cuda")
        lib, ptr = corey.binding.lib(), corey.binding._ptr

        def layer_token(i):
            corey.binding._check(lib.causal_conv1d_silu_fwd(ptr(xt), ptr(cw), ptr(cb), ptr(win[i & 1]), ptr(ut), ptr(win[(i & 1) ^ 1]),
                                                             ptr(cparts), None, 0, corey.binding._dtype_code(xt), Bd, cfg.D, 1, 4,
                                                             corey.binding._stream()))
            corey.selective_state_update(dd["state"], ut.view(Bd, cfg.D), dd["delta"], dd["A"], dd["Bt"], dd["Ct"], Dv=dd["D"],
                                         z=dd["z"], delta_bias=dd["delta_bias"], y=yd)
        layer_token(0)
        torch.cuda.synchronize()
        graph2 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph2):
            for i in range(32):
                layer_token(i)
        ms_g2 = time_kernel(graph2.replay, 20) / 32
        del graph2
        decode[f"B{Bd}"] = {"us_per_token_step_eager_calls": round(ms * 1e3, 2), "us_per_token_step_graph": round(ms_g * 1e3, 2),
                            "us_per_token_conv_plus_state_graph": round(ms_g2 * 1e3, 2),
                            "GBps": round(wl.decode_bytes(dc) / ms_g * 1e-6, 1),
                            "hbm_frac": round(wl.decode_bytes(dc) / ms_g * 1e-6 / HBM_PEAK_GBPS, 4)}
        del graph, dd, yd

    # ---- the paper's own kernel-benchmark shape (batch 1, d 1024, L 4096, d_state 16, FP16), for context only
    paper_shape = None
    if not args.no_sweep:
        pc = wl.CONFIGS["paper_w1_fp16"]
        pw = wl.make(pc)
        pd = {k: dev(v) for k, v in pw.dev.items()}
        p_ws = torch.empty(corey.selective_scan_fwd_workspace(pc.B, pc.N, pc.L), dtype=torch.uint8, device="cuda")
        p_y, p_last = torch.empty_like(pd["u"]), torch.empty((pc.B, pc.D, pc.N), dtype=torch.float32, device="cuda")
        p_ent = corey.corey_entropy_hist(pd["u"], pc.K)
        p_chunk = corey.corey_select_chunk(p_ent["r"].item(), pc.L, pol)

        def p_scan(c, whole_rows=False):
            corey.selective_scan_fwd(pd["u"], pd["delta"], pd["A"], pd["B"], pd["C"], Dv=pd["D"], z=pd["z"],
                                     delta_bias=pd["delta_bias"], chunk=c, y=p_y, last_state=p_last, workspace=p_ws, general_a=True,
                                     whole_rows=whole_rows)

        def p_time(c, whole_rows=False):
            for _ in range(5):
                p_scan(c, whole_rows)
            a0, b0 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a0.record()
            for _ in range(30):
                p_scan(c, whole_rows)
            b0.record()
            torch.cuda.synchronize()
            return a0.elapsed_time(b0) / 30

        paper_shape = {"workload": "B1 D1024 N16 L4096 fp16 (the paper's kernel-level benchmark shape), 5 warm-up + 30 timed",
                       "r": round(p_ent["r"].item(), 4), "routed_chunk": p_chunk,
                       "scan_ms": {str(c): round(p_time(c), 4) for c in (64, 256, 512, 1024, 2048)},
                       "scan_ms_one_row_per_channel": {str(c): round(p_time(c, True), 4) for c in (64, 256, 512, 1024)},
                       "two_rows_per_channel": {str(c): bool(corey.selective_scan_fwd_plan_split(pc.B, pc.D, pc.N, c)) for c in (64, 256, 512, 1024, 2048)},
                       "note": "a launch this small gives every channel two rows of lanes with half of the states each (up to chunk "
                               "1024); scan_ms_one_row_per_channel is the same launch under COREY_SCAN_WHOLE_ROWS",
                       "scan_bytes": wl.scan_bytes(pc)}
        del pd, pw, p_ws, p_y

    # ---- CPU oracle on a bounded sample of the same workload (reported baseline, not a target)
    cpu = None
    if not args.no_cpu:
        import oracle
        cores = min(16, len(os.sched_getaffinity(0)))

        def oracle_pass(nrows, threads=None):
            threads = threads or cores
            sel = np.linspace(0, cfg.D - 1, nrows).astype(np.int64)
            p3 = lambda a: np.ascontiguousarray(a[:, sel, :])
            t = time.perf_counter()
            h = oracle.entropy_hist(p3(w.val["u"]), cfg.K, seqlens=w.seqlens)
            Ls = w.seqlens if w.seqlens is not None else [cfg.L]
            c = max(oracle.select_chunk(float(h["r"][i]), int(Ls[i]), oracle.policy())[1] for i in range(len(h["r"])))
            _, y_ref, s_ref = oracle.selective_scan(p3(w.val["u"]), p3(w.val["delta"]), w.val["A"][sel], w.val["B"], w.val["C"],
                                                    Dv=w.val["D"][sel], z=p3(w.val["z"]), delta_bias=w.val["delta_bias"][sel],
                                                    seqlens=w.seqlens, chunk=c, threads=threads)
            oracle_pass.last = (sel, h, c, y_ref, s_ref)
            return time.perf_counter() - t

        probe_rows = min(cfg.D, 2 * cores)
        t_single = oracle_pass(probe_rows, threads=1)             # the same sample on one core
        t_probe = oracle_pass(probe_rows)
        nrows = int(min(cfg.D, max(probe_rows, probe_rows * args.cpu_seconds / max(t_probe, 1e-3))))
        t_cpu = oracle_pass(nrows)
        frac = nrows / cfg.D
        cpu = {"value": round(scan_bytes * frac / t_cpu * 1e-9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
               "tokens_per_s": round(tokens * frac / t_cpu, 1), "seconds": round(t_cpu, 2),
               "sample": f"{nrows} of {cfg.D} channels of {cfg.name} (all {tokens} tokens), histogram + chunk rule + scan, "
                         f"double precision, OpenMP over channels",
               "single_thread": {"value": round(scan_bytes * probe_rows / cfg.D / t_single * 1e-9, 4), "unit": "GB/s",
                                 "tokens_per_s": round(tokens * probe_rows / cfg.D / t_single, 1),
                                 "sample": f"{probe_rows} of {cfg.D} channels"},
               "cpu_model": cpu_model()}

    # ---- parity of this very run against what the oracle just computed (the tests hold the full checks)
    parity = None
    if cpu is not None:
        sel, h_ref, c_ref, y_ref, s_ref = oracle_pass.last
        scan_routed()                                         # general path, exact statistic, device-routed chunk
        torch.cuda.synchronize()
        idx = torch.from_numpy(sel).cuda()
        yg = y[:, idx, :].float().cpu().numpy().astype(np.float64)
        sg = last[:, idx, :].cpu().numpy().astype(np.float64)
        store = {"f32": 0.0, "bf16": 2.0 ** -8, "f16": 2.0 ** -11}[cfg.dtype]
        rt = 1e-5 * max(1.0, (cfg.L / 256.0) ** 0.5)
        yb = (3e-3 if cfg.dtype != "f32" else rt) * (np.abs(y_ref) + np.sqrt((y_ref ** 2).mean(-1, keepdims=True))) + store * np.abs(y_ref) + 1e-30
        sb = rt * (np.abs(s_ref) + np.sqrt((s_ref ** 2).mean(-1, keepdims=True))) + 1e-30
        y_stated = (3e-3 if cfg.dtype != "f32" else 1e-5) * (np.abs(y_ref) + np.sqrt((y_ref ** 2).mean(-1, keepdims=True))) + 1e-30
        y_tight = rt * (np.abs(y_ref) + np.sqrt((y_ref ** 2).mean(-1, keepdims=True))) + store * np.abs(y_ref) + 1e-30
        s_stated = 1e-5 * (np.abs(s_ref) + np.sqrt((s_ref ** 2).mean(-1, keepdims=True))) + 1e-30
        parity = {"channels_checked": int(len(sel)),
                  "y_worst_error_over_stated_bound_no_store_allowance": round(float((np.abs(yg - y_ref) / y_stated).max()), 3),
                  "y_worst_error_over_fp32_computation_bound_plus_store": round(float((np.abs(yg - y_ref) / y_tight).max()), 3),
                  "state_worst_error_over_1e-5": round(float((np.abs(sg - s_ref) / s_stated).max()), 3),
                  "bounds": "stated: 3e-3 (16-bit) / 1e-5 (fp32) x (|ref| + rms of the row); the tests grant the 16-bit store's half ulp on "
                            "top and let the fp32 bound grow with sqrt(L / 256); all three ratios are reported",
                  "counts_equal": bool(np.array_equal(ent["counts"].cpu().numpy().view(np.uint32).reshape(h_ref["counts"].shape),
                                                      h_ref["counts"])) if len(sel) == cfg.D else None,
                  "chunk_equal": bool(int(chunks_dev.max().item()) == c_ref) if len(sel) == cfg.D else None,
                  "y_worst_error_over_tolerance": round(float((np.abs(yg - y_ref) / yb).max()), 3),
                  "state_worst_error_over_tolerance": round(float((np.abs(sg - s_ref) / sb).max()), 3)}

    gbps = scan_bytes / scan_ms * 1e-6
    out = {
        "metric": "selective_scan_hbm_GBps", "value": round(scan_bytes / ms_step * 1e-6, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "storage_dtype": cfg.dtype,
        "data": "synthetic",
        "targets": {"scan_hbm_frac_goal": 0.70, "scan_hbm_frac": round(gbps / HBM_PEAK_GBPS, 4), "scan_goal_met": bool(gbps / HBM_PEAK_GBPS >= 0.70),
                    "routing_overhead_goal_pct": 2.0,
                    "routing_overhead_pct_best_whole_step": (None if pipeline is None else
                                                             min(v["overhead_pct"] for k, v in pipeline.items() if isinstance(v, dict) and "overhead_pct" in v)),
                    "note": "the scan is bound by vector-instruction issue, not by HBM (see alu, ceilings): the 70 % goal is not met; "
                            "routing overhead is judged on whole steps in `pipeline`"},
        "config": {"workload": f"{cfg.name}: B{cfg.B} D{cfg.D} N{cfg.N} L{cfg.L}, {cfg.dtype} storage, fp32 state, "
                               f"u {cfg.u_kind}, K={cfg.K}, routed chunk {chunk}",
                   "scan_bytes": scan_bytes, "tokens": tokens},
        "tokens_per_s": round(tokens / ms_step * 1e3, 1),
        "routed_chunk": chunk, "r": [round(float(v), 6) for v in r_pinned],
        "roofline": {"bound": "hbm", "binding_resource": "vector-instruction issue (alu); the HBM figure is the benchmark's metric",
                     "kernel": "k_scan_any (selective_scan_fwd, device-routed chunk; the launch also holds k_relayout_bc, ~6 us)", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name), "traffic_from": TRAFFIC_FROM if cfg.name in MEASURED_TRAFFIC_BYTES else None,
                     "avg_launch_ms": round(scan_ms, 4)},
        "alu": {"achieved": round(scan_flop / scan_ms * 1e-9, 2), "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(scan_flop / scan_ms * 1e-9 / FP32_VECTOR_PEAK_TFLOPS, 4),
                "peak_plain_instructions": FP32_VECTOR_PEAK_TFLOPS / 2,      # 16 lanes per SIMD and cycle: packed fp32 is not used
                "frac_plain_instructions": round(scan_flop / scan_ms * 1e-9 / (FP32_VECTOR_PEAK_TFLOPS / 2), 4),
                "simd_cycles_per_wave_update_if_2p4GHz": round(scan_ms * 1e-3 * 2.4e9 * 1024.0 / wave_updates, 2),
                "cycles_note": "launch time x 2.4 GHz x 1024 SIMDs / wave-level state updates: an upper bound on the cycles a SIMD spends "
                               "per update (the chip holds 2.1 to 2.3 GHz under this load); floor of the formulation: 28",
                "flop_per_state_update": 7, "state_updates": state_updates},
        "graph_replay": {"ms_per_step": round(ms_step_graph, 4), "GBps": round(scan_bytes / ms_step_graph * 1e-6, 1),
                         "routed_chunk": chunk_graph,
                         "note": "the timed step (exact statistic + rule + device-routed scan) replayed from a HIP graph of ten steps"},
        "overhead": {"entropy_routing_pct_of_scan": round((ms_step - scan_alone_ms) / scan_alone_ms * 100, 2),
                     "host_routed_ms_per_step": round(ms_step_host, 4),
                     "host_routed_pct_of_scan": round((ms_step_host - scan_alone_ms) / scan_alone_ms * 100, 2),
                     "hist_kernels_ms": round(hist_ms, 4), "scan_alone_ms": round(scan_alone_ms, 4),
                     "hist_pct_of_scan": round(hist_ms / scan_alone_ms * 100, 2),
                     "sampled_stride8_block512": {"ms_per_step": round(ms_step_sampled, 4),
                                                  "entropy_routing_pct_of_scan": round((ms_step_sampled - scan_alone_sampled_ms) / scan_alone_sampled_ms * 100, 2),
                                                  "scan_alone_ms_at_its_chunk": round(scan_alone_sampled_ms, 4),
                                                  "hist_kernels_ms": round(hist_sampled_ms, 4), "r": r_sampled,
                                                  "routed_chunk": chunk_sampled}},
        "ceilings": ceilings,
        "per_chunk": per_chunk,
        "structured_A": structured,
        "producer": producer,
        "pipeline": pipeline,
        "policies": policies,
        "one_sweep": one_sweep,
        "decode": decode,
        "paper_shape": paper_shape,
        "cpu_baseline": cpu,
        "parity": parity,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
