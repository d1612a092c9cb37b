"""GPU parity on seeded random combinations of everything the scan and the statistic accept: shapes from one value to a
few thousand per axis, every chunk, padded batches (including empty sequences), initial state, gate, softplus on and
off, both decay paths, host and device chunk, whole-tensor / per-sequence / sampled statistics.  Each case is checked
against the oracle element by element.  Also: the producer of u with every form of the statistic behind it, and the
routed scan with the reduction deferred, separate, and launched from the host's chunk."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
import paper_2604_10597_amd as corey
from gpu_util import assert_close, fp32_rtol, store_bits, upload, y_rtol, y_to_f64
from paper_2604_10597_amd import workloads as wl

pytestmark = pytest.mark.gpu
NAMES = ["c0_tiny_f32", "c1_mamba130m", "c2_mamba370m", "c4_mamba2p8b", "paper_w1_fp16"]


def _close(got, ref, rtol, what, bits, terms=None):
    # rows of a few elements (N = 1, L = 1) have no row scale of their own: take the scale of the whole sequence
    if ref.shape[-1] < 8:
        flat = lambda a: None if a is None else a.reshape(ref.shape[0], 1, -1)
        return assert_close(flat(got), flat(ref), rtol, what, bits, flat(terms))
    return assert_close(got, ref, rtol, what, bits, terms)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_combinations(seed):
    rng = np.random.default_rng(seed)
    for case in range(40):
        base = wl.CONFIGS[NAMES[rng.integers(len(NAMES))]]
        B = int(rng.choice([1, 1, 2, 3, 5]))
        D = int(rng.choice([1, 2, 7, 16, 33, 64, 100, 257, 600, 1300]))
        N = int(rng.choice([1, 2, 4, 5, 8, 16, 16, 16, 24, 64]))
        L = int(rng.choice([1, 3, 8, 16, 31, 64, 100, 256, 257, 512, 777, 1024, 1500, 2048, 2050, 3000]))
        if B * D * L * N > 3e7:
            D = max(1, int(3e7 / (B * L * N)))
        chunk = int(rng.choice([16, 32, 64, 128, 256, 512, 1024, 2048]))
        seqlens = tuple(int(rng.integers(0, L + 1)) for _ in range(B)) if rng.random() < 0.4 else None
        cfg = dataclasses.replace(wl.scaled(base, B=B, D=D, N=N, L=L), seqlens=seqlens, seed=int(rng.integers(1 << 30)))
        a_kind = "mamba" if rng.random() < 0.4 else "random"
        with_h0, use_z, softplus = bool(rng.random() < 0.5), bool(rng.random() < 0.7), bool(rng.random() < 0.8)
        routed, struct = bool(rng.random() < 0.4), bool(rng.random() < 0.5)
        whole_rows = bool(rng.random() < 0.35)             # small launches split a channel's states over two rows unless told not to
        print(f"[case] seed {seed} #{case}: {cfg.dtype} B{B} D{D} N{N} L{L} chunk {chunk} seqlens {seqlens} A={a_kind} h0={with_h0} "
              f"z={use_z} softplus={softplus} routed={routed} structured={struct} whole_rows={whole_rows}", flush=True)
        w = wl.make(cfg, a_kind=a_kind, with_h0=with_h0)
        d, v = upload(w), w.val
        st, y_ref, s_ref, y_terms = oracle.selective_scan(
            v["u"], v["delta"] if softplus else np.abs(v["delta"]), v["A"], v["B"], v["C"], Dv=v["D"], z=v["z"] if use_z else None,
            delta_bias=v["delta_bias"] if softplus else None, delta_softplus=softplus, h0=v.get("h0") if with_h0 else None,
            seqlens=w.seqlens, chunk=64, threads=8, want_terms=True)
        assert st == oracle.OK
        chunks_dev, host_chunk = None, chunk
        if routed:
            chunks_dev = torch.full((B,), chunk, dtype=torch.int32, device="cuda")
            host_chunk = int(rng.choice([64, 512, 2048]))
        y, last = corey.selective_scan_fwd(
            d["u"], d["delta"] if softplus else d["delta"].abs(), d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"] if use_z else None,
            delta_bias=d["delta_bias"] if softplus else None, delta_softplus=softplus, h0=d.get("h0") if with_h0 else None,
            seqlens=d["seqlens"], chunk=host_chunk, chunks_dev=chunks_dev, general_a=not struct, whole_rows=whole_rows)
        torch.cuda.synchronize()
        # random lengths include sequences of one or two steps, whose rows have no scale of their own: the bound also takes
        # the size of the terms y is summed from (gpu_util.assert_close)
        _close(y_to_f64(y), y_ref, y_rtol(cfg), "y", store_bits(cfg), y_terms)
        _close(last.cpu().numpy().astype(np.float64), s_ref, fp32_rtol(cfg.L), "state", False)
        K = int(rng.choice([2, 16, 64, 256, 1000]))
        stride, block = (1, 1) if rng.random() < 0.5 else (int(rng.choice([2, 3, 8])), int(rng.choice([1, 8, 64, 512, 100])))
        got = corey.corey_entropy_hist(d["u"], K, seqlens=d["seqlens"], stride=stride, block=block)
        ref = oracle.entropy_hist(v["u"], K, seqlens=w.seqlens, stride=stride, block=block)
        torch.cuda.synchronize()
        assert np.array_equal(got["counts"].cpu().numpy().view(np.uint32).reshape(ref["counts"].shape), ref["counts"]), (K, stride, block)


@pytest.mark.parametrize("seed", [21, 22, 23])
def test_random_producer_and_every_statistic(seed):
    """Random shapes, tap counts and storage types through the producer of u, then every form of the statistic on that u
    (two sweeps, the producer's range, sampled on that range, the built-in scratch, one sweep over the bit-pattern table, the
    table filled by the producer) against the oracle's histogram of the same bits: counts bit for bit, H, the routed chunk."""
    import math

    import test_gpu_conv as tc
    import test_gpu_table as tt
    from gpu_util import counts_u32, to_dev
    tws = tt._ws()
    rng = np.random.default_rng(seed)
    for case in range(12):
        dtype = [wl.BF16, wl.F16, wl.F32][int(rng.integers(3))]
        B, D = int(rng.choice([1, 1, 2, 3])), int(rng.choice([1, 3, 17, 64, 200, 700]))
        L = int(rng.choice([1, 5, 64, 333, 1024, 2049, 4104, 8192, 20000]))
        if B * D * L > 6e6:
            D = max(1, int(6e6 / (B * L)))
        W, K = int(rng.integers(1, 5)), int(rng.choice([2, 16, 256, 1000, 4096]))
        with_state, bias = bool(rng.random() < 0.5), bool(rng.random() < 0.8)
        stride, block = int(rng.choice([2, 8, 5])), int(rng.choice([8, 64, 512, 4096, 24, 1]))
        print(f"[case] seed {seed} #{case}: {dtype} B{B} D{D} L{L} W{W} K{K} state={with_state} bias={bias} stride={stride} "
              f"block={block}", flush=True)
        cfg = wl.Config(name="rnd", B=B, D=D, N=16, L=L, dtype=dtype, K=K, chunks=(64,), seed=int(rng.integers(1 << 30)))
        u, parts, xd, wd, bd = tc._run(cfg, W, with_state=with_state, bias=bias)      # the producer against the oracle
        uv = u.float().cpu().numpy()
        ref = oracle.entropy_hist(uv, K)
        ref_s = oracle.entropy_hist(uv, K, stride=stride, block=block, range_all=True)
        pol = corey.policy_default()
        given = corey.corey_route_device(u, K, pol, range_parts=parts)
        two = corey.corey_route_device(u, K, pol)
        sampled = corey.corey_route_device(u, K, pol, range_parts=parts, stride=stride, block=block)
        static = corey.corey_entropy_hist(u, K)
        static["counts"].zero_()
        corey.corey_entropy_hist_static(u, K, static)
        again = corey.corey_route_device(u, K, pol, range_parts=parts)     # the hand-over buffer came back cleared
        torch.cuda.synchronize()
        for what, out, r in (("given range", given, ref), ("two sweeps", two, ref), ("sampled", sampled, ref_s),
                             ("static", static, ref), ("given range again", again, ref)):
            assert np.array_equal(counts_u32(out["counts"]).reshape(-1), r["counts"].reshape(-1)), what
            if not math.isnan(r["H"][0]):
                assert out["H"].item() == pytest.approx(r["H"][0], rel=1e-12, abs=1e-14), what
                st, c_ref, margin = oracle.select_chunk(float(r["r"][0]), L, oracle.policy())
                assert "chunks" not in out or margin < 1e-9 or out["chunks"].item() == c_ref, what
        if dtype == wl.F32:
            continue
        one = corey.corey_entropy_hist_onesweep(u, K, policy=pol, table_ws=tws)
        torch.cuda.synchronize()
        tt._compare(one, ref, K)
        conv = wl.make_conv(cfg, W, with_state=with_state)
        u2 = torch.empty_like(u)
        corey.causal_conv1d_silu_fwd(xd, wd, bd, to_dev(conv["dev"]["state_in"], dtype), u=u2, range_parts=parts, pattern_table=tws)
        from_table = corey.corey_entropy_hist_from_table(tws, u.dtype, L, K, policy=pol)
        torch.cuda.synchronize()
        if L > 16:                                                     # (shorter rows take the single-step kernel without a table)
            assert torch.equal(u2.view(torch.int16), u.view(torch.int16))
        tt._compare(from_table, oracle.entropy_hist(u2.float().cpu().numpy(), K), K)


@pytest.mark.parametrize("seed", [31, 32, 33])
def test_random_routing_deferred_separate_and_host_chunk(seed):
    """Random layers, policies, statistics and launch options: the statistic's reduction and the rule inside the scan's
    first kernel against the separate reduction, and against the scan launched with the routed chunk from the host, every
    output bit for bit, twice in a row on the same buffers."""
    from gpu_util import to_dev
    rng = np.random.default_rng(seed)
    for case in range(10):
        dtype = [wl.BF16, wl.F16, wl.F32][int(rng.integers(3))]
        B, D = int(rng.choice([1, 1, 2, 3])), int(rng.choice([1, 8, 33, 100, 300, 1200]))
        L, N = int(rng.choice([1, 16, 100, 512, 1024, 1500, 2048, 4100])), int(rng.choice([1, 4, 16, 16, 24, 64]))
        if B * D * L * N > 4e7:
            D = max(1, int(4e7 / (B * L * N)))
        K, mode = int(rng.choice([2, 16, 256, 1000])), int(rng.choice([0, 0, 2, 4]))
        per_seq = bool(rng.random() < 0.3) and B > 1
        use_conv = (not per_seq) and bool(rng.random() < 0.5)
        kw = dict(stride=8, block=int(rng.choice([8, 64, 512]))) if rng.random() < 0.5 else {}
        general_a, whole_rows = bool(rng.random() < 0.5), bool(rng.random() < 0.3)
        lens = tuple(int(rng.integers(0, L + 1)) for _ in range(B)) if per_seq else None
        print(f"[case] seed {seed} #{case}: {dtype} B{B} D{D} N{N} L{L} K{K} mode {mode} lens {lens} conv={use_conv} {kw} "
              f"general_a={general_a} whole_rows={whole_rows}", flush=True)
        cfg = dataclasses.replace(wl.scaled(wl.CONFIGS["c2_mamba370m"], B=B, D=D, N=N, L=L, dtype=dtype), seqlens=lens,
                                  seed=int(rng.integers(1 << 30)))
        w = wl.make(cfg, a_kind="mamba" if rng.random() < 0.5 else "random")
        d = upload(w)
        pol = corey.policy_default()
        pol.mode = 1 if per_seq and mode == 0 else mode
        u, parts = d["u"], None
        if use_conv:
            conv = wl.make_conv(cfg, 4)
            u, _, parts = corey.causal_conv1d_silu_fwd(to_dev(conv["dev"]["x"], dtype), torch.from_numpy(conv["dev"]["weight"]).cuda(),
                                                       torch.from_numpy(conv["dev"]["bias"]).cuda())
        stat_lens = d["seqlens"] if per_seq else None
        hint = int(rng.choice([64, 512, 2048]))
        scan = lambda **more: corey.selective_scan_fwd(u, d["delta"], d["A"], d["B"], d["C"], Dv=d["D"], z=d["z"], delta_bias=d["delta_bias"],
                                                       seqlens=d["seqlens"], general_a=general_a, whole_rows=whole_rows, **more)
        for rep in range(2):
            a = corey.corey_route_device(u, K, pol, seqlens=stat_lens, range_parts=parts, **kw)
            ya, sa = scan(chunk=hint, chunks_dev=a["chunks"])
            b = corey.corey_route_device_deferred(u, K, pol, seqlens=stat_lens, range_parts=parts, **kw)
            yb, sb = scan(chunk=hint, route=b["route"])
            torch.cuda.synchronize()
            for k in ("counts", "chunks", "range"):
                assert torch.equal(a[k], b[k]), (k, rep)
            for k in ("H", "r"):
                assert torch.equal(a[k].view(torch.int64), b[k].view(torch.int64)), (k, rep)
            assert torch.equal(ya.view(torch.uint8), yb.view(torch.uint8)) and torch.equal(sa, sb), rep
            chunks = a["chunks"].cpu().tolist()
            if len(set(chunks)) == 1:
                yc, sc = scan(chunk=chunks[0])
                torch.cuda.synchronize()
                assert torch.equal(ya.view(torch.uint8), yc.view(torch.uint8)) and torch.equal(sa, sc), "host chunk"
