"""GPU parity on seeded random combinations of everything the scan and the statistic accept: shapes from one value to a
few thousand per axis, every chunk, padded batches (including empty sequences), initial state, gate, softplus on and
off, both decay paths, host and device chunk, whole-tensor / per-sequence / sampled statistics.  Each case is checked
against the oracle element by element."""
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
