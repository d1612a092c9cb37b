"""Pins for the oracle's histogram entropy (Eq. 1 and r = H / log K).

Each test checks the oracle against something other than itself: values the paper prints
(tests/golden/entropy_table_pins.txt), closed forms, brute force, or numpy's histogram routine on data
where rounding cannot move a sample across a bin edge.
"""
import math

import numpy as np
import pytest

import oracle
from conftest import read_golden


def _x(a):
    a = np.asarray(a, dtype=np.float32)
    return a.reshape(1, 1, -1)


def test_one_sample_per_bin_and_top_edge_closed():
    res = oracle.entropy_hist(_x(np.arange(16)), 16)
    assert res["status"] == oracle.OK
    assert res["counts"][0].tolist() == [1] * 16          # x = hi lands in bin K-1, not K
    assert res["lo"][0] == 0.0 and res["hi"][0] == 15.0


def test_hand_counted_bins():
    # range [0, 8], K = 4, width 2: bins [0,2) [2,4) [4,6) [6,8]
    x = [0.0, 1.9, 2.0, 3.5, 4.0, 4.0, 5.99, 6.0, 7.0, 8.0, 0.1]
    res = oracle.entropy_hist(_x(x), 4, eps=0.0)
    assert res["counts"][0].tolist() == [3, 2, 3, 3]
    p = np.array([3, 2, 3, 3]) / 11.0
    # entropy of (3,2,3,3)/11 written out: 3 * (3/11) ln(11/3) + (2/11) ln(11/2)
    expect = 3 * (3 / 11) * math.log(11 / 3) + (2 / 11) * math.log(11 / 2)
    assert res["H"][0] == pytest.approx(expect, rel=1e-14)
    assert res["r"][0] == pytest.approx(expect / math.log(4), rel=1e-14)
    assert p.sum() == pytest.approx(1.0)


def test_empty_bins_add_nothing_also_without_eps():
    # counts (3, 0, 0, 1): H = -(3/4 ln 3/4 + 1/4 ln 1/4) = 0.5623351446...; the two empty bins are 0 log 0 = 0, so
    # eps = 0 gives the same finite value as a vanishing eps (and not 0 * -inf = NaN)
    expect = 0.75 * math.log(4 / 3) + 0.25 * math.log(4)
    assert expect == pytest.approx(0.5623351446188083, rel=1e-15)
    res0 = oracle.entropy_hist(_x([0, 0, 0, 10]), 4, eps=0.0)
    assert res0["status"] == oracle.OK and res0["counts"][0].tolist() == [3, 0, 0, 1]
    assert res0["H"][0] == pytest.approx(expect, rel=1e-15)
    assert res0["r"][0] == pytest.approx(expect / math.log(4), rel=1e-15)
    res = oracle.entropy_hist(_x([0, 0, 0, 10]), 4, eps=1e-300)
    assert res["H"][0] == pytest.approx(expect, rel=1e-15)
    # with eps > 0 the value is that of the populated bins alone
    res8 = oracle.entropy_hist(_x([0, 0, 0, 10]), 4, eps=1e-8)
    assert res8["H"][0] == pytest.approx(-(0.75 * math.log(0.75 + 1e-8) + 0.25 * math.log(0.25 + 1e-8)), rel=1e-15)


def test_eps_sits_inside_the_log_only():
    # counts (1, 3): p = (.25, .75); eps = 0.5: H = -(.25 ln .75 + .75 ln 1.25) = -0.0954371...
    res = oracle.entropy_hist(_x([0, 1, 1, 1]), 2, eps=0.5)
    assert res["counts"][0].tolist() == [1, 3]
    assert res["H"][0] == pytest.approx(0.071920518 - 0.167357663, abs=1e-8)
    assert res["r"][0] == 0.0                                   # negative H clamps to 0


@pytest.mark.parametrize("K,printed", [(32, 3.466), (64, 4.159), (128, 4.852), (256, 5.545), (512, 6.238)])
def test_uniform_counts_give_log_K(K, printed):
    # K distinct values, each m times: exactly uniform counts, so H = log K up to the eps term (-K*eps)
    x = np.repeat(np.arange(K), 7)
    eps = 1e-8
    res = oracle.entropy_hist(_x(x), K, eps=eps)
    assert (res["counts"][0] == 7).all()
    assert res["H"][0] == pytest.approx(math.log(K) - K * eps, abs=1e-10)
    assert abs(res["H"][0] - printed) < 6e-4                    # the paper's 3-decimal value
    assert res["r"][0] == pytest.approx(1.0, abs=1e-5)
    res0 = oracle.entropy_hist(_x(x), K, eps=0.0)
    assert res0["H"][0] == pytest.approx(math.log(K), rel=1e-14)
    assert res0["r"][0] <= 1.0


def test_against_numpy_histogram_away_from_edges():
    # samples sit in the middle half of their bins, so no rounding convention can move them
    rng = np.random.default_rng(5)
    K, w = 37, 0.25
    k = rng.integers(0, K, size=20000)
    x = (k + rng.uniform(0.25, 0.75, size=k.size)) * w
    x = np.concatenate([x, [0.0, K * w]])                       # pin the range to [0, K*w]
    res = oracle.entropy_hist(_x(x), K, eps=0.0)
    ref, _ = np.histogram(x.astype(np.float32).astype(np.float64), bins=K, range=(0.0, K * w))
    assert res["counts"][0].tolist() == ref.tolist()
    p = ref[ref > 0] / ref.sum()
    assert res["H"][0] == pytest.approx(float(-(p * np.log(p)).sum()), rel=1e-12)


def test_counts_sum_permutation_and_power_of_two_scaling():
    rng = np.random.default_rng(11)
    x = rng.standard_normal(50000).astype(np.float32)
    a = oracle.entropy_hist(_x(x), 256)
    assert int(a["counts"].sum()) == x.size
    b = oracle.entropy_hist(_x(rng.permutation(x)), 256)
    assert (a["counts"] == b["counts"]).all() and a["H"][0] == pytest.approx(b["H"][0], rel=1e-15)
    c = oracle.entropy_hist(_x(x * np.float32(8.0)), 256)      # exact in binary32
    assert (a["counts"] == c["counts"]).all()
    d = oracle.entropy_hist(_x(-x), 256)                        # mirror: counts reverse up to edge ties
    assert abs(int(d["counts"][0][::-1].astype(np.int64).sum()) - x.size) == 0


def test_bounds_hold():
    rng = np.random.default_rng(3)
    for K in (2, 3, 16, 100, 256, 1024):
        for gen in (rng.standard_normal, rng.random, lambda n: rng.laplace(0, 3, n)):
            res = oracle.entropy_hist(_x(gen(4096)), K, eps=1e-8)
            assert 0.0 <= res["r"][0] <= 1.0
            assert res["H"][0] <= math.log(K) + 1e-12


def test_degenerate_range_and_non_finite():
    res = oracle.entropy_hist(_x([2.5] * 9), 8, eps=1e-8)
    assert res["status"] == oracle.OK
    assert res["counts"][0].tolist() == [9, 0, 0, 0, 0, 0, 0, 0]
    assert res["H"][0] == pytest.approx(-math.log1p(1e-8), abs=1e-15) and res["r"][0] == 0.0
    for bad in (np.nan, np.inf, -np.inf):
        res = oracle.entropy_hist(_x([0.0, 1.0, bad, 2.0]), 8)
        assert res["status"] == oracle.ENONFINITE
        assert math.isnan(res["H"][0]) and math.isnan(res["r"][0]) and res["counts"].sum() == 0


def test_layout_seqlens_and_stride():
    rng = np.random.default_rng(8)
    B, D, L = 3, 5, 17
    x = rng.standard_normal((B, D, L)).astype(np.float32)
    whole = oracle.entropy_hist(x, 16)
    flat = oracle.entropy_hist(x.reshape(1, 1, -1), 16)
    assert (whole["counts"] == flat["counts"]).all()
    lens = np.array([17, 4, 9], dtype=np.int32)
    per = oracle.entropy_hist(x, 16, seqlens=lens)
    for b in range(B):
        one = oracle.entropy_hist(np.ascontiguousarray(x[b:b + 1, :, :lens[b]]), 16)
        assert (per["counts"][b] == one["counts"][0]).all()
        assert per["H"][b] == one["H"][0] and per["lo"][b] == one["lo"][0]
    # stride: every 8th element of the flattened tensor (the paper's sampled variant)
    s = oracle.entropy_hist(x, 16, stride=8)
    sub = oracle.entropy_hist(x.reshape(-1)[::8].reshape(1, 1, -1), 16)
    assert (s["counts"] == sub["counts"]).all() and s["H"][0] == sub["H"][0]
    # stride with seqlens numbers only the valid elements of that sequence
    ps = oracle.entropy_hist(x, 16, seqlens=lens, stride=3)
    for b in range(B):
        v = x[b, :, :lens[b]].reshape(-1)[::3]
        one = oracle.entropy_hist(v.reshape(1, 1, -1), 16)
        assert (ps["counts"][b] == one["counts"][0]).all()
    # blocks: every stride-th run of `block` consecutive elements of the flattened tensor (ragged last run kept)
    flat_x = x.reshape(-1)
    for stride, block in ((2, 5), (3, 4), (8, 1), (4, 16), (2, 1000)):
        keep = (np.arange(flat_x.size) // block) % stride == 0
        s = oracle.entropy_hist(x, 16, stride=stride, block=block)
        sub = oracle.entropy_hist(flat_x[keep].reshape(1, 1, -1), 16)
        assert (s["counts"] == sub["counts"]).all() and s["H"][0] == sub["H"][0] and s["counts"].sum() == keep.sum()
    pb = oracle.entropy_hist(x, 16, seqlens=lens, stride=2, block=3)
    for b in range(B):
        v = x[b, :, :lens[b]].reshape(-1)
        v = v[(np.arange(v.size) // 3) % 2 == 0]
        one = oracle.entropy_hist(v.reshape(1, 1, -1), 16)
        assert (pb["counts"][b] == one["counts"][0]).all()
    assert oracle.entropy_hist(x, 16, block=0)["status"] == oracle.EINVAL


def _draw(kind, n, rng):
    if kind == "normal":
        return rng.standard_normal(n, dtype=np.float32)
    if kind == "uniform":
        return rng.random(n, dtype=np.float32)
    if kind == "laplace1":
        return rng.laplace(0.0, 1.0, n).astype(np.float32)
    if kind.startswith("sparse"):
        f = {"sparse10": 0.10, "sparse2": 0.02}[kind]
        x = rng.standard_normal(n, dtype=np.float32)
        x[rng.random(n) >= f] = 0.0
        return x
    raise ValueError(kind)


_DIFF_ENTROPY = {"normal": 0.5 * math.log(2 * math.pi * math.e), "laplace1": 1.0 + math.log(2.0)}


@pytest.mark.parametrize("row", read_golden("entropy_table_pins.txt"), ids=lambda r: "-".join(r[:3]))
def test_values_printed_in_the_paper(row):
    kind, n, K, H_paper, r_paper, tol = row[0], int(row[1]), int(row[2]), float(row[3]), row[4], float(row[5])
    rng = np.random.default_rng(20260410 + K)
    x = _draw(kind, n, rng)
    if n == 4194304:
        x = x.astype(np.float16).astype(np.float32)             # that sweep ran on half-precision tensors
    res = oracle.entropy_hist(_x(x), K, eps=1e-8)
    H = res["H"][0]
    assert abs(H - H_paper) < tol, (H, H_paper)
    if r_paper != "-":
        assert abs(res["r"][0] - float(r_paper)) < tol / math.log(K) + 6e-4
    if kind in _DIFF_ENTROPY and K >= 128:
        # fine-bin limit: H ~ differential entropy - log(bin width)
        width = (float(res["hi"][0]) - float(res["lo"][0])) / K
        assert abs(H - (_DIFF_ENTROPY[kind] - math.log(width))) < 0.02
    if kind.startswith("sparse"):
        f = {"sparse10": 0.10, "sparse2": 0.02}[kind]
        width = (float(res["hi"][0]) - float(res["lo"][0])) / K
        mix = -(1 - f) * math.log(1 - f) - f * math.log(f) + f * (_DIFF_ENTROPY["normal"] - math.log(width))
        assert abs(H - mix) < 0.02


@pytest.mark.parametrize("K,H_paper,r_paper", [(32, 2.644, 0.763), (64, 3.334, 0.802), (128, 4.027, 0.830),
                                               (256, 4.720, 0.851), (512, 5.413, 0.868), (1024, 6.106, 0.881)])
def test_normal_table_with_the_range_its_values_imply(K, H_paper, r_paper):
    # The six printed values differ by exactly log 2 per doubling of K, i.e. they share one sample range;
    # the K = 1024 entry gives it: 6.106 = 1.4189 - log(R / 1024)  =>  R = 9.43.  A standard-normal sample
    # confined to that range must then reproduce every entry to the printed precision.
    R = 1024.0 * math.exp(_DIFF_ENTROPY["normal"] - 6.106)
    assert abs(R - 9.43) < 0.01
    rng = np.random.default_rng(1)
    x = rng.standard_normal(1_000_000, dtype=np.float32)
    x = x[np.abs(x) < R / 2]
    x = np.concatenate([x, np.array([-R / 2, R / 2], dtype=np.float32)])
    res = oracle.entropy_hist(_x(x), K, eps=1e-8)
    assert abs(res["H"][0] - H_paper) < 0.004
    assert abs(res["r"][0] - r_paper) < 0.0012


def test_doubling_K_adds_log_two_for_smooth_densities():
    rng = np.random.default_rng(77)
    x = _x(rng.standard_normal(1_000_000, dtype=np.float32))
    H = [oracle.entropy_hist(x, K)["H"][0] for K in (64, 128, 256, 512)]
    for a, b in zip(H, H[1:]):
        assert abs((b - a) - math.log(2.0)) < 0.01


def test_sampled_counts_on_the_range_of_all_values():
    """range_all: bins bounded by the extremes of every value, counts over the sampled blocks only."""
    rng = np.random.default_rng(21)
    K, w = 29, 0.5
    # numpy's histogram with an explicit range, on samples in the middle half of their bins
    k = rng.integers(3, K - 3, size=6000)
    x = ((k + rng.uniform(0.25, 0.75, size=k.size)) * w).astype(np.float32)
    x[5] = 0.0                                                  # the extremes sit in blocks that are NOT sampled
    x[6] = K * w
    stride, block = 4, 4
    j = np.arange(x.size)
    used = (j // block) % stride == 0
    assert not used[5] and not used[6]
    res = oracle.entropy_hist(_x(x), K, eps=1e-8, stride=stride, block=block, range_all=True)
    ref, _ = np.histogram(x[used].astype(np.float64), bins=K, range=(0.0, K * w))
    assert res["counts"][0].tolist() == ref.tolist() and res["counts"].sum() == used.sum()
    assert res["lo"][0] == 0.0 and res["hi"][0] == np.float32(K * w)
    p = ref / ref.sum()                                         # the end bins are empty: 0 log(eps) = 0
    assert res["H"][0] == pytest.approx(float(-(p * np.log(p + 1e-8)).sum()), rel=1e-12)
    # the plain sampled statistic takes the narrower range of the sampled values: different bins
    plain = oracle.entropy_hist(_x(x), K, eps=0.0, stride=stride, block=block)
    assert plain["lo"][0] > 0.0 and plain["counts"][0].tolist() != ref.tolist()
    # same thing as appending the two extremes to the sample and taking them out of their (end) bins again
    ext = np.concatenate([x[used], [0.0, K * w]]).astype(np.float32)
    e = oracle.entropy_hist(_x(ext), K, eps=0.0)["counts"][0].astype(np.int64)
    e[0] -= 1
    e[K - 1] -= 1
    assert e.tolist() == ref.tolist()
    # stride 1: both readings coincide; extremes inside sampled blocks: both readings coincide
    y = rng.standard_normal((2, 3, 50)).astype(np.float32)
    a, b = oracle.entropy_hist(y, 16), oracle.entropy_hist(y, 16, range_all=True)
    assert (a["counts"] == b["counts"]).all() and a["H"][0] == b["H"][0]
    y.reshape(-1)[0], y.reshape(-1)[1] = -9.0, 9.0
    a, b = oracle.entropy_hist(y, 16, stride=5, block=2), oracle.entropy_hist(y, 16, stride=5, block=2, range_all=True)
    assert (a["counts"] == b["counts"]).all() and a["lo"][0] == b["lo"][0] == -9.0
    # a NaN outside the sample still makes the statistic non-finite; per-sequence histograms number their own values
    z = y.copy()
    z.reshape(-1)[3] = np.nan                                   # block 1 of stride 5: not sampled
    assert oracle.entropy_hist(z, 16, stride=5, block=2)["status"] == oracle.OK
    assert oracle.entropy_hist(z, 16, stride=5, block=2, range_all=True)["status"] == oracle.ENONFINITE
    lens = np.array([50, 20], dtype=np.int32)
    per = oracle.entropy_hist(y, 16, seqlens=lens, stride=3, block=2, range_all=True)
    for bb in range(2):
        v = np.ascontiguousarray(y[bb:bb + 1, :, :lens[bb]])
        one = oracle.entropy_hist(v, 16, stride=3, block=2, range_all=True)
        assert (per["counts"][bb] == one["counts"][0]).all() and per["hi"][bb] == v.max()
