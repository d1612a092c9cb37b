"""Pins for the oracle's chunk rule (Eq. 2 and the scheduler family around it): the decisions the paper prints."""
import math

import pytest

import oracle
from conftest import read_golden


def _href(tok):
    return math.log(int(tok.split(":")[1])) if tok.startswith("logK:") else float(tok)


@pytest.mark.parametrize("row", read_golden("chunk_rule_pins.txt"), ids=lambda r: "-".join(r))
def test_chunks_printed_in_the_paper(row):
    H, href, cmin, cmax, expect = float(row[0]), _href(row[1]), int(row[2]), int(row[3]), int(row[4])
    r = min(H / href, 1.0)
    st, chunk, margin = oracle.select_chunk(r, 4096, oracle.policy(c_min=cmin, c_max=cmax))
    assert st == oracle.OK and chunk == expect, (chunk, expect, margin)
    # the same decision reached through h_ref_scale on the calibrated r (K = 256)
    if not row[1].startswith("logK:"):
        r256 = min(H / math.log(256), 1.0)
        if r256 < 1.0:
            st, c2, _ = oracle.select_chunk(r256, 4096, oracle.policy(c_min=cmin, c_max=cmax,
                                                                      h_ref_scale=math.log(256) / href))
            assert c2 == expect


@pytest.mark.parametrize("row", read_golden("chunk_rule_r_pins.txt"), ids=lambda r: "-".join(r))
def test_chunks_printed_for_r(row):
    r, cmin, cmax, expect = float(row[0]), int(row[1]), int(row[2]), int(row[3])
    st, chunk, _ = oracle.select_chunk(r, 4096, oracle.policy(c_min=cmin, c_max=cmax))
    assert st == oracle.OK and chunk == expect


def test_rule_is_monotone_clipped_and_power_of_two():
    pol = oracle.policy(c_min=64, c_max=2048)
    last = 0
    seen = set()
    for i in range(0, 1001):
        st, c, margin = oracle.select_chunk(i / 1000.0, 1 << 20, pol)
        assert st == oracle.OK and c >= last and 64 <= c <= 2048 and (c & (c - 1)) == 0
        assert 0.0 <= margin <= 0.5
        last = c
        seen.add(c)
    assert seen == {64, 128, 256, 512, 1024, 2048}
    assert oracle.select_chunk(-3.0, 4096, pol)[1] == 64 and oracle.select_chunk(7.0, 4096, pol)[1] == 2048


def test_switch_points_are_the_geometric_midpoints():
    # 2^round(log2 v) flips where v = 2^(k + 1/2): r* = (2^(k+1/2) - c_min) / (c_max - c_min)
    pol = oracle.policy(c_min=32, c_max=512)
    for k in range(5, 9):
        rstar = (2.0 ** (k + 0.5) - 32) / 480.0
        assert oracle.select_chunk(rstar - 1e-9, 4096, pol)[1] == 2 ** k
        assert oracle.select_chunk(rstar + 1e-9, 4096, pol)[1] == 2 ** (k + 1)


def test_sequence_length_table_and_gate():
    table = oracle.policy(mode=2)                               # <= 50 tokens -> 128, else 512
    assert [oracle.select_chunk(0.9, L, table)[1] for L in (25, 50, 51, 976, 2100)] == [128, 128, 512, 512, 512]
    gate = oracle.policy(mode=1, c_min=32, c_max=512)
    assert oracle.select_chunk(0.83, 4096, gate)[1] == 512      # long: entropy rule
    assert oracle.select_chunk(0.83, 40, gate)[1] == 128        # short: table value, as printed
    assert oracle.select_chunk(0.83, 51, gate)[1] == 64         # just past the gate: Eq. 2, capped by L


def test_guarded_fallback():
    # the routed run: prediction 1024 is one bucket from the safe 512 -> guard fires -> 512
    g = oracle.policy(mode=4, c_min=64, c_max=2048, safe_chunk=512, guard_buckets=2)
    assert oracle.select_chunk(0.5, 4096, oracle.policy(c_min=64, c_max=2048))[1] == 1024
    assert oracle.select_chunk(0.5, 4096, g)[1] == 512
    assert oracle.select_chunk(0.0, 4096, g)[1] == 64           # three buckets away: kept
    assert oracle.select_chunk(0.04, 4096, g)[1] == 128         # two buckets away: kept
    assert oracle.select_chunk(1.0, 4096, g)[1] == 2048         # two buckets away: kept
    assert oracle.select_chunk(0.12, 4096, g)[1] == 512         # 256 is one bucket away -> fallback


def test_cap_by_length_static_and_errors():
    pol = oracle.policy(c_min=64, c_max=2048)
    assert oracle.select_chunk(1.0, 256, pol)[1] == 256         # candidates {64,128,256} at L = 256
    assert oracle.select_chunk(1.0, 300, pol)[1] == 512
    assert oracle.select_chunk(1.0, 10, pol)[1] == 64
    assert oracle.select_chunk(0.2, 4096, oracle.policy(mode=3, static_chunk=1024))[1] == 1024
    assert oracle.select_chunk(float("nan"), 4096, pol)[0] == oracle.ENONFINITE
    assert oracle.select_chunk(0.5, 0, pol)[0] == oracle.EINVAL
    assert oracle.select_chunk(0.5, 64, oracle.policy(c_min=48))[0] == oracle.EINVAL
    assert oracle.select_chunk(0.5, 64, oracle.policy(mode=9))[0] == oracle.EINVAL


# ------------------------------------------------------------------------------------------------ EMA of the entropy
def test_ema_closed_forms():
    """H^_t = lambda H^_{t-1} + (1 - lambda) H_t ("Entropy Estimation Protocol").  Pins: a hand-computed three-step run,
    the fixed point of a constant input, the geometric step response H (1 - lambda^t) + lambda^t H^_0, and the
    horizon the paper quotes for lambda = 0.85 (about 1 / (1 - lambda) = 6.7 calls; "stable after 6-8 observations")."""
    nan = float("nan")
    lam = 0.85
    # by hand: start 2.0 (first observation taken as is), then 4.0 -> 0.85*2 + 0.15*4 = 2.3, then 1.0 -> 0.85*2.3 + 0.15 = 2.105
    s = oracle.ema_update(lam, nan, 2.0)
    assert s == 2.0
    s = oracle.ema_update(lam, s, 4.0)
    assert abs(s - 2.3) < 1e-15
    s = oracle.ema_update(lam, s, 1.0)
    assert abs(s - 2.105) < 1e-15
    # constant input is a fixed point
    s = 3.25
    for _ in range(50):
        s = oracle.ema_update(lam, s, 3.25)
    assert s == 3.25
    # step response from H^_0 = 1 towards H = 5: closed form
    s, h0, H = 1.0, 1.0, 5.0
    for t in range(1, 40):
        s = oracle.ema_update(lam, s, H)
        assert abs(s - (H * (1 - lam ** t) + lam ** t * h0)) < 1e-12
    # the paper's horizon: after 7 observations about a third of the initial value is left, after 14 a tenth
    assert 0.30 < lam ** 7 < 0.34 and lam ** 14 < 0.11
    # lambda = 0 follows the input, a NaN observation leaves the estimate alone
    assert oracle.ema_update(0.0, 7.0, 1.5) == 1.5
    assert oracle.ema_update(lam, 2.0, nan) == 2.0


def test_library_ema_matches_oracle():
    from paper_2604_10597_amd import binding
    import numpy as np
    rng = np.random.default_rng(5)
    s_lib = s_or = float("nan")
    for H in rng.uniform(0, 5.5, 200):
        s_lib = binding.corey_ema_update(0.85, s_lib, float(H))
        s_or = oracle.ema_update(0.85, s_or, float(H))
        assert s_lib == s_or
    for bad in (-0.1, 1.0, float("nan")):
        with pytest.raises(binding.CoreyError):
            binding.corey_ema_update(bad, 1.0, 1.0)
