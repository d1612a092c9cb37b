"""Pins for the oracle's selective scan: a hand-worked example, closed forms, special cases that reduce
to numpy/scipy routines, an independent O(L^2) formulation, and the invariants the method must keep."""
import math

import numpy as np
import pytest
from scipy.signal import lfilter
from scipy.special import expit

import oracle
from conftest import read_golden

LN2 = math.log(2.0)


def _rand(shape, rng, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float32)


def _problem(rng, B=2, D=3, N=4, L=37):
    return dict(u=_rand((B, D, L), rng), delta=_rand((B, D, L), rng, 0.5),
                A=-np.exp(_rand((D, N), rng)), Bm=_rand((B, N, L), rng), Cm=_rand((B, N, L), rng),
                Dv=_rand((D,), rng), z=_rand((B, D, L), rng),
                delta_bias=rng.uniform(-3, 0, D).astype(np.float32))


def test_hand_worked_example():
    rows = {r[0]: [float(v) for v in r[1:]] for r in read_golden("scan_hand_example.txt")}
    u = np.array([[[1, 2, -1]]], dtype=np.float32)
    delta = np.ones((1, 1, 3), dtype=np.float32)
    A = np.array([[-LN2, -2 * LN2]], dtype=np.float32)
    Bm = np.array([[[1, 2, 3], [1, 1, 1]]], dtype=np.float32)
    Cm = np.array([[[1, 0, 1], [2, 1, 0]]], dtype=np.float32)
    st, y, last = oracle.selective_scan(u, delta, A, Bm, Cm, Dv=np.array([0.5], np.float32),
                                        delta_softplus=False, chunk=2)
    assert st == oracle.OK
    np.testing.assert_allclose(y[0, 0], rows["y"], rtol=0, atol=5e-7)      # A is binary32(-ln 2)
    np.testing.assert_allclose(last[0, 0], rows["last_state"], rtol=0, atol=5e-7)


def test_constant_inputs_give_a_geometric_series():
    L, N = 200, 3
    dl, uu, bb, cc = 0.25, 1.5, -0.75, 2.0
    A = np.array([[-0.4, -1.0, -3.0]], dtype=np.float32)
    full = lambda v: np.full((1, 1, L), v, dtype=np.float32)
    st, y, last = oracle.selective_scan(full(uu), full(dl), A, np.full((1, N, L), bb, np.float32),
                                        np.full((1, N, L), cc, np.float32), delta_softplus=False, chunk=64)
    abar = np.exp(dl * A[0].astype(np.float64))
    t = np.arange(1, L + 1)[:, None]
    h = dl * bb * uu * (1 - abar ** t) / (1 - abar)             # (L, N)
    np.testing.assert_allclose(y[0, 0], cc * h.sum(1), rtol=1e-12)
    np.testing.assert_allclose(last[0, 0], h[-1], rtol=1e-12)


def test_time_invariant_case_is_a_first_order_filter():
    rng = np.random.default_rng(2)
    B, D, N, L = 1, 2, 3, 120
    p = _problem(rng, B, D, N, L)
    dl = np.float32(0.3)
    delta = np.full((B, D, L), dl, dtype=np.float32)
    st, y, last = oracle.selective_scan(p["u"], delta, p["A"], p["Bm"], p["Cm"], Dv=p["Dv"], z=p["z"],
                                        delta_softplus=False, chunk=32)
    for d in range(D):
        acc = np.zeros(L)
        for n in range(N):
            a = math.exp(float(dl) * float(p["A"][d, n]))
            x = float(dl) * p["Bm"][0, n].astype(np.float64) * p["u"][0, d].astype(np.float64)
            h = lfilter([1.0], [1.0, -a], x)
            acc += p["Cm"][0, n].astype(np.float64) * h
            assert last[0, d, n] == pytest.approx(h[-1], rel=1e-11, abs=1e-13)
        zz = p["z"][0, d].astype(np.float64)
        ref = (acc + float(p["Dv"][d]) * p["u"][0, d].astype(np.float64)) * zz * expit(zz)
        np.testing.assert_allclose(y[0, d], ref, rtol=1e-11, atol=1e-13)


def test_zero_A_is_a_running_sum_and_softplus_is_logaddexp():
    rng = np.random.default_rng(3)
    B, D, N, L = 2, 3, 2, 90
    p = _problem(rng, B, D, N, L)
    p["delta"] = (p["delta"] * 8).astype(np.float32)            # reach both softplus tails
    A = np.zeros((D, N), dtype=np.float32)
    st, y, last = oracle.selective_scan(p["u"], p["delta"], A, p["Bm"], p["Cm"], delta_bias=p["delta_bias"],
                                        delta_softplus=True, chunk=16)
    dl = np.logaddexp(0.0, p["delta"].astype(np.float64) + p["delta_bias"].astype(np.float64)[None, :, None])
    for b in range(B):
        for d in range(D):
            x = dl[b, d][None, :] * p["Bm"][b].astype(np.float64) * p["u"][b, d].astype(np.float64)[None, :]
            h = np.cumsum(x, axis=1)                            # (N, L)
            np.testing.assert_allclose(y[b, d], (p["Cm"][b].astype(np.float64) * h).sum(0), rtol=1e-11, atol=1e-12)
            np.testing.assert_allclose(last[b, d], h[:, -1], rtol=1e-11, atol=1e-12)


def test_against_the_unrolled_sum_over_all_earlier_steps():
    # h_t = sum_{s<=t} exp(S_t - S_s) b_s  with  S = cumsum(delta * A): an O(L^2) formulation with no recurrence
    rng = np.random.default_rng(4)
    B, D, N, L = 2, 2, 3, 48
    p = _problem(rng, B, D, N, L)
    h0 = _rand((B, D, N), rng)
    st, y, last = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], Dv=p["Dv"], z=p["z"],
                                        delta_bias=p["delta_bias"], delta_softplus=True, h0=h0, chunk=16)
    f8 = lambda a: a.astype(np.float64)
    dl = np.logaddexp(0.0, f8(p["delta"]) + f8(p["delta_bias"])[None, :, None])
    tri = np.tril(np.ones((L, L)))
    for b in range(B):
        for d in range(D):
            acc = np.zeros(L)
            for n in range(N):
                S = np.cumsum(dl[b, d] * float(p["A"][d, n]))
                bs = dl[b, d] * f8(p["Bm"][b, n]) * f8(p["u"][b, d])
                W = np.exp(S[:, None] - S[None, :]) * tri          # W[t, s] = prod_{j=s+1..t} abar_j
                h = W @ bs + np.exp(S) * float(h0[b, d, n])
                acc += f8(p["Cm"][b, n]) * h
                assert last[b, d, n] == pytest.approx(h[-1], rel=1e-10, abs=1e-12)
            zz = f8(p["z"][b, d])
            ref = (acc + float(p["Dv"][d]) * f8(p["u"][b, d])) * zz / (1 + np.exp(-zz))
            np.testing.assert_allclose(y[b, d], ref, rtol=1e-10, atol=1e-12)


def test_strong_decay_makes_the_scan_memoryless():
    rng = np.random.default_rng(5)
    p = _problem(rng, 1, 2, 3, 40)
    A = np.full((2, 3), -1e4, dtype=np.float32)
    delta = np.abs(p["delta"]) + np.float32(0.5)
    st, y, last = oracle.selective_scan(p["u"], delta, A, p["Bm"], p["Cm"], Dv=p["Dv"], delta_softplus=False)
    f8 = lambda a: a.astype(np.float64)
    for d in range(2):
        ref = (f8(p["Cm"][0]) * f8(p["Bm"][0])).sum(0) * f8(delta[0, d]) * f8(p["u"][0, d]) \
            + float(p["Dv"][d]) * f8(p["u"][0, d])
        np.testing.assert_allclose(y[0, d], ref, rtol=1e-12, atol=1e-14)


def test_linearity_in_u_is_exact_for_powers_of_two():
    rng = np.random.default_rng(6)
    p = _problem(rng)
    kw = dict(Dv=p["Dv"], z=p["z"], delta_bias=p["delta_bias"], delta_softplus=True, chunk=8)
    _, y1, s1 = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], **kw)
    _, y2, s2 = oracle.selective_scan(p["u"] * np.float32(4), p["delta"], p["A"], p["Bm"], p["Cm"], **kw)
    assert np.array_equal(y2, 4 * y1) and np.array_equal(s2, 4 * s1)


def test_chunk_does_not_change_the_result():
    rng = np.random.default_rng(7)
    p = _problem(rng, 2, 3, 4, 300)
    kw = dict(Dv=p["Dv"], z=p["z"], delta_bias=p["delta_bias"], delta_softplus=True)
    ref = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], chunk=300, **kw)
    for chunk in (1, 7, 64, 128, 256, 2048):
        st, y, s = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], chunk=chunk, **kw)
        assert st == oracle.OK and np.array_equal(y, ref[1]) and np.array_equal(s, ref[2])


def test_split_sequence_continues_from_the_carried_state():
    rng = np.random.default_rng(8)
    p = _problem(rng, 2, 3, 4, 100)
    kw = dict(Dv=p["Dv"], delta_bias=p["delta_bias"], delta_softplus=True)
    _, y, s = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], z=p["z"], **kw)
    cut = 37
    head = lambda a: np.ascontiguousarray(a[..., :cut])
    tail = lambda a: np.ascontiguousarray(a[..., cut:])
    _, y1, s1 = oracle.selective_scan(head(p["u"]), head(p["delta"]), p["A"], head(p["Bm"]), head(p["Cm"]),
                                      z=head(p["z"]), **kw)
    _, y2, s2 = oracle.selective_scan(tail(p["u"]), tail(p["delta"]), p["A"], tail(p["Bm"]), tail(p["Cm"]),
                                      z=tail(p["z"]), h0=s1.astype(np.float32), **kw)
    assert np.array_equal(y1, y[..., :cut])
    np.testing.assert_allclose(y2, y[..., cut:], rtol=1e-6, atol=1e-6)    # the hand-over is rounded to binary32
    np.testing.assert_allclose(s2, s, rtol=1e-6, atol=1e-6)


def test_gate_and_padding():
    rng = np.random.default_rng(9)
    p = _problem(rng, 2, 3, 4, 50)
    kw = dict(Dv=p["Dv"], delta_bias=p["delta_bias"], delta_softplus=True)
    _, y_plain, s_plain = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], **kw)
    _, y_gate, s_gate = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], z=p["z"], **kw)
    zz = p["z"].astype(np.float64)
    np.testing.assert_allclose(y_gate, y_plain * zz * expit(zz), rtol=1e-13, atol=1e-15)
    assert np.array_equal(s_gate, s_plain)
    _, y0, _ = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], z=np.zeros_like(p["z"]), **kw)
    assert not y0.any()
    lens = np.array([50, 13], dtype=np.int32)
    _, yl, sl = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], z=p["z"], seqlens=lens, **kw)
    assert np.array_equal(yl[0], y_gate[0]) and np.array_equal(sl[0], s_gate[0])
    assert not yl[1, :, 13:].any() and np.array_equal(yl[1, :, :13], y_gate[1, :, :13])
    cut = lambda a: np.ascontiguousarray(a[1:2, ..., :13])
    _, yt, stt = oracle.selective_scan(cut(p["u"]), cut(p["delta"]), p["A"], cut(p["Bm"]), cut(p["Cm"]),
                                       z=cut(p["z"]), **kw)
    assert np.array_equal(stt[0], sl[1])


def test_size_of_the_terms_for_a_checkers_rounding_bound():
    """The optional extra output: the sum of the absolute values of the terms every y is made of.  With every term
    positive it is y itself; in general it bounds |y|, equals the unrolled sum of |C h| + |D u| times |gate|, is zero on
    padding, and asking for it changes neither y nor the state."""
    rng = np.random.default_rng(21)
    p = _problem(rng, 2, 3, 4, 29)
    kw = dict(Dv=p["Dv"], delta_bias=p["delta_bias"], delta_softplus=True)
    lens = np.array([29, 11], dtype=np.int32)
    st, y, s, terms = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], z=p["z"], seqlens=lens, want_terms=True, **kw)
    _, y_b, s_b = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], z=p["z"], seqlens=lens, **kw)
    assert st == oracle.OK and np.array_equal(y, y_b) and np.array_equal(s, s_b)
    assert (terms >= np.abs(y) * (1 - 1e-14)).all() and not terms[1, :, 11:].any() and (terms[0] > 0).all()
    # every operand positive, no gate: no cancellation anywhere
    pos = {k: np.abs(v) for k, v in p.items()}
    _, y_p, _, t_p = oracle.selective_scan(pos["u"], p["delta"], p["A"], pos["Bm"], pos["Cm"], Dv=pos["Dv"], delta_bias=p["delta_bias"],
                                           want_terms=True)
    np.testing.assert_allclose(t_p, y_p, rtol=1e-14)
    # written out for one element: states by the recurrence in numpy, then the absolute read-out
    b, d, t_end = 0, 1, 7
    dl = np.logaddexp(0.0, p["delta"][b, d, :t_end + 1].astype(np.float64) + float(p["delta_bias"][d]))
    h = np.zeros(4)
    for t in range(t_end + 1):
        h = np.exp(dl[t] * p["A"][d].astype(np.float64)) * h + dl[t] * p["Bm"][b, :, t].astype(np.float64) * float(p["u"][b, d, t])
    zz = float(p["z"][b, d, t_end])
    want = (np.abs(p["Cm"][b, :, t_end].astype(np.float64) * h).sum() + abs(float(p["Dv"][d]) * float(p["u"][b, d, t_end]))) * abs(zz * expit(zz))
    assert terms[b, d, t_end] == pytest.approx(want, rel=1e-12)


def test_argument_errors():
    rng = np.random.default_rng(10)
    p = _problem(rng, 1, 2, 2, 8)
    st, _, _ = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], chunk=0)
    assert st == oracle.EINVAL
    st, _, _ = oracle.selective_scan(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"],
                                     seqlens=np.array([9], np.int32))
    assert st == oracle.EINVAL
