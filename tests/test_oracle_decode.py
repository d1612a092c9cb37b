"""Pins for the oracle's single-token state update: closed forms, special cases that reduce to library routines, and the
(separately pinned) sequence scan taken one token at a time."""
import math

import numpy as np
import pytest

import oracle


def _rand(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def test_zero_step_size_leaves_the_state_and_reads_it_out():
    B, D, N = 2, 3, 5
    h, x, Bt, Ct, Dv = _rand((B, D, N), 1), _rand((B, D), 2), _rand((B, N), 3), _rand((B, N), 4), _rand((D,), 5)
    A = -np.abs(_rand((D, N), 6))
    so, y = oracle.selective_state_update(h, x, np.zeros((B, D), np.float32), A, Bt, Ct, Dv=Dv, delta_softplus=False)
    np.testing.assert_array_equal(so, h.astype(np.float64))                      # exp(0) h + 0
    want = np.einsum("bn,bdn->bd", Ct.astype(np.float64), h.astype(np.float64)) + Dv[None, :].astype(np.float64) * x
    np.testing.assert_allclose(y, want, rtol=1e-14, atol=1e-15)


def test_softplus_of_zero_is_ln2_and_large_steps_pass_through():
    one = np.ones((1, 1), np.float32)
    zeroA = np.zeros((1, 1), np.float32)
    so, y = oracle.selective_state_update(np.zeros((1, 1, 1), np.float32), one, np.zeros((1, 1), np.float32), zeroA, one, one)
    assert so[0, 0, 0] == pytest.approx(math.log(2.0), rel=1e-15) and y[0, 0] == pytest.approx(math.log(2.0), rel=1e-15)
    so, _ = oracle.selective_state_update(np.zeros((1, 1, 1), np.float32), one, np.full((1, 1), 50.0, np.float32), zeroA, one, one)
    assert so[0, 0, 0] == pytest.approx(50.0, rel=1e-15)
    # the bias is added before the softplus
    so, _ = oracle.selective_state_update(np.zeros((1, 1, 1), np.float32), one, np.full((1, 1), -3.0, np.float32), zeroA, one, one,
                                          delta_bias=np.array([3.0], np.float32))
    assert so[0, 0, 0] == pytest.approx(math.log(2.0), rel=1e-15)


def test_constant_inputs_sum_to_the_geometric_series():
    # h_T = dl * b * x * (1 - q^T) / (1 - q), q = exp(dl * a); with a = 0 it is the arithmetic series T * dl * b * x
    dl, a, b, x, T = 0.25, -0.75, 1.5, 2.0, 40
    for aa in (a, 0.0):
        h = np.zeros((1, 1, 1), np.float64)
        for _ in range(T):
            h, y = oracle.selective_state_update(h.astype(np.float32), np.full((1, 1), x, np.float32), np.full((1, 1), dl, np.float32),
                                                 np.full((1, 1), aa, np.float32), np.full((1, 1), b, np.float32),
                                                 np.full((1, 1), 3.0, np.float32), delta_softplus=False)
        q = math.exp(dl * aa)
        want = T * dl * b * x if aa == 0.0 else dl * b * x * (1 - q ** T) / (1 - q)
        assert h[0, 0, 0] == pytest.approx(want, rel=5e-6)           # the state is handed on as float32 between tokens
        assert y[0, 0] == pytest.approx(3.0 * h[0, 0, 0], rel=1e-14)


def test_gate_multiplies_by_silu_of_z():
    B, D, N = 1, 4, 3
    args = (_rand((B, D, N), 1), _rand((B, D), 2), _rand((B, D), 3), -np.abs(_rand((D, N), 4)), _rand((B, N), 5), _rand((B, N), 6))
    _, y0 = oracle.selective_state_update(*args)
    z = np.array([[0.0, 30.0, -30.0, 1.0]], np.float32)
    s1, y1 = oracle.selective_state_update(*args, z=z)
    gate = np.array([0.0, 30.0, 0.0, 1.0 / (1.0 + math.exp(-1.0))])
    np.testing.assert_allclose(y1[0], y0[0] * gate, rtol=1e-12, atol=1e-11)
    s0, _ = oracle.selective_state_update(*args)
    np.testing.assert_array_equal(s0, s1)                             # the gate does not touch the state


@pytest.mark.parametrize("N", [1, 16, 23])
def test_tokens_one_at_a_time_follow_the_sequence_scan(N):
    B, D, L = 2, 5, 24
    u, dt, z = _rand((B, D, L), 11), _rand((B, D, L), 12, 0.5), _rand((B, D, L), 13)
    A, Dv, bias = -np.exp(_rand((D, N), 14)), _rand((D,), 15), _rand((D,), 16, 0.3)
    Bm, Cm = _rand((B, N, L), 17), _rand((B, N, L), 18)
    st, y_scan, last_scan = oracle.selective_scan(u, dt, A, Bm, Cm, Dv=Dv, z=z, delta_bias=bias, chunk=8)
    assert st == oracle.OK
    # one step from a given state is the scan of a length-1 sequence started there, exactly
    h0 = _rand((B, D, N), 19)
    st, y1, l1 = oracle.selective_scan(u[:, :, :1], dt[:, :, :1], A, Bm[:, :, :1], Cm[:, :, :1], Dv=Dv, z=z[:, :, :1],
                                       delta_bias=bias, h0=h0, chunk=1)
    s1, yy = oracle.selective_state_update(h0, u[:, :, 0], dt[:, :, 0], A, Bm[:, :, 0], Cm[:, :, 0], Dv=Dv, z=z[:, :, 0], delta_bias=bias)
    np.testing.assert_array_equal(s1, l1)
    np.testing.assert_array_equal(yy, y1[:, :, 0])
    # and L steps from the zero state reproduce the whole scan (the state crosses tokens as float32: 2^-24 per token)
    h = np.zeros((B, D, N), np.float64)
    for t in range(L):
        h, y = oracle.selective_state_update(h.astype(np.float32), u[:, :, t], dt[:, :, t], A, Bm[:, :, t], Cm[:, :, t], Dv=Dv,
                                             z=z[:, :, t], delta_bias=bias)
        np.testing.assert_allclose(y, y_scan[:, :, t], rtol=2e-5, atol=2e-5)
    np.testing.assert_allclose(h, last_scan, rtol=1e-5, atol=1e-5)
