"""Pins for the oracle's causal convolution + SiLU (the producer of the scan input, step (1) of the paper's inline hook)
against things that are not the oracle: scipy's FIR filter and logistic function, the impulse response, a hand-worked
example, causality and the continuation property of the carried state."""
import numpy as np
import pytest
from scipy.signal import lfilter
from scipy.special import expit

import oracle


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


@pytest.mark.parametrize("W", [1, 2, 3, 4])
def test_equals_scipy_fir_filter_then_logistic_gate(W):
    B, D, L = 2, 5, 67
    x, w, b = _rand((B, D, L), 1), _rand((D, W), 2), _rand((D,), 3)
    u, _ = oracle.causal_conv1d_silu(x, w, b)
    for bi in range(B):
        for d in range(D):
            # weight[d, W-1] multiplies the current input, weight[d, 0] the oldest: FIR coefficients are the reverse
            v = lfilter(w[d, ::-1].astype(np.float64), [1.0], x[bi, d].astype(np.float64)) + float(b[d])
            np.testing.assert_allclose(u[bi, d], v * expit(v), rtol=1e-13, atol=1e-15)


def test_hand_worked_example():
    # W = 2, weight = [1, 2], bias = 0.5, x = [1, 2, 3]:  v = [2*1, 1*1 + 2*2, 1*2 + 2*3] + 0.5 = [2.5, 5.5, 8.5]
    u, so = oracle.causal_conv1d_silu(np.array([[[1, 2, 3]]], np.float32), np.array([[1, 2]], np.float32), np.array([0.5], np.float32))
    v = np.array([2.5, 5.5, 8.5])
    np.testing.assert_allclose(u[0, 0], v / (1 + np.exp(-v)), rtol=1e-15)
    assert so[0, 0].tolist() == [3.0]


def test_impulse_response_is_the_reversed_taps():
    W, L = 4, 9
    w = np.array([[0.25, -0.5, 2.0, 3.0]], np.float32)
    x = np.zeros((1, 1, L), np.float32)
    x[0, 0, 0] = 1.0
    u, _ = oracle.causal_conv1d_silu(x, w)
    v = np.zeros(L)
    v[:W] = w[0, ::-1]
    np.testing.assert_allclose(u[0, 0], v * expit(v), rtol=1e-15, atol=0)
    # width 1 with unit weight is SiLU itself; silu(0) = 0 and silu(v) -> v for large v
    xs = np.array([[[0.0, 40.0, -40.0, 1.0]]], np.float32)
    u1, _ = oracle.causal_conv1d_silu(xs, np.ones((1, 1), np.float32))
    assert u1[0, 0, 0] == 0.0 and u1[0, 0, 1] == pytest.approx(40.0, rel=1e-15) and abs(u1[0, 0, 2]) < 1e-15
    assert u1[0, 0, 3] == pytest.approx(1.0 / (1.0 + np.exp(-1.0)), rel=1e-15)


def test_causal_and_channelwise():
    B, D, L, W = 1, 3, 40, 4
    x, w, b = _rand((B, D, L), 4), _rand((D, W), 5), _rand((D,), 6)
    u0, _ = oracle.causal_conv1d_silu(x, w, b)
    x2 = x.copy()
    x2[0, 1, 17] += 3.0
    u1, _ = oracle.causal_conv1d_silu(x2, w, b)
    changed = np.argwhere(u0 != u1)
    assert set(map(tuple, changed)) <= {(0, 1, t) for t in range(17, 17 + W)}       # only that channel, only t .. t+W-1
    assert (0, 1, 17) in set(map(tuple, changed))


@pytest.mark.parametrize("W,cut", [(4, 23), (4, 2), (3, 1), (2, 30)])
def test_carried_state_continues_the_sequence(W, cut):
    B, D, L = 2, 3, 41
    x, w, b = _rand((B, D, L), 7), _rand((D, W), 8), _rand((D,), 9)
    whole, s_whole = oracle.causal_conv1d_silu(x, w, b)
    first, s1 = oracle.causal_conv1d_silu(x[:, :, :cut], w, b)
    second, s2 = oracle.causal_conv1d_silu(x[:, :, cut:], w, b, state_in=s1)
    np.testing.assert_array_equal(np.concatenate([first, second], axis=2), whole)
    np.testing.assert_array_equal(s2, s_whole)
    np.testing.assert_array_equal(s_whole, x[:, :, L - (W - 1):])
    # a first part shorter than W - 1 keeps the older zeros in front
    if cut < W - 1:
        assert np.all(s1[:, :, : W - 1 - cut] == 0) and np.array_equal(s1[:, :, W - 1 - cut:], x[:, :, :cut])
