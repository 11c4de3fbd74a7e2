"""Pins of the oracle's ShortConv (paper Sec. 3.1.3) against hand-worked values, numpy.convolve and its structure."""
import os

import numpy as np

import oracle


def _golden(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "short_conv_hand_worked.txt")) as fh:
        for line in fh:
            if line.startswith("#") or ":" not in line:
                continue
            key, rest = line.split(":")
            vals[key.strip()] = np.array([float(t) for t in rest.split()])
    return vals


def test_hand_worked_values(golden_dir):
    gold = _golden(golden_dir)
    x = np.array([1.0, 2.0, 3.0], np.float32).reshape(1, 3, 1)
    w = np.array([[0.5, -1.0, 2.0]], np.float32)
    b = np.array([0.25], np.float32)
    y, st = oracle.short_conv(x, w, b, None, "none")
    assert np.array_equal(y.ravel(), gold["linear_zero_history"])
    assert np.array_equal(st.ravel(), gold["state_after"])
    hist = np.array([7.0, -4.0], np.float32).reshape(1, 2, 1)
    y, st = oracle.short_conv(x, w, b, hist, "none")
    assert np.array_equal(y.ravel(), gold["linear_with_history"])
    assert np.array_equal(st.ravel(), gold["state_after"])
    y, _ = oracle.short_conv(x, w, b, None, "silu")
    np.testing.assert_allclose(y.ravel(), gold["silu_zero_history"], rtol=1e-15)


def test_matches_numpy_convolve_per_channel():
    rng = np.random.default_rng(11)
    B, T, C, W = 2, 37, 5, 4
    x = rng.standard_normal((B, T, C)).astype(np.float32)
    w = rng.standard_normal((C, W)).astype(np.float32)
    b = rng.standard_normal(C).astype(np.float32)
    y, st = oracle.short_conv(x, w, b, None, "none")
    for bi in range(B):
        for c in range(C):
            # convolve flips its second argument: tap j of the causal filter multiplies the input W-1-j steps back
            ref = np.convolve(x[bi, :, c].astype(np.float64), w[c, ::-1].astype(np.float64))[:T] + b[c]
            np.testing.assert_allclose(y[bi, :, c], ref, rtol=1e-13, atol=1e-13)
    assert np.array_equal(st, x[:, T - (W - 1):, :].astype(np.float64))
    ys, _ = oracle.short_conv(x, w, b, None, "silu")
    np.testing.assert_allclose(ys, y / (1.0 + np.exp(-y)), rtol=1e-14)


def test_impulse_response_and_identity():
    C, W, T = 3, 4, 9
    w = np.arange(1, C * W + 1, dtype=np.float32).reshape(C, W)
    x = np.zeros((1, T, C), np.float32)
    x[0, 2, :] = 1.0
    y, _ = oracle.short_conv(x, w, None, None, "none")
    for c in range(C):
        # an impulse at t = 2 meets tap W-1 first (no delay), then W-2, ...
        assert np.array_equal(y[0, 2:2 + W, c], w[c, ::-1].astype(np.float64))
        assert np.all(y[0, :2, c] == 0) and np.all(y[0, 2 + W:, c] == 0)
    # W = 1 with unit tap and no bias is the identity; its carried state is empty
    xr = np.random.default_rng(3).standard_normal((2, 5, 4)).astype(np.float32)
    y, st = oracle.short_conv(xr, np.ones((4, 1), np.float32), None, None, "none")
    assert np.array_equal(y, xr.astype(np.float64)) and st.shape == (2, 0, 4)


def test_split_sequence_chaining_and_short_calls():
    rng = np.random.default_rng(5)
    B, T, C, W = 2, 23, 6, 4
    x = rng.standard_normal((B, T, C)).astype(np.float32)
    w = rng.standard_normal((C, W)).astype(np.float32)
    b = rng.standard_normal(C).astype(np.float32)
    hist = rng.standard_normal((B, W - 1, C)).astype(np.float32)
    y_all, st_all = oracle.short_conv(x, w, b, hist, "silu")
    # one token at a time (the decode form), two tokens at a time (shorter than the history), and an uneven split
    for cuts in ([1] * T, [2] * 11 + [1], [7, 0, 16]):
        st = hist
        pieces, t = [], 0
        for n in cuts:
            y, st64 = oracle.short_conv(x[:, t:t + n], w, b, st, "silu")
            st = st64.astype(np.float32)          # inputs are float32: the carried state is exact
            assert np.array_equal(st.astype(np.float64), st64)
            pieces.append(y)
            t += n
        assert np.array_equal(np.concatenate(pieces, axis=1), y_all)
        assert np.array_equal(st.astype(np.float64), st_all)
    # a planted mistake is caught: reversing the taps changes the result
    y_rev, _ = oracle.short_conv(x, w[:, ::-1].copy(), b, hist, "silu")
    assert np.abs(y_rev - y_all).max() > 0.1
