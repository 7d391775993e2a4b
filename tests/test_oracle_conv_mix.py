"""Pins for the oracle's reverberation and SNR mixing.  CPU only."""
import numpy as np
import pytest

from oracle import aug_oracle as O


def test_delta_is_a_shift():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(300)
    h = np.zeros(64); h[17] = 1.0
    y = O.convolve_direct(x, h)
    assert len(y) == len(x)
    np.testing.assert_array_equal(y[:17], 0.0)
    np.testing.assert_array_equal(y[17:], x[:-17])


def test_two_tap_filter_by_hand():
    # y[n] = 2 x[n] - 3 x[n-2], causal, length kept
    x = np.array([1.0, 2.0, 3.0, 4.0, 5.0])
    y = O.convolve_direct(x, [2.0, 0.0, -3.0])
    np.testing.assert_array_equal(y, [2.0, 4.0, 3.0, 2.0, 1.0])


def test_linearity_and_commutativity():
    rng = np.random.default_rng(1)
    x1, x2 = rng.standard_normal(200), rng.standard_normal(200)
    h = rng.standard_normal(50)
    np.testing.assert_allclose(O.convolve_direct(2 * x1 - 3 * x2, h),
                               2 * O.convolve_direct(x1, h) - 3 * O.convolve_direct(x2, h),
                               atol=1e-12)
    # x * h = h * x on the common support
    a = O.convolve_direct(x1, h)[:50]
    b = O.convolve_direct(h, x1)[:50]
    np.testing.assert_allclose(a, b, atol=1e-12)


def test_rir_longer_than_signal_and_empty():
    rng = np.random.default_rng(2)
    x = rng.standard_normal(30)
    h = rng.standard_normal(100)
    y = O.convolve_direct(x, h)
    ref = np.array([sum(h[k] * x[n - k] for k in range(n + 1)) for n in range(30)])
    np.testing.assert_allclose(y, ref, atol=1e-12)
    assert len(O.convolve_direct(np.zeros(0), h)) == 0
    assert len(O.convolve_fft(np.zeros(0), h)) == 0


def test_fft_and_sampled_forms_equal_direct():
    rng = np.random.default_rng(3)
    x = rng.standard_normal(5000)
    h = rng.standard_normal(700) * np.exp(-np.arange(700) / 200.0)
    yd = O.convolve_direct(x, h)
    np.testing.assert_allclose(O.convolve_fft(x, h), yd, atol=1e-11)
    pos = rng.integers(0, 5000, size=64)
    np.testing.assert_allclose(O.convolve_at(x, h, pos), yd[pos], atol=1e-11)


def test_measured_snr_equals_target():
    rng = np.random.default_rng(4)
    offsets = np.array([0, 3000, 7000], dtype=np.int64)
    speech = rng.standard_normal(7000).astype(np.float32)
    noise = rng.standard_normal((2, 7000)).astype(np.float32) * 3.0
    rir = rng.standard_normal((2, 3, 200)) * np.exp(-np.arange(200) / 40.0)
    snr = np.array([[5.0, 20.0], [0.0, 12.5]], dtype=np.float32)
    mixed, gains = O.convolve_mix_batch(offsets, speech, noise, rir, snr)
    y = O.reverberate(offsets, speech, noise, rir)
    for u in range(2):
        a, b = offsets[u], offsets[u + 1]
        e0 = np.sum(y[0, a:b] ** 2)
        for j in range(2):
            ej = np.sum((gains[u, j] * y[1 + j, a:b]) ** 2)
            assert 10 * np.log10(e0 / ej) == pytest.approx(snr[u, j], abs=1e-9)
        np.testing.assert_allclose(
            mixed[a:b], y[0, a:b] + gains[u, 0] * y[1, a:b] + gains[u, 1] * y[2, a:b], atol=1e-12)


def test_gain_scales_with_snr_and_degenerate_energy():
    g0 = O.snr_gains(4.0, [1.0], [0.0])
    g20 = O.snr_gains(4.0, [1.0], [20.0])
    assert g0[0] == pytest.approx(2.0)
    assert g20[0] / g0[0] == pytest.approx(10 ** (-20 / 20))
    np.testing.assert_array_equal(O.snr_gains(0.0, [1.0, 2.0], [0.0, 0.0]), 0.0)
    np.testing.assert_array_equal(O.snr_gains(1.0, [0.0], [10.0]), 0.0)


def test_no_noise_sources_returns_reverberated_speech():
    rng = np.random.default_rng(5)
    offsets = np.array([0, 500], dtype=np.int64)
    x = rng.standard_normal(500).astype(np.float32)
    rir = rng.standard_normal((1, 1, 32))
    mixed, gains = O.convolve_mix_batch(offsets, x, None, rir, None)
    np.testing.assert_allclose(mixed, O.convolve_direct(x, rir[0, 0]), atol=1e-13)
    assert gains.shape == (1, 0)
