"""Pins of the waveform-resynthesis VTLP oracle against Eq. (1) and what the mathematics fixes."""
import numpy as np
import pytest

from oracle import aug_oracle as O
from oracle import vtlp_resynth_oracle as V


@pytest.mark.parametrize("alpha", [0.8, 0.93, 1.0, 1.1, 1.2])
def test_inverse_warp_undoes_eq1(alpha):
    # Eq. (1) (pinned on its own in test_oracle_frontend.py) applied to the inverse gives the identity
    w_out = np.linspace(0.0, np.pi, 1025)
    np.testing.assert_allclose(O.bilinear_warp(V.inverse_warp(w_out, alpha), alpha), w_out, atol=1e-12)
    w_in = V.inverse_warp(w_out, alpha)
    assert w_in[0] == 0.0 and abs(w_in[-1] - np.pi) < 1e-12 and np.all(np.diff(w_in) > 0)


@pytest.mark.parametrize("alpha", [0.8, 1.2])
def test_interpolation_reads_the_bin_that_eq1_maps_onto_the_output_bin(alpha):
    # A spectrum that is a linear ramp, X[k] = k, is reproduced exactly by linear interpolation, so the
    # warped spectrum is the fractional source bin itself.  The source bin is found here by bisection on
    # Eq. (1), without the closed-form inverse.
    nfft = 256
    Y = V.warp_spectrum(np.arange(nfft // 2 + 1, dtype=np.complex128), alpha, nfft)
    assert np.max(np.abs(Y.imag)) == 0.0
    for k_out in [0, 1, 7, 40, 77, 100, 127, 128]:
        lo, hi = 0.0, np.pi
        for _ in range(80):
            mid = 0.5 * (lo + hi)
            if O.bilinear_warp(mid, alpha) < 2.0 * np.pi * k_out / nfft:
                lo = mid
            else:
                hi = mid
        assert abs(Y[k_out].real - 0.5 * (lo + hi) * nfft / (2.0 * np.pi)) < 1e-9
    # between the two nearest bins: the chord of the convex k^2 lies above it, by at most 1/4 on a unit interval
    # (an extrapolation from the wrong pair of bins falls below)
    kappa = Y.real
    Y2 = V.warp_spectrum(np.arange(nfft // 2 + 1, dtype=np.complex128) ** 2, alpha, nfft).real
    assert np.all(Y2 >= kappa ** 2 - 1e-9) and np.all(Y2 <= kappa ** 2 + 0.25 + 1e-9)
    assert np.max(Y2 - kappa ** 2) > 0.2
    # direction: alpha < 1 moves energy up (Eq. (1) with 1 - alpha > 0), so an output bin reads a lower one
    assert (Y[64].real < 64) == (alpha < 1.0)


def test_window_weights_of_the_two_frames_over_a_sample_add_up_to_one():
    w = V.hann_periodic(800)
    np.testing.assert_allclose(w[:400] + w[400:], 1.0, atol=1e-15)
    assert w[0] == 0.0 and abs(w[400] - 1.0) < 1e-15
    assert [V.resynth_frame_count(n, 400) for n in (0, 1, 400, 401, 800, 801)] == [0, 2, 2, 3, 3, 4]


@pytest.mark.parametrize("n", [1, 399, 400, 401, 1000, 4321])
def test_alpha_one_returns_the_input(n):
    x = np.random.default_rng(n).standard_normal(n)
    np.testing.assert_allclose(V.vtlp_resynth(x, 1.0), x, atol=1e-12)


@pytest.mark.parametrize("alpha", [0.8, 1.2])
def test_impulse_on_a_frame_centre_is_untouched(alpha):
    # It falls on the one sample of its frame with window weight 1 (the neighbouring frames weigh it 0),
    # sits at time zero of the transform buffer, has a flat spectrum, and a flat spectrum warps to itself.
    x = np.zeros(3000)
    x[1200] = 2.5
    np.testing.assert_allclose(V.vtlp_resynth(x, alpha), x, atol=1e-12)
    # off the centre the spectrum has a phase slope and the warp does change the frame
    x = np.zeros(3000)
    x[1300] = 2.5
    assert np.max(np.abs(V.vtlp_resynth(x, alpha) - x)) > 0.1


@pytest.mark.parametrize("alpha,f0", [(0.8, 1000.0), (1.2, 1000.0), (0.9, 2500.0)])
def test_pure_tone_moves_to_the_frequency_of_eq1(alpha, f0):
    fs, n = 16000.0, 16000
    t = np.arange(n)
    y = V.vtlp_resynth(np.cos(2.0 * np.pi * f0 / fs * t), alpha)
    f_want = float(O.bilinear_warp(2.0 * np.pi * f0 / fs, alpha)) * fs / (2.0 * np.pi)
    assert abs(f_want - f0) > 200.0
    seg = y[4000:12192] * np.hanning(8192)
    spec = np.abs(np.fft.rfft(seg, 65536)) ** 2
    freqs = np.arange(spec.shape[0]) * fs / 65536
    # Frames are overlap-added with the input's phase advance, so the output is a cluster of lines one
    # frame rate (fs / hop = 40 Hz) apart under the warped window's envelope, centred on the warped frequency.
    f_peak = freqs[np.argmax(spec)]
    assert abs(f_peak - f_want) <= 20.0 + 1.0
    near = np.abs(freqs - f_want) <= 120.0
    assert spec[near].sum() >= 0.98 * spec.sum()
    centroid = (freqs[near] * spec[near]).sum() / spec[near].sum()
    assert abs(centroid - f_want) <= 10.0
    assert 0.5 <= np.sqrt(np.mean(y[4000:12000] ** 2)) / np.sqrt(0.5) <= 1.2


def test_linear_and_covariant_under_shifts_by_the_hop():
    rng = np.random.default_rng(5)
    x, z = rng.standard_normal(2600), rng.standard_normal(2600)
    np.testing.assert_allclose(V.vtlp_resynth(2.0 * x - 3.0 * z, 0.85),
                               2.0 * V.vtlp_resynth(x, 0.85) - 3.0 * V.vtlp_resynth(z, 0.85), atol=1e-11)
    pad = np.zeros(1200)
    base = V.vtlp_resynth(np.concatenate([pad, x, pad]), 1.15)
    moved = V.vtlp_resynth(np.concatenate([pad, np.zeros(400), x, pad[400:]]), 1.15)
    np.testing.assert_allclose(moved[400:], base[:-400], atol=1e-11)


def test_batch_is_per_utterance():
    rng = np.random.default_rng(6)
    lens = [900, 0, 1, 2500]
    off = np.concatenate([[0], np.cumsum(lens)])
    x = rng.standard_normal(off[-1])
    alpha = np.array([0.8, 1.0, 1.2, 1.1])
    y = V.vtlp_resynth_batch(off, x, alpha)
    for u in range(4):
        np.testing.assert_array_equal(y[off[u]:off[u + 1]], V.vtlp_resynth(x[off[u]:off[u + 1]], alpha[u]))
    # noise keeps roughly its level
    assert 0.7 <= np.sqrt(np.mean(y[off[3]:] ** 2)) / np.sqrt(np.mean(x[off[3]:] ** 2)) <= 1.1


def test_direct_dft_form_equals_the_fft_form():
    """The transform pair written out as sums (2048 points) gives what the library FFT gives."""
    rng = np.random.default_rng(9)
    x = rng.standard_normal(1300)
    for alpha in (0.8, 1.2):
        a = V.vtlp_resynth(x, alpha, method="dft")
        b = V.vtlp_resynth(x, alpha, method="fft")
        np.testing.assert_allclose(a, b, atol=1e-11)
    # the sums themselves: a unit impulse at n0 has the spectrum exp(-2 pi i k n0 / K), and comes back
    g = np.zeros(2048); g[5] = 1.0
    X = V.dft_half(g)
    np.testing.assert_allclose(X, np.exp(-2j * np.pi * np.arange(1025) * 5 / 2048), atol=1e-12)
    np.testing.assert_allclose(V.idft_real(X, 2048), g, atol=1e-12)
