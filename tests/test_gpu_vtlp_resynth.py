"""aug_vtlp_resynth_batch (waveform VTLP, Sec. 2.3 / Eq. (1)) against its fp64 oracle."""
import numpy as np
import pytest

from oracle import vtlp_resynth_oracle as V
from paper_1912_11040_amd import workloads as W
from tests.parity import WAVE_TOL, dev, wave_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def aug():
    from paper_1912_11040_amd.binding import Augmenter
    a = Augmenter(0)
    yield a
    a.close()


def _run(aug, offsets, wave, alpha):
    import torch
    out = torch.full((int(offsets[-1]),), float("nan"), dtype=torch.float32, device="cuda")
    aug.aug_vtlp_resynth_batch(offsets, dev(wave), dev(alpha), out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _check(aug, offsets, wave, alpha):
    got = _run(aug, offsets, wave, alpha)
    ref = V.vtlp_resynth_batch(offsets, wave, alpha)
    assert not np.isnan(got).any()
    err = wave_err(got, ref, offsets)
    print(f"  waveform max error / RMS = {err:.2e} (tolerance {WAVE_TOL:.0e})", flush=True)
    assert err <= WAVE_TOL
    return got, ref


def test_ragged_lengths_and_warp_factors(aug):
    rng = np.random.default_rng(21)
    lens = [0, 1, 399, 400, 401, 800, 1000, 6399, 6400, 6401, 12345, 40000]
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    wave = rng.standard_normal(int(offsets[-1])).astype(np.float32)
    alpha = rng.uniform(0.8, 1.2, len(lens)).astype(np.float32)
    alpha[3], alpha[6], alpha[10] = 0.8, 1.2, 1.0
    print("case: ragged lengths across frame-group boundaries, white noise", flush=True)
    got, _ = _check(aug, offsets, wave, alpha)
    # alpha = 1 returns the input
    a, b = offsets[10], offsets[11]
    assert np.max(np.abs(got[a:b] - wave[a:b])) <= 1e-5 * np.sqrt(np.mean(wave[a:b] ** 2.0)) * 10


def test_tiny_speech(aug):
    w = W.tiny()
    print("case: tiny workload speech", flush=True)
    _check(aug, w.offsets, w.speech, w.alpha)


def test_pure_tone_lands_where_eq1_says(aug):
    from oracle import aug_oracle as O
    fs, n, f0, alpha = 16000.0, 16000, 1000.0, 0.8
    x = np.cos(2.0 * np.pi * f0 / fs * np.arange(n)).astype(np.float32)
    y = _run(aug, np.array([0, n], np.int64), x, np.array([alpha], np.float32)).astype(np.float64)
    f_want = float(O.bilinear_warp(2.0 * np.pi * f0 / fs, alpha)) * fs / (2.0 * np.pi)
    spec = np.abs(np.fft.rfft(y[4000:12192] * np.hanning(8192), 65536)) ** 2
    freqs = np.arange(spec.shape[0]) * fs / 65536
    assert abs(freqs[np.argmax(spec)] - f_want) <= 21.0


def test_varlen_full_size_sampled(aug):
    # the speech stream of the benchmark's workload in one call; the oracle checks sampled utterances
    w = W.varlen()
    print(f"case: varlen speech, {w.n_utt} utterances, {w.total} samples", flush=True)
    got = _run(aug, w.offsets, w.speech, w.alpha)
    assert not np.isnan(got).any()
    lens = w.lengths()
    rng = np.random.default_rng(0)
    for u in [int(np.argmin(lens)), int(np.argmax(lens)), int(rng.integers(0, w.n_utt)), 0, w.n_utt - 1]:
        a, b = int(w.offsets[u]), int(w.offsets[u + 1])
        ref = V.vtlp_resynth(w.speech[a:b], w.alpha[u])
        err = wave_err(got[a:b], ref, np.array([0, b - a]))
        print(f"  utterance {u}: {b - a} samples, error {err:.2e}", flush=True)
        assert err <= WAVE_TOL


def test_argument_errors():
    import torch
    from paper_1912_11040_amd.binding import AugError, Augmenter
    # the binding's own element-count checks are off: this test is about what the library itself refuses
    aug = Augmenter(0, check_sizes=False)
    off = np.array([0, 1000], np.int64)
    x = torch.zeros(1000, device="cuda")
    y = torch.zeros(1000, device="cuda")
    a = torch.ones(1, device="cuda")
    with pytest.raises(AugError) as e:
        aug.aug_vtlp_resynth_batch(off, x, a, y, win=400, hop=200, nfft=1024)
    assert e.value.code == -2
    with pytest.raises(AugError) as e:
        aug.aug_vtlp_resynth_batch(off, x, a, x)
    assert e.value.code == -1
    with pytest.raises(AugError) as e:
        aug.aug_vtlp_resynth_batch(off, x, None, y)
    assert e.value.code == -1
    aug.aug_vtlp_resynth_batch(np.array([0], np.int64), None if False else x, a, y)   # empty batch is fine
    aug.close()
