"""Pin for the oracle's end-to-end composition (simulator, then features: Sec. 2.3).  CPU only.

With reflection coefficient 0 every response is the direct path alone, one impulse 1/(4 pi r) at
delay floor(r fs / c + 1/2), so the whole chain has a closed form that needs no convolution code:

    mixture[n] = a_0 x_0[n - n_0] + sum_j g_j a_j x_j[n - n_j],
    g_j = sqrt(E_0 / (E_j 10^(snr_j / 10))),  E_j = a_j^2 sum_{n < N - n_j} x_j[n]^2,

with distances, delays, amplitudes and energies worked out below from the room rows by hand.  Rooms,
source positions, lengths, SNRs and warp factors all differ between utterances and sources, so that any
mix-up of which row, which column or which signal goes where changes the result.  The last test plants
such mix-ups in copies of the composition and checks that the pin rejects every one of them.
"""
import math

import numpy as np
import pytest

from oracle import aug_oracle as O
from paper_1912_11040_amd.workloads import FrontendConfig

FS, C = 16000.0, 343.0
RIR_LEN = 600
FE = FrontendConfig()
_FRONT_END = O.vtlp_mel_batch        # the pinned front end, bound before any test patches the module


def _case():
    rng = np.random.default_rng(11)
    lengths = np.array([2100, 1500, 2750], dtype=np.int64)
    offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    total = int(offsets[-1])
    n_utt, n_noise = 3, 2
    t = np.arange(total)
    # three signals with very different spectra: a swap of any two changes the features
    speech = (np.sin(2 * np.pi * 700.0 * t / FS) * (1.0 + 0.3 * rng.standard_normal(total))).astype(np.float32)
    noise = np.stack([
        0.5 * rng.standard_normal(total),
        np.sin(2 * np.pi * 3100.0 * t / FS) + 0.05 * rng.standard_normal(total),
    ]).astype(np.float32)
    # rows [Lx,Ly,Lz, sx,sy,sz, mx,my,mz, beta]; beta = 0; distances all different
    geom = np.zeros((n_utt, 1 + n_noise, 10), dtype=np.float32)
    rooms = [(6.0, 5.0, 3.0), (8.0, 4.0, 2.8), (4.5, 7.0, 3.5)]
    mics = [(1.0, 1.0, 1.0), (2.0, 1.5, 1.2), (1.5, 2.0, 1.4)]
    srcs = [[(2.0, 1.0, 1.0), (1.0, 4.0, 1.0), (5.0, 4.0, 2.0)],          # 1 m, 3 m, 5.099 m
            [(2.0, 3.5, 1.2), (6.0, 1.5, 1.2), (7.0, 3.0, 2.2)],          # 2 m, 4 m, 5.315 m
            [(1.5, 2.0, 2.9), (4.0, 6.0, 1.4), (3.0, 3.0, 3.0)]]          # 1.5 m, 4.717 m, 2.417 m
    for u in range(n_utt):
        for j in range(1 + n_noise):
            geom[u, j] = (*rooms[u], *srcs[u][j], *mics[u], 0.0)
    snr_db = np.array([[3.0, 12.0], [20.0, 0.0], [7.5, 15.0]], dtype=np.float32)
    alpha = np.array([0.85, 1.0, 1.15], dtype=np.float32)
    return offsets, speech, noise, geom, snr_db, alpha


def _by_hand(offsets, speech, noise, geom, snr_db):
    """Mixture and gains from distances, delays and energies computed directly from the rows."""
    n_utt = len(offsets) - 1
    n_noise = noise.shape[0]
    mixed = np.zeros(int(offsets[-1]))
    gains = np.zeros((n_utt, n_noise))
    taps = np.zeros((n_utt, 1 + n_noise), dtype=np.int64)
    amps = np.zeros((n_utt, 1 + n_noise))
    for u in range(n_utt):
        a, b = int(offsets[u]), int(offsets[u + 1])
        shifted = []
        for j in range(1 + n_noise):
            row = geom[u, j].astype(np.float64)
            r = math.sqrt(sum((row[3 + i] - row[6 + i]) ** 2 for i in range(3)))
            delay = int(math.floor(r * FS / C + 0.5))
            amp = 1.0 / (4.0 * math.pi * r)
            x = (speech if j == 0 else noise[j - 1])[a:b].astype(np.float64)
            y = np.zeros(b - a)
            y[delay:] = amp * x[: b - a - delay]
            shifted.append(y)
            taps[u, j], amps[u, j] = delay, amp
        e = [float(np.sum(y * y)) for y in shifted]
        z = shifted[0].copy()
        for j in range(1, 1 + n_noise):
            gains[u, j - 1] = math.sqrt(e[0] / (e[j] * 10.0 ** (float(snr_db[u, j - 1]) / 10.0)))
            z += gains[u, j - 1] * shifted[j]
        mixed[a:b] = z
    return mixed, gains, taps, amps


def _check(pipeline):
    """Raises AssertionError unless `pipeline` reproduces the closed form."""
    offsets, speech, noise, geom, snr_db, alpha = _case()
    out = pipeline(offsets, speech, noise, geom, RIR_LEN, FS, C, snr_db, alpha, FE)
    mixed, gains, taps, amps = _by_hand(offsets, speech, noise, geom, snr_db)
    n_utt, n_src = taps.shape
    # responses: one tap each, where and as large as the hand geometry says, in [utterance][source] order
    assert out["rir"].shape == (n_utt, n_src, RIR_LEN)
    for u in range(n_utt):
        for j in range(n_src):
            h = out["rir"][u, j]
            assert np.count_nonzero(h) == 1
            assert int(np.argmax(h)) == taps[u, j]
            assert h[taps[u, j]] == pytest.approx(amps[u, j], rel=1e-12)
            # images are counted whatever their amplitude; the direct path is the nearest of them
            cnt = out["tap_count"][u, j]
            assert cnt[taps[u, j]] >= 1 and not cnt[: taps[u, j]].any()
    np.testing.assert_allclose(out["gains"], gains, rtol=1e-10)
    np.testing.assert_allclose(out["mixed"], mixed, rtol=0, atol=1e-12 * np.max(np.abs(mixed)))
    # the hand delays really differ, so a swap of sources cannot go unnoticed
    assert all(len(set(taps[u])) == n_src for u in range(n_utt))
    # features are those of the mixture (not of the clean speech), each utterance with its own warp factor
    feats = _FRONT_END(offsets, mixed, alpha, FE)
    assert out["feats"].shape == feats.shape
    np.testing.assert_allclose(out["feats"], feats, rtol=1e-9)
    # and the measured SNR of what was mixed is the target
    for u in range(n_utt):
        a, b = int(offsets[u]), int(offsets[u + 1])
        for j in range(1, n_src):
            x = noise[j - 1][a:b].astype(np.float64)
            yj = np.zeros(b - a)
            yj[taps[u, j]:] = amps[u, j] * x[: b - a - taps[u, j]]
            s = speech[a:b].astype(np.float64)
            y0 = np.zeros(b - a)
            y0[taps[u, 0]:] = amps[u, 0] * s[: b - a - taps[u, 0]]
            got = 10.0 * math.log10(np.sum(y0 ** 2) / np.sum((out["gains"][u, j - 1] * yj) ** 2))
            assert got == pytest.approx(float(snr_db[u, j - 1]), abs=1e-8)


def test_pipeline_matches_closed_form_direct_path_rooms():
    _check(O.pipeline_batch)


def test_pipeline_fft_forms_match_closed_form():
    _check(lambda *a: O.pipeline_batch(*a, conv_method="fft", stft_method="fft"))


def test_features_of_a_mixture_dominated_by_one_tone_peak_in_its_channel():
    """Independent of the oracle's own front end: with the speech 40 dB below a 3100 Hz noise tone at alpha = 1
    the largest feature of every frame sits in the mel channel whose triangle holds 3100 Hz."""
    n = 3200
    t = np.arange(n)
    rng = np.random.default_rng(5)
    speech = (0.1 * rng.standard_normal(n)).astype(np.float32)
    noise = np.sin(2 * np.pi * 3100.0 * t / FS)[None, :].astype(np.float32)
    geom = np.array([[[6, 5, 3, 2, 1, 1, 1, 1, 1, 0], [6, 5, 3, 1, 4, 1, 1, 1, 1, 0]]], dtype=np.float32)
    out = O.pipeline_batch(np.array([0, n]), speech, noise, geom, 300, FS, C,
                           np.array([[-40.0]], np.float32), np.array([1.0], np.float32), FE)
    mel = lambda f: 2595.0 * math.log10(1.0 + f / 700.0)
    step = mel(8000.0) / (FE.n_mel + 1)
    peak_channel = int(round(mel(3100.0) / step)) - 1          # channel m peaks at edge m + 1
    frames = out["feats"][2:]                                   # the tone arrives after 3 m = 140 samples
    assert frames.shape[0] >= 10
    assert np.all(np.argmax(frames, axis=1) == peak_channel)


# ---- planted mistakes: each is a copy of the composition with one mix-up; the pin must reject all ----

def _compose(offsets, speech, noise, geom, rir_len, fs, c, snr_db, alpha, fe, *, geom_order="us", h_order="us",
             swap_snr=False, feats_from="mixed", swap_noise=False, alpha_reversed=False):
    offsets = np.asarray(offsets, dtype=np.int64)
    n_utt = len(offsets) - 1
    geom = np.asarray(geom, dtype=np.float32).reshape(n_utt, -1, 10)
    n_src = geom.shape[1]
    rows = geom if geom_order == "us" else geom.transpose(1, 0, 2)       # "su": sources outermost
    h, cnt = O.rir_batch(rows.reshape(-1, 10), rir_len, fs, c)
    if geom_order == "su":
        h = h.reshape(n_src, n_utt, rir_len).transpose(1, 0, 2)
        cnt = cnt.reshape(n_src, n_utt, rir_len).transpose(1, 0, 2)
    if h_order == "su":                                                  # rows reinterpreted in the wrong order
        h = h.reshape(n_src, n_utt, rir_len).transpose(1, 0, 2)
        cnt = cnt.reshape(n_src, n_utt, rir_len).transpose(1, 0, 2)
    h = np.ascontiguousarray(h).reshape(n_utt, n_src, rir_len)
    cnt = np.ascontiguousarray(cnt).reshape(n_utt, n_src, rir_len)
    if swap_noise:
        noise = noise[::-1]
    snr = np.asarray(snr_db)[:, ::-1] if swap_snr else snr_db
    mixed, gains = O.convolve_mix_batch(offsets, speech, noise, h, snr)
    a = alpha[::-1] if alpha_reversed else alpha
    feats = O.vtlp_mel_batch(offsets, mixed if feats_from == "mixed" else speech, a, fe)
    return dict(rir=h, tap_count=cnt, mixed=mixed, gains=gains, feats=feats)


def test_the_pin_accepts_the_faithful_copy_and_rejects_planted_mistakes():
    _check(_compose)                                             # the copy itself is right ...
    _check(lambda *a: _compose(*a, geom_order="su"))             # ... and so is an equivalent reordering
    mistakes = {
        "responses reshaped in the wrong order": dict(h_order="su"),
        "SNR columns swapped": dict(swap_snr=True),
        "noise sources swapped": dict(swap_noise=True),
        "features taken from the clean speech": dict(feats_from="speech"),
        "warp factors paired with the wrong utterances": dict(alpha_reversed=True),
    }
    for name, kw in mistakes.items():
        with pytest.raises(AssertionError):
            _check(lambda *a, kw=kw: _compose(*a, **kw))
            pytest.fail(f"planted mistake went unnoticed: {name}")


def test_source_rows_swapped_inside_the_oracle_fail_the_pin(monkeypatch):
    """The same mistakes planted in the oracle module itself (its building blocks patched), not in a copy."""
    real_rir_batch = O.rir_batch

    def rows_swapped(geom, rir_len, fs, c):
        g = np.asarray(geom, dtype=np.float32).reshape(-1, 10).copy()
        g[[0, 1]] = g[[1, 0]]                                    # speech and first noise of utterance 0
        return real_rir_batch(g, rir_len, fs, c)

    monkeypatch.setattr(O, "rir_batch", rows_swapped)
    with pytest.raises(AssertionError):
        _check(O.pipeline_batch)
    monkeypatch.setattr(O, "rir_batch", real_rir_batch)

    real_mel = O.vtlp_mel_batch
    monkeypatch.setattr(O, "vtlp_mel_batch", lambda off, wave, alpha, fe, method="dft": real_mel(off, wave, alpha[::-1], fe, method))
    with pytest.raises(AssertionError):
        _check(O.pipeline_batch)
