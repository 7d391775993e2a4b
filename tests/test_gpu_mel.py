"""aug_vtlp_mel_batch against the oracle's DFT-matrix front end."""
import numpy as np
import pytest

from oracle import aug_oracle as O
from paper_1912_11040_amd import workloads as W
from tests.parity import FEAT_TOL, DeviceWorkload, dev, feat_err

pytestmark = pytest.mark.gpu
FE = W.FrontendConfig()


@pytest.fixture(scope="module")
def aug():
    from paper_1912_11040_amd.binding import Augmenter
    a = Augmenter(0)
    yield a
    a.close()


def _run(aug, offsets, wave, alpha, fe=FE):
    import torch
    n = np.diff(offsets)
    t = np.where(n >= fe.win, 1 + (n - fe.win) // fe.hop, 0)
    foff = np.concatenate([[0], np.cumsum(t)]).astype(np.int64)
    feats = torch.full((int(foff[-1]), fe.feature_dim), float("nan"), dtype=torch.float32, device="cuda")
    aug.aug_vtlp_mel_batch(offsets, dev(wave), dev(alpha), fe, foff, feats)
    torch.cuda.synchronize()
    return feats.cpu().numpy()


def test_tiny_speech(aug):
    w = W.tiny()
    print("case: tiny speech, 8 x 98 frames", flush=True)
    f = _run(aug, w.offsets, w.speech, w.alpha)
    ref = O.vtlp_mel_batch(w.offsets, w.speech, w.alpha, FE)
    assert f.shape == ref.shape == (784, 40)
    assert feat_err(f, ref) <= FEAT_TOL


def test_features_config_subset(aug):
    w = W.features_only(n_utt=12, seconds=8.0)
    print("case: features-only, 12 x 798 frames", flush=True)
    f = _run(aug, w.offsets, w.speech, w.alpha)
    ref = O.vtlp_mel_batch(w.offsets, w.speech, w.alpha, FE)
    assert feat_err(f, ref) <= FEAT_TOL


def test_features_config_full_size_sampled(aug):
    # the whole features-only configuration in one call, as the benchmark launches it with
    # --workload features; the oracle checks sampled utterances frame by frame
    w = W.features_only()
    print(f"case: features config, {w.n_utt} utterances, {w.total} samples", flush=True)
    f = _run(aug, w.offsets, w.speech, w.alpha)
    assert f.shape == (w.n_utt * 798, 40) and not np.isnan(f).any()
    foff = w.frame_offsets()
    for u in [0, 1, 2047, w.n_utt - 1, int(np.random.default_rng(2).integers(0, w.n_utt))]:
        a, b = int(w.offsets[u]), int(w.offsets[u + 1])
        ref = O.vtlp_mel_batch(np.array([0, b - a]), w.speech[a:b], w.alpha[u:u + 1], FE)
        err = feat_err(f[foff[u]:foff[u + 1]], ref)
        print(f"  utterance {u}: feature error {err:.2e}", flush=True)
        assert err <= FEAT_TOL


def test_large_batch_of_mixed_lengths_with_spare_rows(aug):
    # Many utterances of very different lengths in one call: enough output rows that the library gives its
    # work groups more than the smallest share of rows, so an utterance's rows are divided among several
    # groups of a size that depends on the utterance (none, one, a few, dozens of groups), with spare rows
    # behind some utterances.  Sampled utterances are checked frame by frame, spare rows must be zero.
    import torch
    rng = np.random.default_rng(11)
    n_utt = 3000
    lens = rng.integers(0, 6 * 16000, n_utt)
    lens[:6] = [0, 399, 400, 401, 560, 95999]
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    wave = rng.standard_normal(int(offsets[-1]), dtype=np.float32)
    alpha = rng.uniform(0.8, 1.2, n_utt).astype(np.float32)
    frames = np.where(lens >= FE.win, 1 + (lens - FE.win) // FE.hop, 0)
    spare = rng.integers(0, 3, n_utt) * (rng.random(n_utt) < 0.3)
    foff = np.concatenate([[0], np.cumsum(frames + spare)]).astype(np.int64)
    print(f"case: {n_utt} utterances of 0-6 s, {int(foff[-1])} output rows", flush=True)
    assert foff[-1] > 8 * 3 * 256 * 80          # more than the smallest group size can cover with eight rounds
    feats = torch.full((int(foff[-1]), FE.feature_dim), float("nan"), dtype=torch.float32, device="cuda")
    aug.aug_vtlp_mel_batch(offsets, dev(wave), dev(alpha), FE, foff, feats)
    torch.cuda.synchronize()
    f = feats.cpu().numpy()
    assert not np.isnan(f).any()
    picks = list(range(6)) + [int(np.argmax(lens))] + [int(u) for u in rng.integers(0, n_utt, 9)]
    for u in picks:
        a, b = int(offsets[u]), int(offsets[u + 1])
        ref = O.vtlp_mel_batch(np.array([0, b - a]), wave[a:b], alpha[u:u + 1], FE, method="fft")
        got = f[foff[u]:foff[u] + frames[u]]
        assert got.shape == ref.shape
        if frames[u]:
            assert feat_err(got, ref) <= FEAT_TOL, u
        assert not f[foff[u] + frames[u]:foff[u + 1]].any()          # spare rows


def test_ragged_short_and_empty_utterances(aug):
    rng = np.random.default_rng(0)
    lens = [0, 399, 400, 559, 560, 12345, 1, 400 + 160 * 63, 400 + 160 * 64, 400 + 160 * 65]
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    x = rng.standard_normal(int(offsets[-1])).astype(np.float32)
    alpha = rng.uniform(0.8, 1.2, len(lens)).astype(np.float32)
    print("case: ragged lengths", flush=True)
    f = _run(aug, offsets, x, alpha)
    ref = O.vtlp_mel_batch(offsets, x, alpha, FE)
    assert f.shape == ref.shape
    assert not np.isnan(f).any()
    assert feat_err(f, ref) <= FEAT_TOL


@pytest.mark.parametrize("alpha", [0.8, 1.0, 1.2])
def test_pure_tone_and_alpha_extremes(aug, alpha):
    x = np.cos(2 * np.pi * 64 * np.arange(4000) / 512).astype(np.float32)
    offsets = np.array([0, 4000], np.int64)
    a = np.array([alpha], np.float32)
    f = _run(aug, offsets, x, a)
    ref = O.vtlp_mel_batch(offsets, x, a, FE)
    assert feat_err(f, ref) <= FEAT_TOL
    print(f"feature error = {feat_err(f, ref):.2e}", flush=True)
    assert (np.argmax(f, axis=1) == np.argmax(ref, axis=1)).all()


def test_silence_gives_zero_and_loud_input_is_not_clipped(aug):
    offsets = np.array([0, 2000, 4000], np.int64)
    rng = np.random.default_rng(1)
    x = np.concatenate([np.zeros(2000), 3e4 * rng.standard_normal(2000)]).astype(np.float32)
    a = np.array([0.9, 1.1], np.float32)
    f = _run(aug, offsets, x, a)
    ref = O.vtlp_mel_batch(offsets, x, a, FE)
    np.testing.assert_array_equal(f[:11], 0.0)
    assert f.max() > 3.0
    assert feat_err(f, ref) <= FEAT_TOL


def test_other_mel_counts_and_band(aug):
    import dataclasses
    fe = dataclasses.replace(FE, n_mel=23, f_lo=100.0, f_hi=7000.0, power=0.1)
    w = W.tiny(n_utt=2)
    f = _run(aug, w.offsets, w.speech, w.alpha, fe)
    ref = O.vtlp_mel_batch(w.offsets, w.speech, w.alpha, fe)
    assert f.shape == ref.shape == (196, 23)
    assert feat_err(f, ref) <= FEAT_TOL


def test_padded_batch_layout(aug):
    # frame_offsets[u] = u * Tmax: every utterance owns Tmax rows, the ones past its frames come back zero
    import torch
    from paper_1912_11040_amd.binding import AugError
    rng = np.random.default_rng(31)
    lens = [5000, 0, 399, 16000, 400, 12001, 27000]
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    x = rng.standard_normal(int(offsets[-1])).astype(np.float32)
    alpha = rng.uniform(0.8, 1.2, len(lens)).astype(np.float32)
    t = np.array([O.frame_count(n, FE.win, FE.hop) for n in lens])
    t_max = int(t.max()) + 3
    foff = (np.arange(len(lens) + 1) * t_max).astype(np.int64)
    feats = torch.full((len(lens), t_max, FE.n_mel), float("nan"), dtype=torch.float32, device="cuda")
    aug.aug_vtlp_mel_batch(offsets, dev(x), dev(alpha), FE, foff, feats)
    torch.cuda.synchronize()
    got = feats.cpu().numpy()
    ref = O.vtlp_mel_batch(offsets, x, alpha, FE)
    packed = np.concatenate([[0], np.cumsum(t)])
    for u in range(len(lens)):
        assert np.all(got[u, t[u]:] == 0.0)
        if t[u]:
            assert feat_err(got[u, :t[u]], ref[packed[u]:packed[u + 1]]) <= FEAT_TOL
    # fewer rows than frames is an error
    short = foff.copy()
    short[4:] -= t_max - int(t[3]) + 1
    with pytest.raises(AugError) as e:
        aug.aug_vtlp_mel_batch(offsets, dev(x), dev(alpha), FE, short, feats)
    assert e.value.code == -1


@pytest.mark.parametrize("feature,n_ceps", [("log", 0), ("mfcc", 13), ("mfcc", 40), ("mfcc", 1)])
def test_log_mel_and_mfcc(aug, feature, n_ceps):
    # the conventional features that Sec. 2.3 names beside the power law: other epilogues of the same energies
    import dataclasses
    fe = dataclasses.replace(FE, feature=feature, n_ceps=n_ceps or 13, log_floor=1e-8)
    rng = np.random.default_rng(41)
    lens = [4000, 0, 399, 16000, 560]
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    x = rng.standard_normal(int(offsets[-1])).astype(np.float32)
    x[offsets[3] + 3000:offsets[3] + 9000] = 0.0            # a silent stretch meets the floor
    alpha = rng.uniform(0.8, 1.2, len(lens)).astype(np.float32)
    print(f"case: feature={feature} n_ceps={n_ceps}", flush=True)
    f = _run(aug, offsets, x, alpha, fe)
    ref = O.vtlp_mel_batch(offsets, x, alpha, fe)
    assert f.shape == ref.shape and f.shape[1] == (40 if feature == "log" else n_ceps)
    err = feat_err(f, ref)
    print(f"  feature error {err:.2e}", flush=True)
    assert err <= FEAT_TOL


def test_most_mel_channels_the_interface_takes(aug):
    import dataclasses
    fe = dataclasses.replace(FE, n_mel=128)
    w = W.tiny(n_utt=3)
    alpha = np.array([0.8, 1.0, 1.2], np.float32)
    f = _run(aug, w.offsets, w.speech, alpha, fe)
    ref = O.vtlp_mel_batch(w.offsets, w.speech, alpha, fe)
    assert f.shape == ref.shape and f.shape[1] == 128
    assert feat_err(f, ref) <= FEAT_TOL


@pytest.mark.parametrize("win,hop", [(320, 128), (400, 161), (512, 256), (33, 7)])
def test_other_window_and_hop(aug, win, hop):
    import dataclasses
    fe = dataclasses.replace(FE, win=win, hop=hop)
    rng = np.random.default_rng(win + hop)
    lens = [3001, 0, 2000, win, win - 1, 4097]
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    x = rng.standard_normal(int(offsets[-1])).astype(np.float32)
    alpha = rng.uniform(0.8, 1.2, len(lens)).astype(np.float32)
    print(f"case: win={win} hop={hop}", flush=True)
    f = _run(aug, offsets, x, alpha, fe)
    ref = O.vtlp_mel_batch(offsets, x, alpha, fe)
    assert f.shape == ref.shape and f.shape[0] > 0
    assert feat_err(f, ref) <= FEAT_TOL
