"""Seeded random sweeps of small cases through every entry point, against the oracle.

Each sweep draws a few dozen configurations around the sizes where the kernels change behaviour (block and
window multiples, one-sample utterances, empty ones, rooms of odd shapes) and holds every one of them to
the same bars as the fixed cases."""
import numpy as np
import pytest

from oracle import aug_oracle as O
from oracle import vtlp_resynth_oracle as V
from paper_1912_11040_amd import workloads as W
from tests.parity import FEAT_TOL, GAIN_TOL, RIR_TOL, WAVE_TOL, dev, feat_err, rir_err, wave_err

pytestmark = pytest.mark.gpu
FS, C = 16000.0, 343.0


@pytest.fixture(scope="module")
def aug():
    from paper_1912_11040_amd.binding import Augmenter
    a = Augmenter(0)
    yield a
    a.close()


def test_rooms_of_odd_shapes(aug):
    import torch
    rng = np.random.default_rng(101)
    for case in range(40):
        n_rir = int(rng.integers(1, 4))
        L = int(rng.choice([1, 2, 63, 64, 65, 500, 1500]))
        kind = str(rng.choice(["normal", "small", "flat", "narrow", "cube", "wall"]))
        geom = np.zeros((n_rir, 10), np.float32)
        for r in range(n_rir):
            if kind == "small":
                dims = rng.uniform(0.5, 1.5, 3)
            elif kind == "flat":
                dims = np.array([rng.uniform(3, 8), rng.uniform(3, 8), rng.uniform(0.12, 0.4)])
            elif kind == "narrow":
                dims = np.array([rng.uniform(0.12, 0.4), rng.uniform(3, 8), rng.uniform(2, 4)])
            elif kind == "cube":
                dims = np.full(3, float(rng.choice([1.0, 2.0, 4.0])))
            else:
                dims = rng.uniform([3, 3, 2.5], [10, 8, 4])
            margin = 0.01 if kind == "wall" else 0.05
            src = rng.uniform(margin, 1 - margin, 3) * dims
            mic = rng.uniform(margin, 1 - margin, 3) * dims
            if kind == "cube":                       # lattice positions: many images at exactly equal distances
                src = dims * rng.choice([0.25, 0.5, 0.75], 3)
                mic = dims * rng.choice([0.25, 0.5, 0.75], 3)
            if np.linalg.norm(src - mic) < 0.05:
                mic = np.clip(mic + 0.1, 0.01, dims - 0.01)
            beta = float(rng.choice([0.0, 0.3, 0.7, 0.95, 1.0, rng.uniform(0, 1)]))
            geom[r] = np.concatenate([dims, src, mic, [beta]])
        print(f"case {case}: {kind} rooms, n={n_rir}, L={L}", flush=True)
        h = torch.full((n_rir, L), float("nan"), dtype=torch.float32, device="cuda")
        cnt = torch.full((n_rir, L), -7, dtype=torch.int32, device="cuda")
        aug.aug_rir_batch(dev(geom), L, FS, C, h, cnt)
        torch.cuda.synchronize()
        h_ref, c_ref = O.rir_batch(geom, L, FS, C)
        np.testing.assert_array_equal(cnt.cpu().numpy(), c_ref)
        assert rir_err(h.cpu().numpy(), h_ref) <= RIR_TOL


def test_convolution_around_block_multiples(aug):
    import torch
    rng = np.random.default_rng(102)
    for case in range(30):
        L = int(rng.choice([1, 2, 100, 1023, 1024, 1025, 2048, 3000, 4097, 8192, 8193, 9000]))
        N = 1024
        while N < L and N < 16384:
            N *= 2
        n_utt, n_noise = int(rng.integers(1, 4)), int(rng.integers(0, 3))
        lens = [int(max(0, rng.choice([0, 1, N - 1, N, N + 1, 2 * N, 2 * N + 1, 777]) + rng.choice([0, 0, 1])))
                for _ in range(n_utt)]
        offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        total = int(offsets[-1])
        speech = rng.standard_normal(total).astype(np.float32)
        noise = rng.standard_normal((n_noise, total)).astype(np.float32) if n_noise else None
        rir = (rng.standard_normal((n_utt, 1 + n_noise, L)) * np.exp(-np.arange(L) / (0.25 * L + 1.0))).astype(np.float32)
        delay = int(rng.integers(0, min(L, 300)))
        rir[:, :, :delay] = 0.0
        rir[:, :, delay] += 1.0
        snr = rng.uniform(-5, 30, (n_utt, n_noise)).astype(np.float32) if n_noise else None
        print(f"case {case}: L={L} (blocks of {N}), lens={lens}, n_noise={n_noise}, first tap {delay}", flush=True)
        mixed = torch.full((max(total, 1),), float("nan"), dtype=torch.float32, device="cuda")
        gains = torch.full((n_utt, max(n_noise, 1)), float("nan"), dtype=torch.float32, device="cuda")
        aug.aug_convolve_mix_batch(offsets, dev(speech), None if noise is None else dev(noise), dev(rir), L,
                                   None if snr is None else dev(snr), mixed[:total], gains if n_noise else None)
        torch.cuda.synchronize()
        # the direct sums give exact zeros where nothing has arrived yet, as the library must
        ref, g_ref = O.convolve_mix_batch(offsets, speech, noise, rir.astype(np.float64), snr, "direct")
        got = mixed[:total].cpu().numpy()
        assert not np.isnan(got).any()
        assert wave_err(got, ref, offsets, silent_scale=speech) <= WAVE_TOL
        for u in range(n_utt):
            assert np.all(got[offsets[u]:offsets[u] + min(delay, lens[u])] == 0.0)
        if n_noise and total:
            np.testing.assert_allclose(gains.cpu().numpy()[:, :n_noise], g_ref, rtol=GAIN_TOL)


def test_front_end_and_waveform_vtlp_around_window_multiples(aug):
    import torch
    rng = np.random.default_rng(103)
    for case in range(40):
        n_utt = int(rng.integers(1, 7))
        lens = rng.choice([0, 1, 2, 159, 160, 399, 400, 401, 559, 560, 561, 799, 800, 801, 1199, 1200, 1201, 3000, 6401], n_utt)
        offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        total = int(offsets[-1])
        x = (rng.standard_normal(total) * rng.choice([1e-3, 1.0, 30.0])).astype(np.float32)
        alpha = rng.uniform(0.8, 1.2, n_utt).astype(np.float32)
        if rng.random() < 0.2:
            alpha[rng.integers(0, n_utt)] = 1.0
        kind = str(rng.choice(["power", "log", "mfcc"]))
        n_mel = int(rng.choice([13, 40, 64, 128]))
        fe = W.FrontendConfig(n_mel=n_mel, feature=kind, n_ceps=int(rng.integers(1, min(n_mel, 30) + 1)),
                              log_floor=float(rng.choice([1e-10, 1e-4])))
        print(f"case {case}: lens={lens.tolist()}, {kind}, n_mel={n_mel}", flush=True)
        if total > 0:
            y = torch.full((total,), float("nan"), dtype=torch.float32, device="cuda")
            aug.aug_vtlp_resynth_batch(offsets, dev(x), dev(alpha), y)
            torch.cuda.synchronize()
            ref = V.vtlp_resynth_batch(offsets, x, alpha)
            assert wave_err(y.cpu().numpy(), ref, offsets, silent_scale=x) <= WAVE_TOL
        frames = np.array([O.frame_count(int(n), 400, 160) for n in lens])
        spare = rng.integers(0, 3, n_utt) * int(rng.random() < 0.5)
        foff = np.concatenate([[0], np.cumsum(frames + spare)]).astype(np.int64)
        feats = torch.full((int(foff[-1]), fe.feature_dim), float("nan"), dtype=torch.float32, device="cuda")
        aug.aug_vtlp_mel_batch(offsets, dev(x), dev(alpha), fe, foff, feats)
        torch.cuda.synchronize()
        got = feats.cpu().numpy()
        ref = O.vtlp_mel_batch(offsets, x, alpha, fe)
        roff = np.concatenate([[0], np.cumsum(frames)])
        assert not np.isnan(got).any()
        for u in range(n_utt):
            g, r = got[foff[u]:foff[u] + frames[u]], ref[roff[u]:roff[u + 1]]
            if frames[u]:
                assert feat_err(g, r) <= FEAT_TOL
            assert np.all(got[foff[u] + frames[u]:foff[u + 1]] == 0.0)          # spare rows are zeroed
