"""The seeded input generators: shapes, determinism, geometry margins.  CPU only."""
import numpy as np

from paper_1912_11040_amd import workloads as W


def test_tiny_shapes_and_determinism():
    a, b = W.tiny(), W.tiny()
    assert a.n_utt == 8 and a.total == 128000 and a.n_noise == 1 and a.rir_len == 4096
    assert a.speech.dtype == np.float32 and a.noise.shape == (1, 128000)
    assert a.geom.shape == (8, 2, 10) and a.snr_db.shape == (8, 1) and a.alpha.shape == (8,)
    np.testing.assert_array_equal(a.speech, b.speech)
    np.testing.assert_array_equal(a.geom, b.geom)
    np.testing.assert_array_equal(a.geom[:, :, 0:3], np.broadcast_to([5, 4, 3], (8, 2, 3)))
    assert (a.geom[:, :, 9] == np.float32(0.7)).all() and (a.snr_db == 10).all()
    assert a.frame_offsets()[-1] == 8 * 98
    assert not np.array_equal(W.tiny(seed=5).speech, a.speech)


def test_geometry_margins_and_shared_mic():
    w = W.batch(n_utt=16, seconds=0.1)
    g = w.geom.astype(np.float64)
    room, src, mic = g[..., 0:3], g[..., 3:6], g[..., 6:9]
    assert (src >= 0.5 - 1e-6).all() and (src <= room - 0.5 + 1e-6).all()
    assert (mic >= 0.5 - 1e-6).all() and (mic <= room - 0.5 + 1e-6).all()
    assert (np.linalg.norm(src - mic, axis=-1) >= 0.1 - 1e-6).all()
    np.testing.assert_array_equal(g[:, 0, 6:9], g[:, 1, 6:9])
    assert (room[..., 0] >= 3).all() and (room[..., 0] <= 10).all()
    assert (room[..., 2] >= 2.5).all() and (room[..., 2] <= 4).all()
    assert (g[..., 9] >= 0.2).all() and (g[..., 9] <= 0.9).all()
    assert (w.alpha >= 0.8).all() and (w.alpha <= 1.2).all()
    assert (w.snr_db >= 0).all() and (w.snr_db <= 20).all()


def test_varlen_packing_and_slice():
    w = W.varlen(n_utt=6, rir_len=256, min_s=0.05, max_s=0.2)
    n = w.lengths()
    assert (n >= 800).all() and (n <= 3200).all() and w.noise.shape == (3, w.total)
    assert w.offsets[0] == 0 and w.offsets.dtype == np.int64
    s = w.slice([4, 1])
    np.testing.assert_array_equal(s.speech[:n[4]], w.speech[w.offsets[4]:w.offsets[5]])
    np.testing.assert_array_equal(s.noise[2, n[4]:], w.noise[2, w.offsets[1]:w.offsets[2]])
    np.testing.assert_array_equal(s.geom[1], w.geom[1])
    assert s.total == n[4] + n[1]


def test_signals_are_unit_scale_and_coloured():
    rng = np.random.default_rng(0)
    for fn in (W.white_noise, W.pink_noise, W.babble_noise):
        x = fn(rng, 16000).astype(np.float64)
        assert 0.9 < np.sqrt(np.mean(x ** 2)) < 1.1
    p = np.abs(np.fft.rfft(W.pink_noise(rng, 1 << 16).astype(np.float64))) ** 2
    lo, hi = p[200:400].mean(), p[20000:20200].mean()       # ~50-100 Hz vs ~5 kHz
    assert lo > 20 * hi
    s = W.speech_like(rng, 16000).astype(np.float64)
    assert 0.3 < np.sqrt(np.mean(s ** 2)) < 1.0


def test_features_only_has_no_room():
    w = W.features_only(n_utt=3, seconds=0.5)
    assert w.noise is None and w.geom is None and w.n_noise == 0
    assert w.frame_offsets().tolist() == [0, 48, 96, 144]


def test_microphone_arrays():
    w = W.tiny(n_utt=4)
    geom = w.geom.reshape(-1, 10)
    m = W.microphone_arrays(geom, 3, 0.05, seed=2)
    assert m.shape == (len(geom), 3, 3) and m.dtype == np.float32
    np.testing.assert_array_equal(m, W.microphone_arrays(geom, 3, 0.05, seed=2))
    np.testing.assert_allclose(m[:, 1], geom[:, 6:9], atol=1e-6)                 # centred on the row's microphone
    np.testing.assert_allclose(np.linalg.norm(m[:, 2] - m[:, 0], axis=1), 0.10, atol=1e-5)
    assert np.all(m[:, :, 2] == geom[:, None, 8])                                # horizontal
    assert np.all(m > 0.4) and np.all(m < geom[:, None, 0:3] - 0.4)              # still inside the margin
