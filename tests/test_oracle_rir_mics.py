"""Pins for the several-microphones form of the image-method oracle.  CPU only.

The one-microphone oracle is pinned on its own (closed forms, hand geometry,
brute force); here the shared-image-list form is tied to it and to what the
geometry of a microphone pair fixes."""
import math

import numpy as np
import pytest

from oracle import aug_oracle as O

FS, C = 16000.0, 343.0


def _geom(room, src, mic, beta):
    return np.array(list(room) + list(src) + list(mic) + [beta], dtype=np.float32)


def test_each_microphone_equals_the_one_microphone_response():
    # the shared list of images must give every microphone what it gets on its own
    room, src = (5.2, 4.1, 2.9), (1.3, 2.2, 1.1)
    mics = np.array([[3.9, 1.0, 1.6], [3.9, 1.068, 1.6], [0.4, 3.7, 2.5]], np.float32)
    g = _geom(room, src, (9, 9, 9), 0.83)          # the row's own microphone columns are not used
    h, cnt = O.rir_mics_single(g, mics, 1800, FS, C)
    assert h.shape == (3, 1800) and cnt.shape == (3, 1800) and cnt.dtype == np.int32
    for m in range(3):
        h1, c1 = O.rir_single(_geom(room, src, mics[m], 0.83), 1800, FS, C)
        np.testing.assert_array_equal(cnt[m], c1)
        np.testing.assert_allclose(h[m], h1, rtol=1e-14, atol=0)
    # and they do differ from one another
    assert not np.array_equal(cnt[0], cnt[1])


def test_direct_paths_of_a_pair_by_hand():
    # beta = 0: one impulse per microphone, 1/(4 pi r_m) at the sample nearest r_m fs / c;
    # a pair 6.8 cm apart along the line to the source differs by 0.068 fs / c = 3.17 samples
    room, src = (6.0, 5.0, 3.0), (1.0, 2.5, 1.5)
    mics = np.array([[4.0, 2.5, 1.5], [4.068, 2.5, 1.5]], np.float32)
    h, cnt = O.rir_mics_single(_geom(room, src, (0, 0, 0), 0.0), mics, 1024, FS, C)
    taps = []
    for m in range(2):
        r = float(np.float64(mics[m, 0]) - 1.0)
        n0 = int(math.floor(r * FS / C + 0.5))
        assert np.flatnonzero(h[m]).tolist() == [n0]
        assert h[m, n0] == pytest.approx(1.0 / (4 * math.pi * r), rel=1e-12)
        taps.append(n0)
    assert taps == [140, 143]


def test_mirrored_pair_hears_a_centred_source_alike():
    # source on the plane x = Lx / 2, microphones mirror images of each other in that plane:
    # the room is symmetric about it, so the two responses are the same (dyadic coordinates keep
    # the mirrored distances bit-identical)
    room, src = (4.0, 3.5, 2.75), (2.0, 1.25, 1.5)
    mics = np.array([[0.75, 2.5, 1.0], [3.25, 2.5, 1.0]], np.float32)
    h, cnt = O.rir_mics_single(_geom(room, src, (1, 1, 1), 0.7), mics, 1200, FS, C)
    np.testing.assert_array_equal(cnt[0], cnt[1])
    np.testing.assert_allclose(h[0], h[1], rtol=1e-12, atol=0)
    # moving one of them off the mirror position breaks it
    mics[1, 0] = 3.0
    h, cnt = O.rir_mics_single(_geom(room, src, (1, 1, 1), 0.7), mics, 1200, FS, C)
    assert not np.array_equal(cnt[0], cnt[1])


def test_far_microphone_still_gets_every_image():
    # microphones in opposite corners: the per-axis bound on the image list must hold for both;
    # compare the image count below L with the volume of the ball of that radius (8 images per room cell)
    room, src = (3.0, 2.5, 2.4), (0.2, 0.2, 0.2)
    mics = np.array([[0.3, 0.3, 0.3], [2.9, 2.4, 2.3]], np.float32)
    L = 3000
    _, cnt = O.rir_mics_single(_geom(room, src, (1, 1, 1), 0.5), mics, L, FS, C)
    radius = L * C / FS
    expect = (4.0 / 3.0) * math.pi * radius ** 3 / (3.0 * 2.5 * 2.4)
    for m in range(2):
        assert cnt[m].sum() == pytest.approx(expect, rel=0.01)


def test_batch_layout():
    rng = np.random.default_rng(3)
    geom = np.stack([_geom((5, 4, 3), (1, 1, 1), (0, 0, 0), 0.6), _geom((3, 3, 2.5), (2, 1, 1.5), (0, 0, 0), 0.9)])
    mics = rng.uniform(0.3, 2.2, (2, 2, 3)).astype(np.float32)
    h, cnt = O.rir_mics_batch(geom, mics, 700, FS, C)
    assert h.shape == (2, 2, 700) and h.dtype == np.float64 and cnt.dtype == np.int32
    for r in range(2):
        for m in range(2):
            g = geom[r].copy()
            g[6:9] = mics[r, m]
            h1, c1 = O.rir_single(g, 700, FS, C)
            np.testing.assert_array_equal(cnt[r, m], c1)
            np.testing.assert_allclose(h[r, m], h1, rtol=1e-14, atol=0)
