"""Pins for the image-method RIR oracle: closed forms, hand geometry, an
independent enumeration and counting laws.  CPU only."""
import itertools
import math

import numpy as np
import pytest

from oracle import aug_oracle as O

FS, C = 16000.0, 343.0
K = np.float64(np.float32(FS)) / np.float64(np.float32(C))


def _geom(room, src, mic, beta):
    return np.array(list(room) + list(src) + list(mic) + [beta], dtype=np.float32)


def test_zero_reflection_is_single_impulse():
    # beta = 0 leaves the direct path only: 1/(4 pi r) at the sample nearest r fs / c.
    g = _geom((5, 4, 3), (1.0, 1.5, 1.2), (3.5, 2.0, 1.7), 0.0)
    h, cnt = O.rir_single(g, 2048, FS, C)
    gd = g.astype(np.float64)
    r = math.sqrt(sum((gd[3 + a] - gd[6 + a]) ** 2 for a in range(3)))
    n0 = int(round(r * FS / C))
    assert np.count_nonzero(h) == 1
    assert h[n0] == pytest.approx(1.0 / (4 * math.pi * r), rel=1e-12)
    assert cnt[n0] >= 1
    # every image is still counted, only its amplitude vanishes
    assert cnt.sum() > 1000


def test_first_order_images_by_hand():
    # Mirror the source by hand in each of the six walls; with the response cut
    # just past the farthest of them, d h / d beta at beta = 0 is exactly those six taps.
    room, src, mic = (6.0, 5.0, 3.0), (2.0, 1.5, 1.0), (4.5, 3.0, 2.0)
    mirrors = []
    for a in range(3):
        lo = list(src); lo[a] = -src[a]
        hi = list(src); hi[a] = 2 * room[a] - src[a]
        mirrors += [lo, hi]
    dists = [math.dist(p, mic) for p in mirrors]
    L = int(max(dists) * FS / C) + 3
    eps = 1e-6
    h0, _ = O.rir_single(_geom(room, src, mic, 0.0), L, FS, C)
    h1, _ = O.rir_single(_geom(room, src, mic, eps), L, FS, C)
    eps32 = float(np.float32(eps))
    deriv = (h1 - h0) / eps32
    expect = np.zeros(L)
    for d in dists:
        expect[int(math.floor(d * FS / C + 0.5))] += 1.0 / (4 * math.pi * d)
    np.testing.assert_allclose(deriv, expect, rtol=0, atol=1e-4 * expect.max())
    # and the six delays are where the response is non-zero beyond the direct path
    assert set(np.nonzero(expect)[0]) <= set(np.nonzero(h1)[0])


def _unfold_axis(s, room, max_refl):
    """Images along one axis by physically reflecting back and forth between the
    walls at 0 and `room`; returns {coordinate: reflections}."""
    out = {s: 0}
    for first in (0, 1):                      # which wall is hit first
        p, wall = s, first
        for n in range(1, max_refl + 1):
            p = -p if wall == 0 else 2 * room - p
            out[p] = n
            wall ^= 1
    return out


def test_axis_images_equal_mirror_unfolding():
    s, room = 1.25, 4.0
    coord, count = O._axis_images(s, room, 3)
    ref = _unfold_axis(s, room, 7)
    got = dict(zip(coord.tolist(), count.tolist()))
    assert len(got) == len(coord)             # no image listed twice
    for x, n in got.items():
        assert ref[x] == n
    # the lattice with |n| <= 3 holds every image of up to 5 reflections
    for x, n in ref.items():
        if n <= 5:
            assert got[x] == n


def test_brute_force_reflection_sequences():
    # Independent enumeration: all per-axis unfoldings up to a reflection order
    # that covers the truncated response, summed the slow way.
    room, src, mic, beta = (3.0, 2.5, 2.0), (1.0, 0.7, 1.1), (2.2, 1.6, 0.8), 0.6
    L = 400                                   # 8.6 m of travel
    g = _geom(room, src, mic, beta)
    h, cnt = O.rir_single(g, L, FS, C)
    gd = g.astype(np.float64)
    axes = [_unfold_axis(gd[3 + a], gd[a], 8) for a in range(3)]
    ref = np.zeros(L)
    ref_cnt = np.zeros(L, dtype=np.int64)
    for (x, nx), (y, ny), (z, nz) in itertools.product(*[ax.items() for ax in axes]):
        d = math.sqrt((x - gd[6]) ** 2 + (y - gd[7]) ** 2 + (z - gd[8]) ** 2)
        n = int(math.floor(d * K + 0.5))
        if n < L:
            ref[n] += float(gd[9]) ** (nx + ny + nz) / (4 * math.pi * d)
            ref_cnt[n] += 1
    np.testing.assert_array_equal(cnt, ref_cnt)
    np.testing.assert_allclose(h, ref, rtol=1e-12, atol=0)


def test_image_count_follows_sphere_volume():
    # Images are one per room volume: taps below L hold about (4/3) pi R^3 / V of
    # them, R = L c / fs, and the count per tap grows like n^2.
    room = (5.0, 4.0, 3.0)
    g = _geom(room, (1.3, 2.2, 1.1), (3.9, 1.2, 1.9), 0.5)
    L = 4096
    _, cnt = O.rir_single(g, L, FS, C)
    R = L * C / FS
    expect = 4.0 / 3.0 * math.pi * R ** 3 / np.prod(room)
    assert cnt.sum() == pytest.approx(expect, rel=0.03)
    inner = cnt[1024:2048].sum()
    outer = cnt[2048:4096].sum()
    assert outer / inner == pytest.approx((4096 ** 3 - 2048 ** 3) / (2048 ** 3 - 1024 ** 3), rel=0.05)


def test_reciprocity():
    # Swapping source and microphone leaves the set of path lengths unchanged.
    room, a, b = (4.0, 3.5, 2.8), (1.0, 2.5, 0.9), (3.1, 0.8, 2.0)
    h1, c1 = O.rir_single(_geom(room, a, b, 0.8), 1500, FS, C)
    h2, c2 = O.rir_single(_geom(room, b, a, 0.8), 1500, FS, C)
    # rounding-boundary cases may move single images between neighbouring taps
    assert np.abs(np.cumsum(c1) - np.cumsum(c2)).max() <= 2
    assert np.sum(h1) == pytest.approx(np.sum(h2), rel=1e-3)


def test_axis_permutation_symmetry():
    # Relabelling the axes of the room does not change the response.
    room, s, m = (4.0, 3.0, 2.5), (1.0, 2.0, 0.7), (3.0, 0.9, 1.9)
    h1, c1 = O.rir_single(_geom(room, s, m, 0.7), 1200, FS, C)
    p = [2, 0, 1]
    perm = lambda v: [v[i] for i in p]
    h2, c2 = O.rir_single(_geom(perm(room), perm(s), perm(m), 0.7), 1200, FS, C)
    # the fixed summation order ((x + y) + z) can move an image on an exact rounding tie only
    assert np.abs(np.cumsum(c1) - np.cumsum(c2)).max() <= 1
    np.testing.assert_allclose(np.cumsum(h1), np.cumsum(h2), rtol=1e-3)


def test_mean_reflection_count_follows_mean_free_path():
    # An image at distance d has crossed |dx|/Lx + |dy|/Ly + |dz|/Lz walls; over
    # all directions that averages to d S / (4 V) (the mean free path is 4V/S).
    # d/d(beta) of the summed response at beta = 1 reads the mean reflection
    # count of the images in a window of taps.
    room = (6.0, 5.0, 3.0)
    src, mic = (1.7, 2.1, 1.2), (4.1, 3.3, 1.6)
    L, a, b = 3600, 3000, 3500
    eps = 2.0 ** -10
    h1, _ = O.rir_single(_geom(room, src, mic, 1.0), L, FS, C)
    h2, _ = O.rir_single(_geom(room, src, mic, 1.0 - eps), L, FS, C)
    mean_k = (h1[a:b].sum() - h2[a:b].sum()) / eps / h1[a:b].sum()
    V = np.prod(room)
    S = 2 * (room[0] * room[1] + room[1] * room[2] + room[0] * room[2])
    d_mid = 0.5 * (a + b) * C / FS
    assert mean_k == pytest.approx(d_mid * S / (4 * V), rel=0.05)


def test_batch_matches_single_and_dtypes():
    g = np.stack([_geom((5, 4, 3), (1, 1, 1), (3, 2, 1.5), 0.7),
                  _geom((3, 3, 2.5), (1, 2, 1), (2, 1, 1.5), 0.3)])
    h, c = O.rir_batch(g, 512, FS, C)
    assert h.dtype == np.float64 and c.dtype == np.int32 and h.shape == (2, 512)
    for r in range(2):
        hs, cs = O.rir_single(g[r], 512, FS, C)
        np.testing.assert_array_equal(h[r], hs)
        np.testing.assert_array_equal(c[r], cs)
