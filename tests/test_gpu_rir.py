"""aug_rir_batch against the oracle: tap counts bit for bit, amplitudes to 1e-5."""
import numpy as np
import pytest

from oracle import aug_oracle as O
from paper_1912_11040_amd import workloads as W
from tests.parity import RIR_TOL, dev, rir_err

pytestmark = pytest.mark.gpu
FS, C = 16000.0, 343.0


@pytest.fixture(scope="module")
def aug():
    import torch
    from paper_1912_11040_amd.binding import Augmenter
    assert torch.cuda.is_available()
    a = Augmenter(0)
    yield a
    a.close()


def _run(aug, geom, L, counts=True):
    import torch
    g = dev(np.asarray(geom, np.float32).reshape(-1, 10))
    n = g.shape[0]
    h = torch.full((n, L), float("nan"), dtype=torch.float32, device="cuda")
    cnt = torch.full((n, L), -7, dtype=torch.int32, device="cuda") if counts else None
    aug.aug_rir_batch(g, L, FS, C, h, cnt)
    torch.cuda.synchronize()
    return h.cpu().numpy(), (cnt.cpu().numpy() if counts else None)


def _check(aug, geom, L):
    geom = np.asarray(geom, np.float32).reshape(-1, 10)
    h, cnt = _run(aug, geom, L)
    h_ref, cnt_ref = O.rir_batch(geom, L, FS, C)
    np.testing.assert_array_equal(cnt, cnt_ref)          # integer work: bit exact
    assert rir_err(h, h_ref) <= RIR_TOL
    return h, cnt


def test_tiny_config_rirs(aug):
    w = W.tiny()
    print("case: tiny geom, L=4096", flush=True)
    _check(aug, w.geom, 4096)


@pytest.mark.parametrize("L", [1, 63, 1000, 5000])
def test_ragged_lengths(aug, L):
    w = W.tiny(n_utt=2)
    print(f"case: tiny geom, L={L}", flush=True)
    _check(aug, w.geom, L)


def test_random_rooms_8000_taps(aug):
    w = W.batch(n_utt=6, seconds=0.1)
    print("case: batch geom 12 rirs, L=8000", flush=True)
    _check(aug, w.geom, 8000)


def test_split_over_several_groups_16000_taps(aug):
    # small rooms at 16000 taps hold millions of images and are cut over many work groups
    g = np.array([[3.0, 3.1, 2.5, 1.0, 1.2, 1.1, 2.2, 2.0, 1.4, 0.9],
                  [9.5, 7.5, 3.9, 2.0, 3.0, 1.5, 7.0, 5.0, 2.0, 0.35]], np.float32)
    print("case: two rooms, L=16000", flush=True)
    _, cnt = _check(aug, g, 16000)
    assert cnt[0].sum() > 5_000_000


def test_longest_response_the_interface_takes(aug):
    w = W.throughput(n_utt=1, seconds=0.1)
    print("case: throughput geom, 3 rirs, L=32768", flush=True)
    _check(aug, w.geom, 32768)


def test_unusable_rooms_give_silence_and_leave_the_rest_alone(aug):
    # the library's guard against an unbounded image lattice: a side under 10 cm or not a number
    w = W.tiny(n_utt=2)
    geom = np.asarray(w.geom, np.float32).reshape(-1, 10).copy()
    good = geom.copy()
    geom[1, 0] = 0.05
    geom[2, 1] = np.nan
    h, cnt = _run(aug, geom, 1500)
    for bad_beta in (-0.5, 1.5, np.nan):
        g2 = good.copy()
        g2[1, 9] = bad_beta
        h2, cnt2 = _run(aug, g2, 700)
        assert np.all(h2[1] == 0.0) and np.all(cnt2[1] == 0) and np.any(h2[0] != 0.0)
    assert np.all(h[1] == 0.0) and np.all(cnt[1] == 0) and np.all(h[2] == 0.0) and np.all(cnt[2] == 0)
    h_ref, cnt_ref = O.rir_batch(good[[0, 3]], 1500, FS, C)
    np.testing.assert_array_equal(cnt[[0, 3]], cnt_ref)
    assert rir_err(h[[0, 3]], h_ref) <= RIR_TOL


def test_zero_reflection_closed_form(aug):
    g = np.array([[5, 4, 3, 1.0, 1.5, 1.2, 3.5, 2.0, 1.7, 0.0]], np.float32)
    h, _ = _run(aug, g, 2048)
    gd = g[0].astype(np.float64)
    r = np.sqrt(np.sum((gd[3:6] - gd[6:9]) ** 2))
    n0 = int(np.floor(r * FS / C + 0.5))
    assert np.count_nonzero(h) == 1
    assert h[0, n0] == pytest.approx(1 / (4 * np.pi * r), rel=1e-6)


def test_without_counts_and_empty_batch(aug):
    import torch
    w = W.tiny(n_utt=1)
    h, _ = _run(aug, w.geom, 777, counts=False)
    h_ref, _ = O.rir_batch(w.geom.reshape(-1, 10), 777, FS, C)
    assert rir_err(h, h_ref) <= RIR_TOL
    aug.aug_rir_batch(None, 128, FS, C, None, None)       # n_rir == 0: no-op
    torch.cuda.synchronize()


def test_beta_one_and_repeatable_counts(aug):
    g = np.array([[4.0, 3.0, 2.6, 1.0, 1.1, 1.2, 3.0, 2.0, 1.3, 1.0]], np.float32)
    h, cnt = _check(aug, g, 3000)
    h2, cnt2 = _run(aug, g, 3000)
    np.testing.assert_array_equal(cnt, cnt2)
    assert rir_err(h2, h.astype(np.float64)) <= RIR_TOL


def test_very_flat_room_walks_images_directly(aug):
    # a 12 cm high room has more z images than the kernel's LDS table holds; it then walks them directly
    g = np.array([[3.0, 3.2, 0.12, 1.0, 1.1, 0.04, 2.1, 2.0, 0.08, 0.5],
                  [4.0, 3.0, 2.7, 1.0, 1.1, 1.0, 2.1, 2.0, 1.5, 0.6]], np.float32)
    print("case: flat room, L=2000", flush=True)
    _check(aug, g, 2000)


@pytest.mark.parametrize("axis", [0, 1])
def test_very_narrow_rooms_walk_images_directly(aug, axis):
    # 12 cm wide along x (more than 320 x images per parity inside the response's radius: the rows of the
    # column table do not fit) or along y (the sorted y table does not fit): both take the plain path
    dims = [3.0, 3.2, 2.7]
    src, mic = [1.0, 1.1, 1.0], [2.1, 2.0, 1.5]
    dims[axis], src[axis], mic[axis] = 0.12, 0.04, 0.08
    g = np.array([dims + src + mic + [0.5],
                  [4.0, 3.0, 2.7, 1.0, 1.1, 1.0, 2.1, 2.0, 1.5, 0.6]], np.float32)
    print(f"case: room 12 cm wide along axis {axis}, L=2000", flush=True)
    _, cnt = _check(aug, g, 2000)
    assert cnt[0].sum() > 200_000


def test_symmetric_geometry_with_tied_distances(aug):
    # source and microphone at mid height: images above and below tie exactly in distance
    g = np.array([[4.0, 4.0, 3.0, 1.0, 2.0, 1.5, 3.0, 2.0, 1.5, 0.8],
                  [4.0, 4.0, 3.0, 2.0, 2.0, 1.5, 2.0, 2.0, 1.0, 0.5]], np.float32)
    print("case: symmetric rooms, L=3000", flush=True)
    _check(aug, g, 3000)
