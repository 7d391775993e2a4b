"""aug_rir_mics_batch against the several-microphones oracle: tap counts bit for bit, amplitudes to 1e-5."""
import numpy as np
import pytest

from oracle import aug_oracle as O
from paper_1912_11040_amd import binding
from paper_1912_11040_amd import workloads as W
from tests.parity import RIR_TOL, dev, rir_err

pytestmark = pytest.mark.gpu
FS, C = 16000.0, 343.0


@pytest.fixture(scope="module")
def aug():
    from paper_1912_11040_amd.binding import Augmenter
    a = Augmenter(0)
    yield a
    a.close()


def _run(aug, geom, mics, L, counts=True):
    import torch
    n, K = mics.shape[0], mics.shape[1]
    h = torch.full((n, K, L), float("nan"), dtype=torch.float32, device="cuda")
    cnt = torch.full((n, K, L), -7, dtype=torch.int32, device="cuda") if counts else None
    aug.aug_rir_mics_batch(dev(geom), dev(mics), L, FS, C, h, cnt)
    torch.cuda.synchronize()
    return h.cpu().numpy(), (cnt.cpu().numpy() if counts else None)


def test_pair_of_microphones_6p8_cm_apart(aug):
    w = W.tiny(n_utt=3)
    geom = np.asarray(w.geom, np.float32).reshape(-1, 10)
    mics = W.microphone_arrays(geom, 2, 0.068, seed=11)
    L = 3000
    print(f"case: {len(geom)} rooms x 2 microphones 6.8 cm apart, L={L}", flush=True)
    h, cnt = _run(aug, geom, mics, L)
    h_ref, cnt_ref = O.rir_mics_batch(geom, mics, L, FS, C)
    np.testing.assert_array_equal(cnt, cnt_ref)
    assert rir_err(h, h_ref) <= RIR_TOL
    # the two channels are different responses, a few taps apart at most in their direct paths
    first = np.argmax(h > 0, axis=2)
    assert np.all(np.abs(first[:, 0] - first[:, 1]) <= 4) and not np.array_equal(h[:, 0], h[:, 1])


def test_each_slice_is_the_single_microphone_result_bit_for_bit(aug):
    import torch
    rng = np.random.default_rng(5)
    w = W.batch(n_utt=4, seconds=0.1)
    geom = np.asarray(w.geom, np.float32).reshape(-1, 10)
    K, L = 3, 1700
    lo, hi = 0.15, geom[:, None, 0:3] - 0.15
    mics = (lo + rng.uniform(0, 1, (len(geom), K, 3)) * (hi - lo)).astype(np.float32)
    print(f"case: {len(geom)} rooms x {K} microphones anywhere in the room, L={L}", flush=True)
    h, cnt = _run(aug, geom, mics, L)
    h_ref, cnt_ref = O.rir_mics_batch(geom, mics, L, FS, C)
    np.testing.assert_array_equal(cnt, cnt_ref)
    assert rir_err(h, h_ref) <= RIR_TOL
    for m in range(K):
        g = geom.copy()
        g[:, 6:9] = mics[:, m]
        one = torch.empty((len(geom), L), dtype=torch.float32, device="cuda")
        aug.aug_rir_batch(dev(g), L, FS, C, one)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(h[:, m], one.cpu().numpy())


def test_one_microphone_and_most_microphones(aug):
    w = W.tiny(n_utt=1)
    geom = np.asarray(w.geom, np.float32).reshape(-1, 10)[:2]
    rng = np.random.default_rng(9)
    for K in (1, binding_max_mic()):
        mics = (geom[:, None, 6:9] + rng.uniform(-0.1, 0.1, (len(geom), K, 3))).astype(np.float32)
        h, cnt = _run(aug, geom, mics, 900)
        h_ref, cnt_ref = O.rir_mics_batch(geom, mics, 900, FS, C)
        np.testing.assert_array_equal(cnt, cnt_ref)
        assert rir_err(h, h_ref) <= RIR_TOL


def binding_max_mic():
    import os
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    return int(re.search(r"#define\s+AUG_MAX_MIC\s+(\d+)", open(os.path.join(root, "include", "aug.h")).read()).group(1))


def test_argument_errors():
    import torch
    # the binding's own element-count checks are off: this test is about what the library itself refuses
    aug = binding.Augmenter(0, check_sizes=False)
    g = torch.zeros(1, 10, device="cuda")
    m = torch.zeros(1, 2, 3, device="cuda")
    out = torch.zeros(1, 2, 16, device="cuda")

    def code(*a, **k):
        try:
            aug.aug_rir_mics_batch(*a, **k)
        except binding.AugError as e:
            return e.code
        return 0
    assert code(g, m, 16, FS, C, out, n_mic=0) == binding.AUG_ERR_INVALID_ARG
    assert code(g, m, 16, FS, C, out, n_mic=binding_max_mic() + 1) == binding.AUG_ERR_INVALID_ARG
    assert code(g, None, 16, FS, C, out, n_mic=2) == binding.AUG_ERR_INVALID_ARG
    assert code(g, m, 16, FS, C, None) == binding.AUG_ERR_INVALID_ARG
    assert code(g, m, 0, FS, C, out) == binding.AUG_ERR_INVALID_ARG
    # zero rooms is a no-op; a degenerate room gives silence for each of its microphones
    assert code(None, None, 16, FS, C, None, n_mic=2) == 0
    aug.aug_rir_mics_batch(g, m, 16, FS, C, out)
    torch.cuda.synchronize()
    assert np.all(out.cpu().numpy() == 0.0)
    aug.close()
