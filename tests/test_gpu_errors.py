"""Error paths of the C ABI on a real device: bad arguments come back as codes, nothing is launched."""
import ctypes

import numpy as np
import pytest

from paper_1912_11040_amd import workloads as W
from paper_1912_11040_amd import binding
from tests.parity import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def aug():
    # the binding's own element-count checks are off here: these tests are about what the library itself refuses
    a = binding.Augmenter(0, check_sizes=False)
    yield a
    a.close()


def _code(fn, *a, **k):
    with pytest.raises(binding.AugError) as e:
        fn(*a, **k)
    return e.value.code, str(e.value)


def test_rir_argument_errors(aug):
    import torch
    g = dev(W.tiny(n_utt=1).geom)
    out = torch.zeros(2, 64, device="cuda")
    assert _code(aug.aug_rir_batch, g, 0, 16000.0, 343.0, out)[0] == binding.AUG_ERR_INVALID_ARG
    assert _code(aug.aug_rir_batch, g, 1 << 20, 16000.0, 343.0, out)[0] == binding.AUG_ERR_UNSUPPORTED
    assert _code(aug.aug_rir_batch, g, 64, 0.0, 343.0, out)[0] == binding.AUG_ERR_INVALID_ARG
    code, msg = _code(aug.aug_rir_batch, g, 64, 16000.0, 343.0, None)
    assert code == binding.AUG_ERR_INVALID_ARG and "null" in msg


def test_offsets_and_frontend_errors(aug):
    import dataclasses
    import torch
    x = torch.zeros(1000, device="cuda")
    alpha = torch.ones(2, device="cuda")
    feats = torch.zeros(8, 40, device="cuda")
    fe = W.FrontendConfig()
    bad = np.array([0, 600, 500], np.int64)
    assert _code(aug.aug_vtlp_mel_batch, bad, x, alpha, fe, [0, 2, 2], feats)[0] == binding.AUG_ERR_INVALID_ARG
    good = np.array([0, 600, 1000], np.int64)
    code, msg = _code(aug.aug_vtlp_mel_batch, good, x, alpha, fe, [0, 2, 2], feats)     # one frame, no row for it
    assert code == binding.AUG_ERR_INVALID_ARG and "frame" in msg
    aug.aug_vtlp_mel_batch(good, x, alpha, fe, [0, 2, 4], feats)                          # a spare row is padding
    torch.cuda.synchronize()
    assert float(feats[3].abs().max()) == 0.0
    fe256 = dataclasses.replace(fe, nfft=256, win=200)
    assert _code(aug.aug_vtlp_mel_batch, good, x, alpha, fe256, [0, 3, 5], feats)[0] == binding.AUG_ERR_UNSUPPORTED
    fe_bad = dataclasses.replace(fe, n_mel=0)
    assert _code(aug.aug_vtlp_mel_batch, good, x, alpha, fe_bad, [0, 2, 3], feats)[0] == binding.AUG_ERR_INVALID_ARG
    fe_kind = dataclasses.replace(fe, feature="mfcc", n_ceps=41)
    assert _code(aug.aug_vtlp_mel_batch, good, x, alpha, fe_kind, [0, 2, 3], feats)[0] == binding.AUG_ERR_INVALID_ARG
    fe_floor = dataclasses.replace(fe, feature="log", log_floor=0.0)
    assert _code(aug.aug_vtlp_mel_batch, good, x, alpha, fe_floor, [0, 2, 3], feats)[0] == binding.AUG_ERR_INVALID_ARG
    # a good call after failures still works
    aug.aug_vtlp_mel_batch(good, x, alpha, fe, [0, 2, 3], feats)
    torch.cuda.synchronize()


def test_mix_argument_errors(aug):
    import torch
    x = torch.zeros(100, device="cuda")
    rir = torch.zeros(1, 2, 16, device="cuda")
    off = np.array([0, 100], np.int64)
    out = torch.zeros(100, device="cuda")
    assert _code(aug.aug_convolve_mix_batch, off, x, None, rir, 16, None, out, n_noise=1)[0] == \
        binding.AUG_ERR_INVALID_ARG
    assert _code(aug.aug_convolve_mix_batch, off, x, None, rir, 16, None, None)[0] == binding.AUG_ERR_INVALID_ARG
    assert _code(aug.aug_convolve_mix_batch, off, x, None, rir, 0, None, out)[0] == binding.AUG_ERR_INVALID_ARG


def test_bad_device_is_rejected():
    lib = binding.load_library()
    h = ctypes.c_void_p()
    assert lib.aug_create(ctypes.byref(h), 99, None) == binding.AUG_ERR_INVALID_ARG
    assert not h.value


def test_binding_refuses_short_tensors_before_the_library_sees_them():
    import torch
    g = dev(W.tiny(n_utt=1).geom)
    with binding.Augmenter(0) as a:
        with pytest.raises(ValueError, match="rir_out"):
            a.aug_rir_batch(g, 64, 16000.0, 343.0, torch.zeros(2 * 64 - 1, device="cuda"))
        x = torch.zeros(1000, device="cuda")
        with pytest.raises(ValueError, match="frame_offsets"):
            a.aug_vtlp_mel_batch([0, 600, 1000], x, torch.ones(2, device="cuda"), W.FrontendConfig(), [0, 2],
                                 torch.zeros(8, 40, device="cuda"))
