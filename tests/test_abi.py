"""The C-ABI library builds, loads and exports what include/aug.h declares.  CPU only:
no kernel is launched here."""
import ctypes
import os
import re

import pytest

from paper_1912_11040_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.load_library()


def _declared():
    text = open(os.path.join(ROOT, "include", "aug.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aug_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_entry_points():
    names = _declared()
    for n in ("aug_rir_batch", "aug_convolve_mix_batch", "aug_vtlp_mel_batch", "aug_pipeline_batch",
              "aug_create", "aug_destroy", "aug_last_error", "aug_frame_count"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    for name in _declared():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == _declared()


def test_frame_count_helper(lib):
    assert binding.aug_frame_count(16000, 400, 160) == 98
    assert binding.aug_frame_count(399, 400, 160) == 0
    assert binding.aug_frame_count(400, 400, 160) == 1
    assert binding.aug_frame_count(100, 0, 160) == -1


def test_frontend_struct_matches_header():
    assert ctypes.sizeof(binding.FrontendCfg) == 44
    assert [f[0] for f in binding.FrontendCfg._fields_] == \
        ["fs", "win", "hop", "nfft", "n_mel", "f_lo", "f_hi", "power", "feature", "n_ceps", "log_floor"]
    # the field order and the enumerators are the header's
    hdr = open(os.path.join(ROOT, "include", "aug.h")).read()
    body = hdr[hdr.index("typedef struct aug_frontend_cfg {"):hdr.index("} aug_frontend_cfg;")]
    names = re.findall(r"^\s*(?:float|int)\s+(\w+);", body, flags=re.M)
    assert names == [f[0] for f in binding.FrontendCfg._fields_]
    for name, value in (("AUG_FEAT_POWER_LAW", "power"), ("AUG_FEAT_LOG", "log"), ("AUG_FEAT_MFCC", "mfcc")):
        assert int(re.search(name + r"\s*=\s*(\d+)", hdr).group(1)) == binding.FEATURE_KINDS[value]


def test_feature_dim_helper(lib):
    from paper_1912_11040_amd.workloads import FrontendConfig
    import dataclasses
    fe = FrontendConfig()
    assert lib.aug_feature_dim(ctypes.byref(binding.FrontendCfg.of(fe))) == 40
    assert lib.aug_feature_dim(ctypes.byref(binding.FrontendCfg.of(dataclasses.replace(fe, feature="log")))) == 40
    assert lib.aug_feature_dim(ctypes.byref(binding.FrontendCfg.of(dataclasses.replace(fe, feature="mfcc")))) == 13
    assert lib.aug_feature_dim(None) == 0


def test_null_context_is_rejected(lib):
    assert lib.aug_rir_batch(None, 1, None, 16, 16000.0, 343.0, None, None) == binding.AUG_ERR_INVALID_ARG
    assert lib.aug_rir_mics_batch(None, 1, 2, None, None, 16, 16000.0, 343.0, None, None) == binding.AUG_ERR_INVALID_ARG
    assert lib.aug_vtlp_resynth_batch(None, 0, None, None, None, None, None) == binding.AUG_ERR_INVALID_ARG
    assert lib.aug_destroy(None) == binding.AUG_OK
    assert lib.aug_last_error(None) == b"context is null"


def test_limits_in_the_header_match_the_binding():
    text = open(os.path.join(ROOT, "include", "aug.h")).read()
    limit = lambda name: int(re.search(r"#define\s+" + name + r"\s+(\d+)", text).group(1))
    assert limit("AUG_MAX_RIR_LEN") == 32768 and limit("AUG_MAX_NOISE") == 8
    assert limit("AUG_MAX_MEL") == 128 and limit("AUG_MAX_MIC") == 16 and limit("AUG_MAX_UTT") == 65535


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libaug.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load_library()
