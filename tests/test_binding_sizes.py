"""The Python layer refuses tensors that are too small for the call before anything reaches the library
(the C ABI sees bare addresses and takes the counts on trust).  CPU only: the checks read element counts."""
import numpy as np
import pytest
import torch

from paper_1912_11040_amd import binding as B

OFF = np.array([0, 1000, 1000, 2500], dtype=np.int64)       # three utterances, the middle one empty
FOFF = np.array([0, 4, 4, 18], dtype=np.int64)
N_UTT, TOTAL, N_NOISE, L, DIM = 3, 2500, 2, 300, 40


def t(n, dtype=torch.float32):
    return torch.zeros(n, dtype=dtype)


def good_pipeline():
    return dict(off=OFF, foff=FOFF, speech=t(TOTAL), n_noise=N_NOISE, noise=t(N_NOISE * TOTAL).view(N_NOISE, TOTAL),
                geom=t(N_UTT * 3 * 10), rir_len=L, snr_db=t(N_UTT * N_NOISE), alpha=t(N_UTT), feature_dim=DIM,
                feats_out=t(18 * DIM), rir_out=t(N_UTT * 3 * L), mixed_out=t(TOTAL), gains_out=t(N_UTT * N_NOISE))


def test_well_sized_calls_pass():
    B.check_pipeline_sizes(**good_pipeline())
    B.check_convolve_mix_sizes(OFF, t(TOTAL), N_NOISE, t(N_NOISE * TOTAL), t(N_UTT * 3 * L), L, t(6), t(TOTAL), t(6))
    B.check_mel_sizes(OFF, FOFF, t(TOTAL), t(N_UTT), t(18 * DIM), DIM)
    B.check_rir_sizes(t(50), L, t(5 * L), t(5 * L, torch.int32))
    B.check_rir_sizes(t(50), L, t(10 * L), None, t(5 * 2 * 3), 2)
    B.check_resynth_sizes(OFF, t(TOTAL), t(N_UTT), t(TOTAL))
    # optional outputs left out, no noise at all, an empty batch
    B.check_pipeline_sizes(**{**good_pipeline(), "rir_out": None, "mixed_out": None, "gains_out": None})
    B.check_pipeline_sizes(OFF, FOFF, t(TOTAL), 0, None, t(N_UTT * 10), L, None, t(N_UTT), DIM, t(18 * DIM))
    B.check_pipeline_sizes(np.zeros(1, np.int64), np.zeros(1, np.int64), None, 0, None, None, L, None, None, DIM, None)


@pytest.mark.parametrize("field,size", [
    ("speech", TOTAL - 1), ("noise", N_NOISE * TOTAL - 1), ("geom", N_UTT * 3 * 10 - 10), ("geom", N_UTT * 3 * 10 + 10),
    ("snr_db", N_UTT * N_NOISE - 1), ("alpha", N_UTT - 1), ("feats_out", 18 * DIM - 1), ("rir_out", N_UTT * 3 * L - 1),
    ("mixed_out", TOTAL - 1), ("gains_out", N_UTT * N_NOISE - 1)])
def test_pipeline_refuses_a_short_tensor(field, size):
    with pytest.raises(ValueError, match=field):
        B.check_pipeline_sizes(**{**good_pipeline(), field: t(size)})


def test_frame_offsets_must_be_as_long_as_offsets():
    with pytest.raises(ValueError, match="frame_offsets"):
        B.check_pipeline_sizes(**{**good_pipeline(), "foff": FOFF[:-1]})
    with pytest.raises(ValueError, match="frame_offsets"):
        B.check_mel_sizes(OFF, FOFF[:-1], t(TOTAL), t(N_UTT), t(18 * DIM), DIM)


def test_stage_calls_refuse_short_tensors():
    with pytest.raises(ValueError, match="rir_out"):
        B.check_rir_sizes(t(50), L, t(5 * L - 1), None)
    with pytest.raises(ValueError, match="tap_count_out"):
        B.check_rir_sizes(t(50), L, t(5 * L), t(5 * L - 1, torch.int32))
    with pytest.raises(ValueError, match="10 values"):
        B.check_rir_sizes(t(49), L, t(5 * L), None)
    with pytest.raises(ValueError, match="mics"):
        B.check_rir_sizes(t(50), L, t(10 * L), None, t(5 * 2 * 3 - 3), 2)
    with pytest.raises(ValueError, match="rir_out"):
        B.check_rir_sizes(t(50), L, t(5 * L), None, t(5 * 2 * 3), 2)
    with pytest.raises(ValueError, match="rir "):
        B.check_convolve_mix_sizes(OFF, t(TOTAL), N_NOISE, t(N_NOISE * TOTAL), t(N_UTT * 3 * L - 1), L, t(6), t(TOTAL))
    with pytest.raises(ValueError, match="mixed_out"):
        B.check_convolve_mix_sizes(OFF, t(TOTAL), N_NOISE, t(N_NOISE * TOTAL), t(N_UTT * 3 * L), L, t(6), t(TOTAL - 1))
    with pytest.raises(ValueError, match="feats_out"):
        B.check_mel_sizes(OFF, FOFF, t(TOTAL), t(N_UTT), t(18 * DIM - 1), DIM)
    with pytest.raises(ValueError, match="wave_out"):
        B.check_resynth_sizes(OFF, t(TOTAL), t(N_UTT), t(TOTAL - 1))
