"""ctypes binding of libaug.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/aug.h.  PyTorch tensors supply device memory and the stream.  There is
no CPU fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaug.so")

AUG_OK = 0
AUG_ERR_INVALID_ARG = -1
AUG_ERR_UNSUPPORTED = -2
AUG_ERR_NOMEM = -3
AUG_ERR_HIP = -4

EXPORTS = ("aug_create", "aug_destroy", "aug_last_error", "aug_frame_count", "aug_feature_dim", "aug_rir_batch",
           "aug_rir_mics_batch",
           "aug_convolve_mix_batch", "aug_vtlp_mel_batch", "aug_vtlp_mel_batch_static", "aug_vtlp_resynth_batch",
           "aug_pipeline_batch",
           "aug_profile_enable", "aug_profile_read", "aug_rir_visited_images")

FEATURE_KINDS = {"power": 0, "log": 1, "mfcc": 2}      # AUG_FEAT_*

STAGES = ("rir", "rir_spectrum", "convolve", "mix", "mel", "other", "vtlp")


class VtlpCfg(ctypes.Structure):
    """Mirror of aug_vtlp_cfg."""
    _fields_ = [("win", ctypes.c_int), ("hop", ctypes.c_int), ("nfft", ctypes.c_int)]


class AugError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libaug error {code}: {message}")
        self.code = code


class FrontendCfg(ctypes.Structure):
    """Mirror of aug_frontend_cfg."""
    _fields_ = [("fs", ctypes.c_float), ("win", ctypes.c_int), ("hop", ctypes.c_int),
                ("nfft", ctypes.c_int), ("n_mel", ctypes.c_int), ("f_lo", ctypes.c_float),
                ("f_hi", ctypes.c_float), ("power", ctypes.c_float), ("feature", ctypes.c_int),
                ("n_ceps", ctypes.c_int), ("log_floor", ctypes.c_float)]

    @classmethod
    def of(cls, fe) -> "FrontendCfg":
        return cls(float(fe.fs), int(fe.win), int(fe.hop), int(fe.nfft), int(fe.n_mel),
                   float(fe.f_lo), float(fe.f_hi), float(fe.power),
                   FEATURE_KINDS[getattr(fe, "feature", "power")], int(getattr(fe, "n_ceps", 0)),
                   float(getattr(fe, "log_floor", 1e-10)))


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libaug.so (built in-tree by build.py); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build the HIP library first "
            "(python -m paper_1912_11040_amd.build); there is no CPU fallback")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cf, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_int64
    p_i64 = ctypes.POINTER(ctypes.c_int64)
    p_cfg = ctypes.POINTER(FrontendCfg)
    lib.aug_create.argtypes = [ctypes.POINTER(vp), ci, vp]
    lib.aug_create.restype = ci
    lib.aug_destroy.argtypes = [vp]
    lib.aug_destroy.restype = ci
    lib.aug_last_error.argtypes = [vp]
    lib.aug_last_error.restype = ctypes.c_char_p
    lib.aug_frame_count.argtypes = [i64, ci, ci]
    lib.aug_frame_count.restype = i64
    lib.aug_feature_dim.argtypes = [p_cfg]
    lib.aug_feature_dim.restype = ci
    lib.aug_rir_batch.argtypes = [vp, ci, vp, ci, cf, cf, vp, vp]
    lib.aug_rir_batch.restype = ci
    lib.aug_rir_mics_batch.argtypes = [vp, ci, ci, vp, vp, ci, cf, cf, vp, vp]
    lib.aug_rir_mics_batch.restype = ci
    lib.aug_convolve_mix_batch.argtypes = [vp, ci, p_i64, vp, ci, vp, vp, ci, vp, vp, vp]
    lib.aug_convolve_mix_batch.restype = ci
    lib.aug_vtlp_mel_batch.argtypes = [vp, ci, p_i64, vp, vp, p_cfg, p_i64, vp]
    lib.aug_vtlp_mel_batch.restype = ci
    lib.aug_vtlp_mel_batch_static.argtypes = [vp, ci, p_i64, vp, vp, p_cfg, p_i64, vp]
    lib.aug_vtlp_mel_batch_static.restype = ci
    lib.aug_vtlp_resynth_batch.argtypes = [vp, ci, p_i64, vp, vp, ctypes.POINTER(VtlpCfg), vp]
    lib.aug_vtlp_resynth_batch.restype = ci
    lib.aug_pipeline_batch.argtypes = [vp, ci, p_i64, vp, ci, vp, vp, ci, cf, cf, vp, vp, p_cfg,
                                       p_i64, vp, vp, vp, vp]
    lib.aug_pipeline_batch.restype = ci
    lib.aug_rir_visited_images.argtypes = [vp, ci, vp, ci, cf, cf, vp, ctypes.POINTER(ctypes.c_uint64)]
    lib.aug_rir_visited_images.restype = ci
    lib.aug_profile_enable.argtypes = [vp, ci]
    lib.aug_profile_enable.restype = ci
    lib.aug_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int32)]
    lib.aug_profile_read.restype = ci
    _lib = lib
    return lib


def aug_frame_count(n_samples: int, win: int, hop: int) -> int:
    return int(load_library().aug_frame_count(int(n_samples), int(win), int(hop)))


def _host_i64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int64))


def _ptr(t, dtype=None):
    """Device address of a contiguous CUDA/HIP torch tensor (None -> NULL)."""
    if t is None:
        return None
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("expected a torch tensor in device memory")
    if not t.is_contiguous():
        raise ValueError("device tensors must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected dtype {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _numel(t) -> int:
    return 0 if t is None else int(t.numel())


def _need(name: str, t, count: int, exact: bool = False):
    """Raise ValueError unless tensor `t` holds at least (exactly) `count` elements; None counts as empty."""
    have = _numel(t)
    if (have != count) if exact else (have < count):
        raise ValueError(f"{name} holds {have} elements, the call needs {'exactly' if exact else 'at least'} {count}")


# Element counts that the C ABI takes on trust (it sees bare addresses): checked here, on the host, before
# anything is launched.  An undersized output would otherwise be written past its end by a kernel.

def check_offsets_pair(off: np.ndarray, foff: Optional[np.ndarray] = None):
    if off.ndim != 1 or len(off) < 1:
        raise ValueError("offsets must be a one-dimensional array of n_utt + 1 entries")
    if foff is not None and len(foff) != len(off):
        raise ValueError(f"frame_offsets has {len(foff)} entries, offsets has {len(off)}")


def check_rir_sizes(geom, rir_len: int, rir_out, tap_count_out, mics=None, n_mic: int = 1):
    if _numel(geom) % 10:
        raise ValueError("geom must hold 10 values per response")
    n_rir = _numel(geom) // 10
    n_mic, rir_len = max(int(n_mic), 0), max(int(rir_len), 0)      # the library refuses the negative ones itself
    if mics is not None:
        _need("mics", mics, n_rir * n_mic * 3)
    _need("rir_out", rir_out, n_rir * n_mic * rir_len)
    if tap_count_out is not None:
        _need("tap_count_out", tap_count_out, n_rir * n_mic * rir_len)


def check_mix_sizes(off: np.ndarray, speech, n_noise: int, noise, snr_db, gains_out=None):
    n_utt, total = len(off) - 1, int(off[-1])
    _need("speech", speech, total)
    _need("noise", noise, n_noise * total)
    _need("snr_db", snr_db, n_utt * n_noise)
    if gains_out is not None:
        _need("gains_out", gains_out, n_utt * n_noise)


def check_convolve_mix_sizes(off: np.ndarray, speech, n_noise: int, noise, rir, rir_len: int, snr_db, mixed_out,
                             gains_out=None):
    check_offsets_pair(off)
    check_mix_sizes(off, speech, n_noise, noise, snr_db, gains_out)
    _need("rir", rir, (len(off) - 1) * (1 + n_noise) * int(rir_len))
    _need("mixed_out", mixed_out, int(off[-1]))


def check_mel_sizes(off: np.ndarray, foff: np.ndarray, wave, alpha, feats_out, feature_dim: int):
    check_offsets_pair(off, foff)
    _need("wave", wave, int(off[-1]))
    _need("alpha", alpha, len(off) - 1)
    _need("feats_out", feats_out, int(foff[-1]) * int(feature_dim))


def check_pipeline_sizes(off: np.ndarray, foff: np.ndarray, speech, n_noise: int, noise, geom, rir_len: int,
                         snr_db, alpha, feature_dim: int, feats_out, rir_out=None, mixed_out=None, gains_out=None):
    check_offsets_pair(off, foff)
    n_utt = len(off) - 1
    check_mix_sizes(off, speech, n_noise, noise, snr_db, gains_out)
    _need("geom", geom, n_utt * (1 + n_noise) * 10, exact=True)
    _need("alpha", alpha, n_utt)
    _need("feats_out", feats_out, int(foff[-1]) * int(feature_dim))
    if rir_out is not None:
        _need("rir_out", rir_out, n_utt * (1 + n_noise) * int(rir_len))
    if mixed_out is not None:
        _need("mixed_out", mixed_out, int(off[-1]))


def check_resynth_sizes(off: np.ndarray, wave, alpha, wave_out):
    check_offsets_pair(off)
    _need("wave", wave, int(off[-1]))
    _need("alpha", alpha, len(off) - 1)
    _need("wave_out", wave_out, int(off[-1]))


class Augmenter:
    """One library context bound to a device and a stream (torch's current stream by default)."""

    def __init__(self, device: int = 0, stream=None, check_sizes: bool = True):
        """check_sizes=False skips the host-side element-count checks of the tensors (the library still
        validates everything it can see: nulls, sizes, offsets)."""
        import torch
        self._lib = load_library()
        self._check_sizes = bool(check_sizes)
        if stream is None:
            stream = torch.cuda.current_stream(device)
        self.stream = stream
        self.device = device
        handle = ctypes.c_void_p()
        rc = self._lib.aug_create(ctypes.byref(handle), int(device), ctypes.c_void_p(stream.cuda_stream))
        if rc != AUG_OK:
            raise AugError(rc, "aug_create failed")
        self._h = handle

    def close(self):
        if getattr(self, "_h", None):
            self._lib.aug_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def _check(self, rc: int):
        if rc != AUG_OK:
            raise AugError(rc, self._lib.aug_last_error(self._h).decode())

    def aug_profile_enable(self, on: bool):
        self._check(self._lib.aug_profile_enable(self._h, int(bool(on))))

    def aug_profile_read(self):
        """Wait for the stream; {stage: (total ms, launches)} since the last read."""
        ms = (ctypes.c_float * len(STAGES))()
        n = (ctypes.c_int32 * len(STAGES))()
        self._check(self._lib.aug_profile_read(self._h, ms, n))
        return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(STAGES)}

    # ---- the four entry points, same names as the C ABI ----

    def aug_rir_batch(self, geom, rir_len: int, fs: float, c: float, rir_out, tap_count_out=None):
        import torch
        if self._check_sizes:
            check_rir_sizes(geom, rir_len, rir_out, tap_count_out)
        n_rir = int(geom.numel() // 10) if geom is not None else 0
        self._check(self._lib.aug_rir_batch(
            self._h, n_rir, _ptr(geom, torch.float32), int(rir_len), float(fs), float(c),
            _ptr(rir_out, torch.float32), _ptr(tap_count_out, torch.int32)))

    def aug_rir_visited_images(self, geom, rir_len: int, fs: float, c: float, rir_out) -> int:
        """Images the amplitude kernel walks for these rooms (measurement helper; waits for the stream)."""
        import torch
        if self._check_sizes:
            check_rir_sizes(geom, rir_len, rir_out, None)
        n_rir = int(geom.numel() // 10) if geom is not None else 0
        n = ctypes.c_uint64(0)
        self._check(self._lib.aug_rir_visited_images(
            self._h, n_rir, _ptr(geom, torch.float32), int(rir_len), float(fs), float(c),
            _ptr(rir_out, torch.float32), ctypes.byref(n)))
        return int(n.value)

    def aug_rir_mics_batch(self, geom, mics, rir_len: int, fs: float, c: float, rir_out, tap_count_out=None,
                           n_mic: Optional[int] = None):
        """geom [n_rir][10], mics [n_rir][n_mic][3]; n_mic is read from mics' shape unless given."""
        import torch
        n_rir = int(geom.numel() // 10) if geom is not None else 0
        if n_mic is None:
            n_mic = int(mics.shape[-2]) if mics is not None and mics.dim() >= 2 else 0
        if self._check_sizes:
            check_rir_sizes(geom, rir_len, rir_out, tap_count_out, mics, int(n_mic))
        self._check(self._lib.aug_rir_mics_batch(
            self._h, n_rir, int(n_mic), _ptr(geom, torch.float32), _ptr(mics, torch.float32), int(rir_len),
            float(fs), float(c), _ptr(rir_out, torch.float32), _ptr(tap_count_out, torch.int32)))

    def aug_convolve_mix_batch(self, offsets, speech, noise, rir, rir_len: int, snr_db, mixed_out,
                               gains_out=None, n_noise: Optional[int] = None):
        import torch
        off = _host_i64(offsets)
        if n_noise is None:
            n_noise = 0 if noise is None else int(noise.shape[0])
        if self._check_sizes:
            check_convolve_mix_sizes(off, speech, int(n_noise), noise, rir, rir_len, snr_db, mixed_out, gains_out)
        self._check(self._lib.aug_convolve_mix_batch(
            self._h, len(off) - 1, off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
            _ptr(speech, torch.float32), int(n_noise), _ptr(noise, torch.float32),
            _ptr(rir, torch.float32), int(rir_len), _ptr(snr_db, torch.float32),
            _ptr(mixed_out, torch.float32), _ptr(gains_out, torch.float32)))

    def aug_vtlp_mel_batch(self, offsets, wave, alpha, cfg, frame_offsets, feats_out):
        import torch
        off = _host_i64(offsets)
        foff = _host_i64(frame_offsets)
        c = cfg if isinstance(cfg, FrontendCfg) else FrontendCfg.of(cfg)
        if self._check_sizes:
            check_mel_sizes(off, foff, wave, alpha, feats_out, self._lib.aug_feature_dim(ctypes.byref(c)))
        self._check(self._lib.aug_vtlp_mel_batch(
            self._h, len(off) - 1, off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
            _ptr(wave, torch.float32), _ptr(alpha, torch.float32), ctypes.byref(c),
            foff.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), _ptr(feats_out, torch.float32)))

    def aug_vtlp_mel_batch_static(self, offsets, wave, alpha, cfg, frame_offsets, feats_out):
        """aug_vtlp_mel_batch with its tables in the library's static device array: the call allocates nothing."""
        import torch
        off = _host_i64(offsets)
        foff = _host_i64(frame_offsets)
        c = cfg if isinstance(cfg, FrontendCfg) else FrontendCfg.of(cfg)
        if self._check_sizes:
            check_mel_sizes(off, foff, wave, alpha, feats_out, self._lib.aug_feature_dim(ctypes.byref(c)))
        self._check(self._lib.aug_vtlp_mel_batch_static(
            self._h, len(off) - 1, off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
            _ptr(wave, torch.float32), _ptr(alpha, torch.float32), ctypes.byref(c),
            foff.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), _ptr(feats_out, torch.float32)))

    def aug_vtlp_resynth_batch(self, offsets, wave, alpha, wave_out, win: int = 800, hop: int = 400,
                               nfft: int = 2048):
        import torch
        off = _host_i64(offsets)
        c = VtlpCfg(int(win), int(hop), int(nfft))
        if self._check_sizes:
            check_resynth_sizes(off, wave, alpha, wave_out)
        self._check(self._lib.aug_vtlp_resynth_batch(
            self._h, len(off) - 1, off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
            _ptr(wave, torch.float32), _ptr(alpha, torch.float32), ctypes.byref(c),
            _ptr(wave_out, torch.float32)))

    def aug_pipeline_batch(self, offsets, speech, noise, geom, rir_len: int, fs: float, c: float,
                           snr_db, alpha, cfg, frame_offsets, feats_out, rir_out=None,
                           mixed_out=None, gains_out=None, n_noise: Optional[int] = None):
        import torch
        off = _host_i64(offsets)
        foff = _host_i64(frame_offsets)
        fc = cfg if isinstance(cfg, FrontendCfg) else FrontendCfg.of(cfg)
        if n_noise is None:
            n_noise = 0 if noise is None else int(noise.shape[0])
        if self._check_sizes:
            check_pipeline_sizes(off, foff, speech, int(n_noise), noise, geom, rir_len, snr_db, alpha,
                                 self._lib.aug_feature_dim(ctypes.byref(fc)), feats_out, rir_out, mixed_out,
                                 gains_out)
        self._check(self._lib.aug_pipeline_batch(
            self._h, len(off) - 1, off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
            _ptr(speech, torch.float32), int(n_noise), _ptr(noise, torch.float32),
            _ptr(geom, torch.float32), int(rir_len), float(fs), float(c),
            _ptr(snr_db, torch.float32), _ptr(alpha, torch.float32), ctypes.byref(fc),
            foff.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), _ptr(feats_out, torch.float32),
            _ptr(rir_out, torch.float32), _ptr(mixed_out, torch.float32),
            _ptr(gains_out, torch.float32)))
