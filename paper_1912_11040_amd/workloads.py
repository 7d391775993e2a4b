"""Seeded synthetic inputs for the augmentation + feature hot path.

This module only *draws inputs*: waveforms, room geometry, SNRs and warp
factors.  It holds none of the method's arithmetic (no image sums, no
convolution, no mixing, no STFT/mel code) so that the CPU oracle and the HIP
path can both be fed from it without sharing any computation.

The paper (Sec. 2.3) draws one warp factor per utterance and simulates a new
room, reverberation time and SNR per example on the fly; its corpora are not
reproduced here.  The signals below stand in for them: 16 kHz mono,
speech-like second-order resonances under a 4 Hz syllabic envelope, and
white / pink / babble noise.

Draw order inside one workload (fixed, so a seed names one data set):
lengths -> speech -> noise sources -> geometry -> SNR -> alpha.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np
from scipy.signal import lfilter

FS = 16000.0
SPEED_OF_SOUND = 343.0


@dataclass(frozen=True)
class FrontendConfig:
    """STFT / mel front-end constants shared by every workload."""
    fs: float = FS
    win: int = 400
    hop: int = 160
    nfft: int = 512
    n_mel: int = 40
    f_lo: float = 0.0
    f_hi: float = 8000.0
    power: float = 1.0 / 15.0
    feature: str = "power"      # "power": E^power;  "log": ln max(E, log_floor);  "mfcc": DCT-II of the log energies
    n_ceps: int = 13            # coefficients kept when feature == "mfcc"
    log_floor: float = 1e-10

    @property
    def feature_dim(self) -> int:
        return self.n_ceps if self.feature == "mfcc" else self.n_mel


@dataclass
class Workload:
    name: str
    seed: int
    offsets: np.ndarray                  # int64 [n_utt+1], sample offsets into the packed arrays
    speech: np.ndarray                   # float32 [total]
    noise: Optional[np.ndarray]          # float32 [n_noise, total] or None
    geom: Optional[np.ndarray]           # float32 [n_utt, 1+n_noise, 10] or None
    snr_db: Optional[np.ndarray]         # float32 [n_utt, n_noise] or None
    alpha: np.ndarray                    # float32 [n_utt]
    rir_len: int
    fs: float = FS
    c: float = SPEED_OF_SOUND
    frontend: FrontendConfig = field(default_factory=FrontendConfig)

    @property
    def n_utt(self) -> int:
        return len(self.offsets) - 1

    @property
    def n_noise(self) -> int:
        return 0 if self.noise is None else int(self.noise.shape[0])

    @property
    def total(self) -> int:
        return int(self.offsets[-1])

    @property
    def audio_seconds(self) -> float:
        return self.total / self.fs

    def lengths(self) -> np.ndarray:
        return np.diff(self.offsets)

    def frame_offsets(self) -> np.ndarray:
        """Prefix sum of per-utterance frame counts (no padding, floor framing)."""
        n = self.lengths()
        fe = self.frontend
        t = np.where(n >= fe.win, 1 + (n - fe.win) // fe.hop, 0)
        out = np.zeros(self.n_utt + 1, dtype=np.int64)
        np.cumsum(t, out=out[1:])
        return out

    def slice(self, utts) -> "Workload":
        """A workload holding only the listed utterances (same draws, repacked)."""
        utts = list(utts)
        lens = self.lengths()[utts]
        off = np.zeros(len(utts) + 1, dtype=np.int64)
        np.cumsum(lens, out=off[1:])
        idx = np.concatenate([np.arange(self.offsets[u], self.offsets[u + 1]) for u in utts]) \
            if utts else np.zeros(0, dtype=np.int64)
        return Workload(
            name=f"{self.name}[{len(utts)}]", seed=self.seed, offsets=off,
            speech=np.ascontiguousarray(self.speech[idx]),
            noise=None if self.noise is None else np.ascontiguousarray(self.noise[:, idx]),
            geom=None if self.geom is None else np.ascontiguousarray(self.geom[utts]),
            snr_db=None if self.snr_db is None else np.ascontiguousarray(self.snr_db[utts]),
            alpha=np.ascontiguousarray(self.alpha[utts]), rir_len=self.rir_len,
            fs=self.fs, c=self.c, frontend=self.frontend)


# --------------------------------------------------------------------------
# signal recipes
# --------------------------------------------------------------------------

def _unit_rms(x: np.ndarray) -> np.ndarray:
    if x.size == 0:
        return x
    r = np.sqrt(np.mean(np.square(x, dtype=np.float64)))
    return x / r if r > 0 else x


def _ar2(rng: np.random.Generator, n: int) -> np.ndarray:
    """x[t] = 2 r cos(theta) x[t-1] - r^2 x[t-2] + u[t], r = 0.95, unit RMS."""
    theta = rng.uniform(0.05 * np.pi, 0.3 * np.pi)
    r = 0.95
    u = rng.standard_normal(n)
    x = lfilter([1.0], [1.0, -2.0 * r * np.cos(theta), r * r], u)
    return _unit_rms(x)


def _envelope(rng: np.random.Generator, n: int, fs: float) -> np.ndarray:
    """0.1 + 0.9 * (1 + sin(2 pi 4 t + phi)) / 2 with a random phase."""
    phi = rng.uniform(0.0, 2.0 * np.pi)
    t = np.arange(n) / fs
    return 0.1 + 0.9 * 0.5 * (1.0 + np.sin(2.0 * np.pi * 4.0 * t + phi))


def speech_like(rng: np.random.Generator, n: int, fs: float = FS) -> np.ndarray:
    return (_ar2(rng, n) * _envelope(rng, n, fs)).astype(np.float32)


def white_noise(rng: np.random.Generator, n: int, fs: float = FS) -> np.ndarray:
    return rng.standard_normal(n).astype(np.float32)


def pink_noise(rng: np.random.Generator, n: int, fs: float = FS) -> np.ndarray:
    """White noise whose spectrum is scaled by 1/sqrt(max(f, 20 Hz)); unit RMS."""
    u = rng.standard_normal(n)
    if n == 0:
        return u.astype(np.float32)
    spec = np.fft.rfft(u)
    f = np.fft.rfftfreq(n, d=1.0 / fs)
    spec /= np.sqrt(np.maximum(f, 20.0))
    return _unit_rms(np.fft.irfft(spec, n)).astype(np.float32)


def babble_noise(rng: np.random.Generator, n: int, fs: float = FS) -> np.ndarray:
    """Sum of five independent speech-like signals; unit RMS."""
    acc = np.zeros(n)
    for _ in range(5):
        acc += _ar2(rng, n) * _envelope(rng, n, fs)
    return _unit_rms(acc).astype(np.float32)


_NOISE_KINDS = {"white": white_noise, "pink": pink_noise, "babble": babble_noise}


# --------------------------------------------------------------------------
# geometry
# --------------------------------------------------------------------------

def _position(rng: np.random.Generator, dims: np.ndarray, margin: float) -> np.ndarray:
    return np.array([rng.uniform(margin, d - margin) for d in dims])


def draw_geometry(rng: np.random.Generator, n_src: int, dims, beta: float,
                  margin: float = 0.5, min_dist: float = 0.1) -> np.ndarray:
    """Rows [Lx,Ly,Lz, sx,sy,sz, mx,my,mz, beta] for n_src sources and one shared mic.

    Source and microphone stay `margin` metres from every wall and at least
    `min_dist` metres from each other (rejection sampling on the source).
    """
    dims = np.asarray(dims, dtype=np.float64)
    mic = _position(rng, dims, margin)
    rows = np.zeros((n_src, 10), dtype=np.float32)
    for j in range(n_src):
        while True:
            src = _position(rng, dims, margin)
            if np.linalg.norm(src - mic) >= min_dist:
                break
        rows[j, 0:3] = dims
        rows[j, 3:6] = src
        rows[j, 6:9] = mic
        rows[j, 9] = beta
    return rows


def microphone_arrays(geom, n_mic: int = 2, spacing: float = 0.068, seed: int = 0) -> np.ndarray:
    """A small horizontal line array in place of each row's microphone: [n_rows, n_mic, 3] float32.

    The n_mic microphones of a row are `spacing` metres apart along a randomly oriented horizontal line
    centred on that row's own microphone position (two microphones 6.8 cm apart by default, the device
    of Sec. 4).  Rows keep their `margin` from the walls as long as the array is shorter than it.
    """
    geom = np.asarray(geom, dtype=np.float32).reshape(-1, 10)
    rng = np.random.default_rng(seed)
    phi = rng.uniform(0.0, 2.0 * np.pi, len(geom))
    along = np.stack([np.cos(phi), np.sin(phi), np.zeros_like(phi)], axis=1)            # [n, 3]
    steps = (np.arange(n_mic) - 0.5 * (n_mic - 1)) * spacing                              # [n_mic]
    mics = geom[:, None, 6:9].astype(np.float64) + steps[None, :, None] * along[:, None, :]
    return mics.astype(np.float32)


def _random_room(rng: np.random.Generator):
    dims = np.array([rng.uniform(3.0, 10.0), rng.uniform(3.0, 8.0), rng.uniform(2.5, 4.0)])
    beta = rng.uniform(0.2, 0.9)
    return dims, beta


# --------------------------------------------------------------------------
# workload assembly
# --------------------------------------------------------------------------

def _assemble(name, seed, lengths, noise_kinds, rir_len, snr_range, fixed_room=None,
              with_room=True) -> Workload:
    rng = np.random.default_rng(seed)
    lengths = np.asarray(lengths, dtype=np.int64)
    n_utt = len(lengths)
    offsets = np.zeros(n_utt + 1, dtype=np.int64)
    np.cumsum(lengths, out=offsets[1:])
    total = int(offsets[-1])

    speech = np.empty(total, dtype=np.float32)
    for u in range(n_utt):
        speech[offsets[u]:offsets[u + 1]] = speech_like(rng, int(lengths[u]))

    n_noise = len(noise_kinds)
    noise = None
    if n_noise:
        noise = np.empty((n_noise, total), dtype=np.float32)
        for u in range(n_utt):
            for j, kind in enumerate(noise_kinds):
                noise[j, offsets[u]:offsets[u + 1]] = _NOISE_KINDS[kind](rng, int(lengths[u]))

    geom = None
    snr = None
    if with_room:
        geom = np.zeros((n_utt, 1 + n_noise, 10), dtype=np.float32)
        for u in range(n_utt):
            dims, beta = fixed_room if fixed_room is not None else _random_room(rng)
            geom[u] = draw_geometry(rng, 1 + n_noise, dims, beta)
        snr = rng.uniform(snr_range[0], snr_range[1], size=(n_utt, n_noise)).astype(np.float32)

    alpha = rng.uniform(0.8, 1.2, size=n_utt).astype(np.float32)
    return Workload(name=name, seed=seed, offsets=offsets, speech=speech, noise=noise,
                    geom=geom, snr_db=snr, alpha=alpha, rir_len=rir_len)


def tiny(n_utt: int = 8, seconds: float = 1.0, rir_len: int = 4096, seed: int = 0) -> Workload:
    """8 x 1 s, one 5x4x3 m room with reflection 0.7, one white source at 10 dB."""
    n = int(round(seconds * FS))
    return _assemble("tiny", seed, [n] * n_utt, ["white"], rir_len, (10.0, 10.0),
                     fixed_room=(np.array([5.0, 4.0, 3.0]), 0.7))


def features_only(n_utt: int = 4096, seconds: float = 8.0, seed: int = 1) -> Workload:
    """Front end only: no room, no noise; isolates STFT + warped mel + power law."""
    n = int(round(seconds * FS))
    return _assemble("features", seed, [n] * n_utt, [], 0, (0.0, 0.0), with_room=False)


def batch(n_utt: int = 64, seconds: float = 4.0, rir_len: int = 8000, seed: int = 2) -> Workload:
    """Random rooms, 8000-tap RIRs, one Gaussian source at SNR ~ U[0, 20] dB."""
    n = int(round(seconds * FS))
    return _assemble("batch", seed, [n] * n_utt, ["white"], rir_len, (0.0, 20.0))


def varlen(n_utt: int = 256, rir_len: int = 16000, seed: int = 3,
           min_s: float = 1.0, max_s: float = 16.0) -> Workload:
    """Lengths ~ U[1, 16] s packed contiguously; white, pink and babble sources."""
    rng = np.random.default_rng([seed, 0x1E46])
    lengths = rng.integers(int(min_s * FS), int(max_s * FS) + 1, size=n_utt)
    return _assemble("varlen", seed, lengths, ["white", "pink", "babble"], rir_len, (0.0, 30.0))


def throughput(n_utt: int = 1024, seconds: float = 10.0, rir_len: int = 32768,
               seed: int = 4) -> Workload:
    """1024 x 10 s, 32768-tap RIRs, two independent noise sources at SNR ~ U[0, 20] dB."""
    n = int(round(seconds * FS))
    return _assemble("throughput", seed, [n] * n_utt, ["white", "pink"], rir_len, (0.0, 20.0))


WORKLOADS = {
    "tiny": tiny,
    "features": features_only,
    "batch": batch,
    "varlen": varlen,
    "throughput": throughput,
}
