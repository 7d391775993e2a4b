"""CPU oracle for the augmentation + feature path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 NumPy statement of what the path computes: image-method
room impulse responses, causal convolution of every source with its RIR,
SNR-scaled mixing, framed DFT power spectrum, a bilinear-warped (VTLP) mel
filterbank and the power-law nonlinearity.  It exists so that the HIP kernels
can be checked against something that can be read against the paper by eye.
Only tests, the smoke check and the benchmark's CPU-baseline leg may import
it; the product path never does, and it imports nothing from the product.

What the paper fixes (Sec. 2.3): the bilinear warp of Eq. (1) with
omega_k = 2 pi k / K, one warp factor per utterance, power mel filterbank
energies, the exponent 1/15, room impulse responses computed on the fly, and
(Sec. 3) no peak normalisation and no feature clipping.  The image method,
the convolution, the SNR rule, the framing and the mel bank are only cited
there; the readings taken for them are written at each function.

Each function is the definition written out.  `method="fft"` variants use
numpy's FFT as a library step for sizes where the direct sums would take
hours; tests tie them to the direct forms on small shapes.

Every function below is pinned by CPU tests against closed forms or
independent formulas (none is "parity unpinned").  The paper prints no
end-to-end value; the composition `pipeline_batch` is pinned by the closed
form that rooms without reflections give (every response a single impulse
1/(4 pi r): the mixture is a sum of shifted, scaled inputs whose delays,
amplitudes, energies and gains can be worked out by hand).
"""
from __future__ import annotations

import math

import numpy as np

__all__ = [
    "frame_count", "rir_single", "rir_batch", "rir_mics_single", "rir_mics_batch", "convolve_direct", "convolve_fft",
    "convolve_at", "reverberate", "snr_gains", "convolve_mix_batch", "hamming",
    "dft_matrix", "stft_power", "bilinear_warp", "mel_edges_hz", "warped_mel_matrix",
    "dct2_matrix", "mel_epilogue", "vtlp_mel_batch", "pipeline_batch",
]


# --------------------------------------------------------------------------
# Room impulse response: image method (acoustic simulator, Sec. 2.3)
# --------------------------------------------------------------------------

def _axis_images(s: float, room: float, n_max: int):
    """Image coordinates of a source along one axis of a box [0, room].

    Mirror images of a point s between two parallel walls at 0 and `room` sit
    at (1 - 2q) s + 2 n room for q in {0, 1} and integer n; that image has been
    reflected |n - q| times by the wall at 0 and |n| times by the wall at
    `room`.  Returns (coordinates, reflection counts), fp64 / int64.
    """
    q = np.array([0, 1], dtype=np.int64)[:, None]
    n = np.arange(-n_max, n_max + 1, dtype=np.int64)[None, :]
    coord = (1.0 - 2.0 * q) * s + 2.0 * n * room
    count = np.abs(n - q) + np.abs(n)
    return coord.ravel(), count.ravel()


def rir_single(geom_row, rir_len: int, fs: float, c: float):
    """Image-method RIR of one source/microphone pair in a shoebox room.

    geom_row = [Lx, Ly, Lz, sx, sy, sz, mx, my, mz, beta] (fp32 values, widened
    exactly to fp64).  Reading taken where the paper only cites the simulator:
    one reflection coefficient beta for all six walls, every image source
    contributes a unit impulse at the nearest sample,
        h[round(d fs / c)] += beta^(number of reflections) / (4 pi d),
    d the image-to-microphone distance, rounding half up, all taps below
    `rir_len` kept, no order cap, no high-pass, no fractional delay.

    The tap index is taken in fp64 in this exact order so that it can be
    reproduced bit for bit:  d2 = (dx*dx + dy*dy) + dz*dz;  d = sqrt(d2);
    idx = floor(d * (fs / c) + 0.5), with fs / c one fp64 division of the two
    fp32 values.

    Returns (h fp64 [rir_len], tap_count int32 [rir_len]) where tap_count[n]
    is the number of images that landed on tap n.
    """
    g = np.asarray(geom_row, dtype=np.float32).astype(np.float64)
    room, src, mic, beta = g[0:3], g[3:6], g[6:9], g[9]
    k = np.float64(np.float32(fs)) / np.float64(np.float32(c))
    radius = rir_len / k                      # images farther than this cannot land below rir_len
    per_axis = []
    for a in range(3):
        n_max = int(math.ceil(radius / (2.0 * room[a]))) + 1
        coord, count = _axis_images(src[a], room[a], n_max)
        delta = coord - mic[a]
        per_axis.append((delta * delta, count))
    (dx2, cx), (dy2, cy), (dz2, cz) = per_axis

    h = np.zeros(rir_len, dtype=np.float64)
    tap_count = np.zeros(rir_len, dtype=np.int64)
    for ix in range(len(dx2)):
        d2 = (dx2[ix] + dy2[:, None]) + dz2[None, :]
        d = np.sqrt(d2)
        idx = np.floor(d * k + 0.5).astype(np.int64)
        refl = cx[ix] + cy[:, None] + cz[None, :]
        keep = idx < rir_len
        if not keep.any():
            continue
        amp = np.power(beta, refl[keep].astype(np.float64)) / (4.0 * np.pi * d[keep])
        h += np.bincount(idx[keep], weights=amp, minlength=rir_len)
        tap_count += np.bincount(idx[keep], minlength=rir_len)
    return h, tap_count.astype(np.int32)


def rir_batch(geom, rir_len: int, fs: float, c: float):
    """RIRs for geom [n_rir, 10]; returns (h [n_rir, L] fp64, tap_count [n_rir, L] int32)."""
    geom = np.asarray(geom, dtype=np.float32).reshape(-1, 10)
    h = np.zeros((len(geom), rir_len), dtype=np.float64)
    cnt = np.zeros((len(geom), rir_len), dtype=np.int32)
    for r in range(len(geom)):
        h[r], cnt[r] = rir_single(geom[r], rir_len, fs, c)
    return h, cnt


def rir_mics_single(geom_row, mics, rir_len: int, fs: float, c: float):
    """Responses from one source to several microphones in the same room.

    The recording device of Sec. 4 carries two microphones 6.8 cm apart; a
    simulated counterpart needs one response per microphone for the same room
    and source.  The image sources of a room do not depend on where the
    microphone is, so they are listed once (per axis: coordinate and reflection
    count) and every microphone sums its own response over that one list, tap
    rule and amplitude as in `rir_single`.  geom_row's own microphone columns
    are not used.  mics = [K, 3] (fp32 values).

    Every image that can land below `rir_len` for any of the microphones must
    be on the list: a microphone at most `room` away from the source along an
    axis sees image n at a distance of at least (2|n| - 2) room, so the same
    per-axis bound as for one microphone holds for each of them.

    Returns (h fp64 [K, rir_len], tap_count int32 [K, rir_len]).
    """
    g = np.asarray(geom_row, dtype=np.float32).astype(np.float64)
    mics = np.asarray(mics, dtype=np.float32).astype(np.float64).reshape(-1, 3)
    room, src, beta = g[0:3], g[3:6], g[9]
    k = np.float64(np.float32(fs)) / np.float64(np.float32(c))
    radius = rir_len / k
    images = []                                   # the shared list: per axis (coordinates, reflection counts)
    for a in range(3):
        n_max = int(math.ceil(radius / (2.0 * room[a]))) + 1
        images.append(_axis_images(src[a], room[a], n_max))
    (px, cx), (py, cy), (pz, cz) = images
    refl_yz = cy[:, None] + cz[None, :]

    h = np.zeros((len(mics), rir_len), dtype=np.float64)
    tap_count = np.zeros((len(mics), rir_len), dtype=np.int64)
    for m, mic in enumerate(mics):
        dx2 = (px - mic[0]) * (px - mic[0])
        dy2 = (py - mic[1]) * (py - mic[1])
        dz2 = (pz - mic[2]) * (pz - mic[2])
        for ix in range(len(px)):
            d = np.sqrt((dx2[ix] + dy2[:, None]) + dz2[None, :])
            idx = np.floor(d * k + 0.5).astype(np.int64)
            keep = idx < rir_len
            if not keep.any():
                continue
            amp = np.power(beta, (cx[ix] + refl_yz)[keep].astype(np.float64)) / (4.0 * np.pi * d[keep])
            h[m] += np.bincount(idx[keep], weights=amp, minlength=rir_len)
            tap_count[m] += np.bincount(idx[keep], minlength=rir_len)
    return h, tap_count.astype(np.int32)


def rir_mics_batch(geom, mics, rir_len: int, fs: float, c: float):
    """geom [n_rir, 10], mics [n_rir, K, 3]; returns (h [n_rir, K, L] fp64, tap_count [n_rir, K, L] int32)."""
    geom = np.asarray(geom, dtype=np.float32).reshape(-1, 10)
    mics = np.asarray(mics, dtype=np.float32)
    mics = mics.reshape(len(geom), -1, 3)
    h = np.zeros((len(geom), mics.shape[1], rir_len), dtype=np.float64)
    cnt = np.zeros((len(geom), mics.shape[1], rir_len), dtype=np.int32)
    for r in range(len(geom)):
        h[r], cnt[r] = rir_mics_single(geom[r], mics[r], rir_len, fs, c)
    return h, cnt


# --------------------------------------------------------------------------
# Reverberation and additive noise at a target SNR
# --------------------------------------------------------------------------

def convolve_direct(x, h):
    """y[n] = sum_{k <= n, k < len(h)} h[k] x[n-k] for n < len(x): causal, input length kept.

    The propagation delay stays in the signal and the reverberation tail past
    the end of the input is dropped.  numpy.convolve evaluates the sum directly
    in the time domain.
    """
    x = np.asarray(x, dtype=np.float64)
    h = np.asarray(h, dtype=np.float64)
    if len(x) == 0:
        return np.zeros(0)
    return np.convolve(x, h)[: len(x)]


def convolve_fft(x, h):
    """Same result as convolve_direct through one zero-padded fp64 FFT (library step)."""
    x = np.asarray(x, dtype=np.float64)
    h = np.asarray(h, dtype=np.float64)
    if len(x) == 0:
        return np.zeros(0)
    n = len(x) + len(h) - 1
    nfft = 1 << (n - 1).bit_length()
    return np.fft.irfft(np.fft.rfft(x, nfft) * np.fft.rfft(h, nfft), nfft)[: len(x)]


def convolve_at(x, h, positions):
    """The direct sum of convolve_direct at the listed output positions only."""
    x = np.asarray(x, dtype=np.float64)
    h = np.asarray(h, dtype=np.float64)
    out = np.zeros(len(positions))
    for i, n in enumerate(positions):
        k_hi = min(int(n), len(h) - 1)
        k = np.arange(0, k_hi + 1)
        out[i] = np.dot(h[k], x[int(n) - k])
    return out


def reverberate(offsets, speech, noise, rir, method="direct"):
    """Convolve every source of every utterance with its own RIR.

    offsets int64 [B+1]; speech [total]; noise [J, total] or None;
    rir [B, 1+J, L].  Returns y [1+J, total] fp64, row 0 the speech.
    """
    conv = {"direct": convolve_direct, "fft": convolve_fft}[method]
    offsets = np.asarray(offsets, dtype=np.int64)
    n_utt = len(offsets) - 1
    n_noise = 0 if noise is None else len(noise)
    y = np.zeros((1 + n_noise, int(offsets[-1])), dtype=np.float64)
    for u in range(n_utt):
        a, b = int(offsets[u]), int(offsets[u + 1])
        y[0, a:b] = conv(speech[a:b], rir[u, 0])
        for j in range(n_noise):
            y[1 + j, a:b] = conv(noise[j][a:b], rir[u, 1 + j])
    return y


def snr_gains(energy_speech, energy_noise, snr_db):
    """Gain per noise source so that 10 log10(E_speech / (g^2 E_noise)) = snr_db.

    Energies are those of the reverberated signals over the utterance; a
    silent speech or noise signal gets gain 0.
    """
    e0 = np.float64(energy_speech)
    en = np.asarray(energy_noise, dtype=np.float64)
    snr = np.asarray(snr_db, dtype=np.float32).astype(np.float64)
    g = np.zeros_like(en)
    ok = (e0 > 0) & (en > 0)
    g[ok] = np.sqrt(e0 / (en[ok] * np.power(10.0, snr[ok] / 10.0)))
    return g


def convolve_mix_batch(offsets, speech, noise, rir, snr_db, method="direct"):
    """Reverberate, then add each noise at its own SNR relative to the reverberated speech.

    Returns (mixed fp64 [total], gains fp64 [B, J]).
    """
    offsets = np.asarray(offsets, dtype=np.int64)
    n_utt = len(offsets) - 1
    y = reverberate(offsets, speech, noise, rir, method)
    n_noise = y.shape[0] - 1
    mixed = y[0].copy()
    gains = np.zeros((n_utt, n_noise), dtype=np.float64)
    for u in range(n_utt):
        a, b = int(offsets[u]), int(offsets[u + 1])
        if n_noise == 0:
            continue
        e0 = np.sum(y[0, a:b] ** 2)
        en = np.array([np.sum(y[1 + j, a:b] ** 2) for j in range(n_noise)])
        gains[u] = snr_gains(e0, en, np.asarray(snr_db)[u])
        for j in range(n_noise):
            mixed[a:b] += gains[u, j] * y[1 + j, a:b]
    return mixed, gains


# --------------------------------------------------------------------------
# Front end: STFT power, VTLP-warped mel bank (Eq. 1), power law
# --------------------------------------------------------------------------

def frame_count(n_samples: int, win: int, hop: int) -> int:
    """Frames that fit entirely inside the signal (no padding): 1 + (N - win) // hop."""
    return 0 if n_samples < win else 1 + (int(n_samples) - win) // hop


def hamming(win: int):
    """Symmetric Hamming window 0.54 - 0.46 cos(2 pi i / (win - 1))."""
    i = np.arange(win, dtype=np.float64)
    return 0.54 - 0.46 * np.cos(2.0 * np.pi * i / (win - 1))


def dft_matrix(win: int, nfft: int):
    """exp(-j 2 pi k i / nfft) for bins k = 0..nfft/2 and samples i < win."""
    k = np.arange(nfft // 2 + 1, dtype=np.float64)[:, None]
    i = np.arange(win, dtype=np.float64)[None, :]
    return np.exp(-2j * np.pi * k * i / nfft)


def stft_power(x, win: int, hop: int, nfft: int, method="dft"):
    """|DFT_nfft(x[t hop : t hop + win] * hamming)|^2 for bins 0..nfft/2, frames as rows.

    No centring, no pre-emphasis, no dither, no DC removal, no peak
    normalisation (Sec. 3), no 1/nfft scaling.  `method="dft"` multiplies by
    the DFT matrix; "fft" calls numpy's rfft on the zero-padded frames.
    """
    x = np.asarray(x, dtype=np.float64)
    n_frames = frame_count(len(x), win, hop)
    if n_frames == 0:
        return np.zeros((0, nfft // 2 + 1))
    idx = np.arange(n_frames)[:, None] * hop + np.arange(win)[None, :]
    frames = x[idx] * hamming(win)[None, :]
    if method == "dft":
        spec = frames @ dft_matrix(win, nfft).T
    else:
        spec = np.fft.rfft(frames, nfft, axis=1)
    return spec.real ** 2 + spec.imag ** 2


def bilinear_warp(omega, alpha):
    """Eq. (1): omega' = omega + 2 atan((1 - alpha) sin omega / (1 - (1 - alpha) cos omega))."""
    omega = np.asarray(omega, dtype=np.float64)
    a = 1.0 - np.float64(alpha)
    return omega + 2.0 * np.arctan(a * np.sin(omega) / (1.0 - a * np.cos(omega)))


def _hz_to_mel(f):
    return 2595.0 * np.log10(1.0 + np.asarray(f, dtype=np.float64) / 700.0)


def _mel_to_hz(m):
    return 700.0 * (np.power(10.0, np.asarray(m, dtype=np.float64) / 2595.0) - 1.0)


def mel_edges_hz(n_mel: int, f_lo: float, f_hi: float):
    """n_mel + 2 band edges equally spaced on the mel scale 2595 log10(1 + f/700)."""
    return _mel_to_hz(np.linspace(_hz_to_mel(f_lo), _hz_to_mel(f_hi), n_mel + 2))


def warped_mel_matrix(alpha, n_mel: int, nfft: int, fs: float, f_lo: float, f_hi: float):
    """W[m, k] = Tri_m(f'_k): unit-peak triangles evaluated at the warped bin frequencies.

    Eq. (1) names omega_k = 2 pi k / K the input and omega'_k the output
    frequency, so the energy measured in bin k is placed at
    f'_k = omega'_k fs / (2 pi) and the fixed triangular filters are read
    there.  Tri_m rises from edge m to edge m+1 and falls to edge m+2.
    """
    alpha = np.float64(np.float32(alpha))
    e = mel_edges_hz(n_mel, f_lo, f_hi)
    k = np.arange(nfft // 2 + 1, dtype=np.float64)
    f_warp = bilinear_warp(2.0 * np.pi * k / nfft, alpha) * fs / (2.0 * np.pi)
    w = np.zeros((n_mel, len(k)))
    for m in range(n_mel):
        rise = (f_warp - e[m]) / (e[m + 1] - e[m])
        fall = (e[m + 2] - f_warp) / (e[m + 2] - e[m + 1])
        w[m] = np.maximum(0.0, np.minimum(rise, fall))
    return w


def dct2_matrix(n_ceps: int, n_mel: int):
    """Orthonormal DCT-II: D[q, m] = s_q cos(pi q (m + 1/2) / M), s_0 = sqrt(1/M), s_q = sqrt(2/M)."""
    q = np.arange(n_ceps, dtype=np.float64)[:, None]
    m = np.arange(n_mel, dtype=np.float64)[None, :]
    d = np.cos(np.pi * q * (m + 0.5) / n_mel) * np.sqrt(2.0 / n_mel)
    d[0] *= np.sqrt(0.5)
    return d


def mel_epilogue(energies, fe):
    """What is kept of the mel energies E[t, m] (Sec. 2.3 names all three).

    "power" (the paper's feature): E^power, 0 -> 0.  "log": the conventional log-mel, natural logarithm
    of max(E, log_floor).  "mfcc": the first n_ceps coefficients of the orthonormal DCT-II of the log-mel
    vector (no liftering, no energy term).  The floor and the DCT normalisation are readings: the paper
    only names these features as the ones it replaces.
    """
    kind = getattr(fe, "feature", "power")
    if kind == "power":
        return np.power(energies, fe.power)
    logmel = np.log(np.maximum(energies, fe.log_floor))
    if kind == "log":
        return logmel
    if kind == "mfcc":
        return logmel @ dct2_matrix(fe.n_ceps, fe.n_mel).T
    raise ValueError(f"unknown feature kind {kind!r}")


def vtlp_mel_batch(offsets, wave, alpha, fe, method="dft"):
    """Mel features [total_frames, feature_dim] fp64 from the warped mel energies W_alpha P_t.

    `fe` has fields fs, win, hop, nfft, n_mel, f_lo, f_hi, power and, optionally, feature, n_ceps,
    log_floor (see mel_epilogue).  One warp factor per utterance (Sec. 2.3); the paper's feature is
    the power law with exponent 1/15.
    """
    offsets = np.asarray(offsets, dtype=np.int64)
    rows = []
    for u in range(len(offsets) - 1):
        x = np.asarray(wave[int(offsets[u]):int(offsets[u + 1])], dtype=np.float64)
        p = stft_power(x, fe.win, fe.hop, fe.nfft, method)
        w = warped_mel_matrix(alpha[u], fe.n_mel, fe.nfft, fe.fs, fe.f_lo, fe.f_hi)
        rows.append(mel_epilogue(p @ w.T, fe))
    if not rows:
        dim = fe.n_ceps if getattr(fe, "feature", "power") == "mfcc" else fe.n_mel
        return np.zeros((0, dim))
    return np.concatenate(rows, axis=0)


def pipeline_batch(offsets, speech, noise, geom, rir_len, fs, c, snr_db, alpha, fe,
                   conv_method="direct", stft_method="dft"):
    """RIR synthesis -> reverberation -> SNR mix -> warped power-mel features.

    Returns dict(rir, tap_count, mixed, gains, feats), all fp64 except tap_count.
    """
    offsets = np.asarray(offsets, dtype=np.int64)
    n_utt = len(offsets) - 1
    geom = np.asarray(geom, dtype=np.float32).reshape(n_utt, -1, 10)
    n_src = geom.shape[1]
    h, cnt = rir_batch(geom.reshape(-1, 10), rir_len, fs, c)
    h = h.reshape(n_utt, n_src, rir_len)
    mixed, gains = convolve_mix_batch(offsets, speech, noise, h, snr_db, conv_method)
    feats = vtlp_mel_batch(offsets, mixed, alpha, fe, stft_method)
    return dict(rir=h, tap_count=cnt.reshape(n_utt, n_src, rir_len), mixed=mixed,
                gains=gains, feats=feats)
