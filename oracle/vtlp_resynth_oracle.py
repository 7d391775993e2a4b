"""CPU oracle for VTLP by waveform resynthesis.  TEST INFRASTRUCTURE ONLY.

Sec. 2.3 applies vocal tract length perturbation to the input *waveform*, before
the acoustic simulator: the signal is analysed in short frames, each frame's
spectrum is moved along the frequency axis by the bilinear rule of Eq. (1) with
one warp factor per utterance, and the frames are put back together by
overlap-add.  The paper fixes Eq. (1), omega_k = 2 pi k / K, the per-utterance
factor and (Sec. 4, Table 2) the best window length, 50 ms; the rest of the algorithm is
in a cited paper only, so the steps below are readings, each stated where it is
taken:

  V-1  frames of W = 800 samples (50 ms at 16 kHz) with the periodic Hann window
       w[i] = 0.5 - 0.5 cos(2 pi i / W), hop W/2; frame t is centred on sample
       t W/2 and covers [t W/2 - W/2, t W/2 + W/2); samples outside the utterance
       are zero; t = 0 .. floor((N-1)/(W/2)) + 1, so that every sample of the
       utterance lies in exactly two frames and their window weights add up to 1.
  V-2  K = 2048-point DFT of the frame arranged around time zero (sample at
       offset tau from the frame centre sits at index tau mod K), which keeps the
       phase of neighbouring bins close and makes interpolation between them
       meaningful.
  V-3  output bin k' takes the input spectrum at the frequency that Eq. (1) maps
       onto it: omega = omega' - 2 atan(a sin omega' / (1 + a cos omega')),
       a = 1 - alpha (the inverse of Eq. (1), which is Eq. (1) with a -> -a), read
       by linear interpolation of the complex spectrum between the two nearest
       bins.  Bins 0 and K/2 map onto themselves.
  V-4  inverse K-point DFT (with its 1/K), all K samples overlap-added at the
       frame's position; no synthesis window, no gain correction; the output has
       the input's length.  alpha = 1 therefore returns the input.

Everything is fp64 NumPy.  `method="dft"` writes the K-point transform pair of
V-2 / V-4 out as the sums that define it; the default `method="fft"` calls
numpy's FFT as a library step (a test ties the two together).  Pins are in
tests/test_oracle_vtlp_resynth.py (inverse warp against Eq. (1) itself, identity
at alpha = 1, where a pure tone lands, linearity, hop-shift covariance); no
function here is "parity unpinned".  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this module; it imports nothing from
the product.
"""
from __future__ import annotations

import numpy as np

__all__ = ["hann_periodic", "resynth_frame_count", "inverse_warp", "source_bins",
           "warp_spectrum", "dft_half", "idft_real", "vtlp_resynth", "vtlp_resynth_batch"]


def hann_periodic(win: int):
    """w[i] = 0.5 - 0.5 cos(2 pi i / W): w[i] + w[i + W/2] = 1 (V-1)."""
    i = np.arange(win, dtype=np.float64)
    return 0.5 - 0.5 * np.cos(2.0 * np.pi * i / win)


def resynth_frame_count(n_samples: int, hop: int) -> int:
    """Frames centred on 0, hop, 2 hop, ... up to the first centre at or past the last sample (V-1)."""
    return 0 if n_samples <= 0 else (n_samples - 1) // hop + 2


def inverse_warp(omega_out, alpha):
    """The input frequency that Eq. (1) sends to omega_out (V-3)."""
    w = np.asarray(omega_out, dtype=np.float64)
    a = 1.0 - np.float64(alpha)
    return w - 2.0 * np.arctan(a * np.sin(w) / (1.0 + a * np.cos(w)))


def source_bins(alpha, nfft: int):
    """Fractional input bin read by each output bin k' = 0..K/2 (V-3)."""
    k_out = np.arange(nfft // 2 + 1, dtype=np.float64)
    kappa = inverse_warp(2.0 * np.pi * k_out / nfft, alpha) * nfft / (2.0 * np.pi)
    return np.clip(kappa, 0.0, nfft / 2.0)


def warp_spectrum(X, alpha, nfft: int):
    """Y[k'] = (1 - f) X[j] + f X[j + 1], j = floor(kappa), f = kappa - j (V-3)."""
    kappa = source_bins(alpha, nfft)
    j = np.minimum(np.floor(kappa).astype(np.int64), nfft // 2 - 1)
    f = kappa - j
    return (1.0 - f) * X[j] + f * X[j + 1]


def dft_half(g):
    """X[k] = sum_n g[n] exp(-2 pi i k n / K), k = 0..K/2, as the sum itself (V-2)."""
    g = np.asarray(g, dtype=np.float64)
    nfft = g.shape[0]
    k = np.arange(nfft // 2 + 1, dtype=np.float64)[:, None]
    n = np.arange(nfft, dtype=np.float64)[None, :]
    return np.exp(-2j * np.pi * k * n / nfft) @ g


def idft_real(Y, nfft: int):
    """y[n] = Re (1/K) sum_{k<K} Z[k] exp(+2 pi i k n / K), Z the Hermitian extension of Y[0..K/2] (V-4)."""
    Y = np.asarray(Y, dtype=np.complex128)
    Z = np.concatenate([Y, np.conj(Y[-2:0:-1])])
    k = np.arange(nfft, dtype=np.float64)[None, :]
    n = np.arange(nfft, dtype=np.float64)[:, None]
    return np.real(np.exp(2j * np.pi * k * n / nfft) @ Z) / nfft


def vtlp_resynth(x, alpha, win: int = 800, nfft: int = 2048, method: str = "fft"):
    """One utterance through analysis, warp and overlap-add (V-1 .. V-4)."""
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[0]
    half = win // 2
    w = hann_periodic(win)
    out = np.zeros(n, dtype=np.float64)
    tau = np.arange(-nfft // 2, nfft // 2)
    for t in range(resynth_frame_count(n, half)):
        centre = t * half
        idx = centre - half + np.arange(win)
        ok = (idx >= 0) & (idx < n)
        frame = np.zeros(win, dtype=np.float64)
        frame[ok] = x[idx[ok]] * w[ok]
        g = np.zeros(nfft, dtype=np.float64)
        g[:half] = frame[half:]                  # offsets 0 .. W/2 - 1
        g[nfft - half:] = frame[:half]           # offsets -W/2 .. -1
        if method == "dft":
            y = idft_real(warp_spectrum(dft_half(g), alpha, nfft), nfft)
        else:
            y = np.fft.irfft(warp_spectrum(np.fft.rfft(g), alpha, nfft), nfft)
        pos = centre + tau
        ok = (pos >= 0) & (pos < n)
        out[pos[ok]] += y[tau[ok] % nfft]
    return out


def vtlp_resynth_batch(offsets, wave, alpha, win: int = 800, nfft: int = 2048):
    """Packed batch: utterance u is wave[offsets[u]:offsets[u+1]] with its own alpha[u]."""
    offsets = np.asarray(offsets, dtype=np.int64)
    out = np.zeros(int(offsets[-1]), dtype=np.float64)
    for u in range(len(offsets) - 1):
        a, b = int(offsets[u]), int(offsets[u + 1])
        out[a:b] = vtlp_resynth(wave[a:b], alpha[u], win, nfft)
    return out
