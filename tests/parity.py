"""Comparators and device helpers shared by the GPU parity tests."""
import numpy as np

WAVE_TOL = 1e-4      # max-abs error <= WAVE_TOL * RMS of the oracle signal, per utterance
FEAT_TOL = 1e-3      # relative error of features, denominators floored at 1e-3 * RMS
RIR_TOL = 1e-5       # relative error of summed tap amplitudes
GAIN_TOL = 1e-4      # relative error of SNR gains


def wave_err(got, ref, offsets, silent_scale=None):
    """Largest per-utterance max|got - ref| / RMS(ref).

    An utterance whose reference is identically zero (it ends before the direct path arrives) has no RMS
    to scale by; with `silent_scale` (the signal that was convolved) the RMS of that utterance's input is
    the scale instead, since a transform-based convolution leaves rounding noise where the exact result is 0.
    """
    worst = 0.0
    for u in range(len(offsets) - 1):
        a, b = int(offsets[u]), int(offsets[u + 1])
        if b == a:
            continue
        rms = np.sqrt(np.mean(ref[a:b] ** 2))
        if rms == 0 and silent_scale is not None:
            rms = np.sqrt(np.mean(np.asarray(silent_scale[a:b], np.float64) ** 2))
        err = np.max(np.abs(got[a:b].astype(np.float64) - ref[a:b]))
        worst = max(worst, err / rms if rms > 0 else (0.0 if err == 0 else np.inf))
    return worst


def feat_err(got, ref):
    """max |got - ref| / max(|ref|, 1e-3 RMS(ref))."""
    if ref.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(ref ** 2))
    den = np.maximum(np.abs(ref), 1e-3 * rms)
    den = np.where(den > 0, den, 1.0)
    return float(np.max(np.abs(got.astype(np.float64) - ref) / den))


def rir_err(got, ref):
    """max |got - ref| / max(|ref|, 1e-6 max|ref|) over taps (all amplitudes are >= 0)."""
    den = np.maximum(np.abs(ref), 1e-6 * np.max(np.abs(ref)) if ref.size else 1.0)
    den = np.where(den > 0, den, 1.0)
    return float(np.max(np.abs(got.astype(np.float64) - ref) / den)) if ref.size else 0.0


def dev(a, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


class DeviceWorkload:
    """A workload's arrays resident on the GPU."""

    def __init__(self, w):
        import torch
        self.w = w
        self.speech = dev(w.speech)
        self.noise = None if w.noise is None else dev(w.noise)
        self.geom = None if w.geom is None else dev(w.geom)
        self.snr_db = None if w.snr_db is None else dev(w.snr_db)
        self.alpha = dev(w.alpha)
        self.frame_offsets = w.frame_offsets()
        self.n_frames = int(self.frame_offsets[-1])
        self.torch = torch

    def empty_feats(self):
        return self.torch.full((self.n_frames, self.w.frontend.n_mel), float("nan"),
                               dtype=self.torch.float32, device="cuda")


# ---- the oracle on many utterances at once (host processes; nothing here touches the GPU) ----

def _oracle_utterance(job):
    from oracle import aug_oracle as O
    s, conv, stft = job
    return O.pipeline_batch(s.offsets, s.speech, s.noise, s.geom, s.rir_len, s.fs, s.c, s.snr_db, s.alpha,
                            s.frontend, conv_method=conv, stft_method=stft)


def _oracle_rir_rows(job):
    from oracle import aug_oracle as O
    geom, rir_len, fs, c = job
    return O.rir_batch(geom, rir_len, fs, c)


def _pool(workers):
    # fresh interpreters ("spawn"): the parent has the GPU open, and a forked copy of it must not exist
    import multiprocessing as mp
    from concurrent.futures import ProcessPoolExecutor
    return ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn"))


def oracle_utterances(w, utts, conv="fft", stft="dft", workers=8):
    """pipeline_batch of the oracle for each listed utterance of workload w (one-utterance slices), in parallel."""
    jobs = [(w.slice([u]), conv, stft) for u in utts]
    with _pool(min(workers, max(1, len(jobs)))) as ex:
        return list(ex.map(_oracle_utterance, jobs))


def oracle_rirs(geom, rir_len, fs, c, workers=8):
    """rir_batch of the oracle over the rows of geom, in parallel; returns (h, tap_count)."""
    geom = np.asarray(geom, np.float32).reshape(-1, 10)
    jobs = [(geom[r:r + 1], rir_len, fs, c) for r in range(len(geom))]
    with _pool(min(workers, max(1, len(jobs)))) as ex:
        parts = list(ex.map(_oracle_rir_rows, jobs))
    return np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts])


def spread(n, count, extra=()):
    """`count` indices spread evenly over range(n), always with the first and the last, plus `extra`."""
    picks = set(int(round(i * (n - 1) / max(count - 1, 1))) for i in range(count)) | set(int(e) for e in extra)
    return sorted(picks)
