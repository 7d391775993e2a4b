#!/usr/bin/env python3
"""Throughput of the augmentation + feature path on one MI355X.

A step is one aug_pipeline_batch call (impulse responses, reverberation, SNR mix,
warped power-mel features) over one batch of seeded synthetic utterances that is
already resident in HBM.  Prints one JSON line with the whole-call throughput in
audio-seconds per second on the variable-length workload, the roofline of its dominant
kernel (timed with HIP events on the library's stream inside the timed region), the
same figures for all five workloads (`per_config`), the step time when every call
brings a batch with new lengths (`rotating`), and the CPU oracle timed on a bounded
sample of the same workload on all host cores.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "augmented audio-sec/sec (RIR+conv+mix+VTLP mel) on 1 GPU"
METRIC_BY_VTLP = {"mel": METRIC,
                  "waveform": "augmented audio-sec/sec (waveform VTLP+RIR+conv+mix+mel) on 1 GPU",
                  "waveform-only": "waveform-VTLP audio-sec/sec on 1 GPU"}
PEAK_HBM_GBS = 8000.0
PEAK_FP32_TFLOPS = 157.3      # vector fp32 with packed instructions; plain FMAs, all this build issues, reach 78.6
PEAK_FP64_TFLOPS = 78.6
RIR_FLOP_PER_IMAGE = 12.0     # 2 add, sqrt, mul, add, floor, table product, divide, scale, accumulate ...
KERNEL_OF_STAGE = {"rir": "rir_image_kernel", "convolve": "convolve_kernel", "mel": "mel_kernel",
                   "mix": "mix_kernel", "rir_spectrum": "rir_spectrum_kernel", "vtlp": "vtlp_resynth_kernel"}
# timed steps per workload for the per-config figures (about a second of GPU time each)
PER_CONFIG_STEPS = {"tiny": 300, "features": 100, "batch": 300, "varlen": 200, "throughput": 30}

# HBM bytes per launch (read + written) of each stage's kernel, from the rocprofv3 FETCH_SIZE / WRITE_SIZE
# runs summarised in profiles/hbm_traffic_<workload>.md, scaled there by a 1 GiB copy.  They describe the
# kernel sources with this digest only; for any other sources `traffic` is reported as null.
RECORDED_TRAFFIC = {
    "digest": "b10178e637ae96d5",
    "varlen": {"rir": 144776913, "rir_spectrum": 201797926, "convolve": 1254849701, "mel": 617857198},
    "throughput": {"rir": 782242713, "rir_spectrum": 1213474671, "convolve": 13819990189, "mel": 2201970965},
}


def kernel_source_digest() -> str:
    """Digest of the device code (kernels, their launchers and argument structures; not the host entry
    points) with comments and white space removed."""
    import glob
    import hashlib
    import re
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_1912_11040_amd", "csrc", "*"))):
        if f.endswith(("_kernels.hip", ".h")):
            with open(f) as fh:
                text = fh.read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            text = re.sub(r"//[^\n]*", "", text)
            h.update(os.path.basename(f).encode())
            h.update("".join(text.split()).encode())
    return h.hexdigest()[:16]


def recorded_traffic(workload: str, stage: str):
    if kernel_source_digest() != RECORDED_TRAFFIC["digest"]:
        return None
    return RECORDED_TRAFFIC.get(workload, {}).get(stage)


def describe(w) -> str:
    n = w.lengths()
    return (f"{w.name}: {w.n_utt} utterances, {n.min() / w.fs:.1f}-{n.max() / w.fs:.1f} s at 16 kHz fp32 "
            f"({w.audio_seconds:.0f} audio-s), {w.n_noise} noise sources, RIR {w.rir_len} taps, "
            f"seed {w.seed}")


def conv_flop_per_sample(rir_len: int) -> float:
    """One forward and one inverse real FFT of nfft = next pow2 >= 2 L plus the spectrum product,
    per output sample of a classical overlap-save block (2.5 nfft log2 nfft flop per real FFT)."""
    nfft = 1 << (2 * rir_len - 1).bit_length()
    return (2 * 2.5 * nfft * math.log2(nfft) + 6 * (nfft / 2 + 1)) / (nfft - rir_len + 1)


def stage_work(w, n_images: float):
    """Algorithmic work of each stage for one step: (bound, amount).  `n_images` is the number of image
    sources the image-sum kernel is charged with (bench.py passes the number it actually walks)."""
    n_src = 1 + w.n_noise
    frames = int(w.frame_offsets()[-1])
    fe = w.frontend
    n_len = w.lengths()
    work = {"mel": ("hbm", 4.0 * w.total + 4.0 * fe.n_mel * frames)}
    # waveform VTLP: two 2048-point real transforms, the window and two interpolated bins per output pair, per frame
    vtlp_frames = float(np.sum((n_len[n_len > 0] - 1) // 400 + 2))
    work["vtlp"] = ("alu32", vtlp_frames * (2 * 2.5 * 2048 * 11 + 800 + 8 * 1025))
    if w.geom is not None:
        # the timed call does not materialise the mixture: the front end reads every reverberated source
        # and scales it on the way in; what is left of the mix stage is the gain kernel (no roofline line)
        work["mel"] = ("hbm", 4.0 * w.total * n_src + 4.0 * fe.n_mel * frames)
        work["rir"] = ("alu", RIR_FLOP_PER_IMAGE * n_images)
        work["convolve"] = ("alu32", conv_flop_per_sample(w.rir_len) * w.total * n_src)
        work["rir_spectrum"] = ("alu32", 2.5 * (2 * w.rir_len) * math.log2(2 * w.rir_len) * w.n_utt * n_src)
    return work


def roofline_for(stage: str, work, ms: float):
    bound, amount = work[stage]
    sec = ms * 1e-3
    if bound == "hbm":
        achieved, peak, unit, b = amount / sec / 1e9, PEAK_HBM_GBS, "GB/s", "hbm"
    elif bound == "alu":
        achieved, peak, unit, b = amount / sec / 1e12, PEAK_FP64_TFLOPS, "TFLOP/s", "alu"
    else:
        achieved, peak, unit, b = amount / sec / 1e12, PEAK_FP32_TFLOPS, "TFLOP/s", "alu"
    frac = achieved / peak
    if not frac <= 1.0:
        raise RuntimeError(f"roofline fraction {frac:.3f} of stage {stage} exceeds 1: the work model charges "
                           "the kernel with work it does not do")
    return {"bound": b, "achieved": achieved, "peak": peak, "unit": unit, "frac": frac, "traffic": None}


# ---- CPU baseline: the oracle as it stands, one process per host core ----

def _oracle_job(job):
    """One utterance through the oracle in a worker process (one thread); returns (seconds, audio seconds)."""
    s, vtlp, fft = job
    from oracle import aug_oracle as O
    try:
        from threadpoolctl import threadpool_limits
    except Exception:                                  # pragma: no cover
        import contextlib
        threadpool_limits = lambda limits: contextlib.nullcontext()
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        if vtlp != "mel":
            from oracle import vtlp_resynth_oracle as V
            import dataclasses
            warped = V.vtlp_resynth_batch(s.offsets, s.speech, s.alpha)
            s = dataclasses.replace(s, speech=warped.astype(np.float32), alpha=np.ones_like(s.alpha))
        if vtlp == "waveform-only":
            pass
        elif s.geom is not None:
            O.pipeline_batch(s.offsets, s.speech, s.noise, s.geom, s.rir_len, s.fs, s.c, s.snr_db,
                             s.alpha, s.frontend, conv_method="fft" if fft else "direct",
                             stft_method="fft" if fft else "dft")
        else:
            O.vtlp_mel_batch(s.offsets, s.speech, s.alpha, s.frontend, "fft" if fft else "dft")
        return time.perf_counter() - t0, s.audio_seconds


def cpu_baseline(w, budget_s: float = 12.0, vtlp: str = "mel", fft: bool = False):
    """The oracle, unchanged, on every host core this process may use: one worker process per core
    (fresh interpreters, one thread each), utterances of the workload handed out one at a time from the
    first on, for about `budget_s` seconds of wall time.  fft=True times the oracle's own FFT forms
    (fp64 numpy FFT convolution and STFT) instead of its direct sums."""
    import multiprocessing as mp
    from concurrent.futures import FIRST_COMPLETED, ProcessPoolExecutor, wait
    # the cores this process may use, capped by the machine's per-job CPU share where it states one
    cores = len(os.sched_getaffinity(0))
    share = os.environ.get("OMP_NUM_THREADS", "")
    if share.isdigit() and int(share) > 0:
        cores = min(cores, int(share))
    done_audio, done_n, pending = 0.0, 0, set()
    with ProcessPoolExecutor(max_workers=cores, mp_context=mp.get_context("spawn")) as ex:
        list(ex.map(abs, range(cores)))                # workers up and imported before the clock starts
        t0 = time.perf_counter()
        nxt = 0
        while True:
            while len(pending) < cores and nxt < w.n_utt and time.perf_counter() - t0 < budget_s:
                pending.add(ex.submit(_oracle_job, (w.slice([nxt]), vtlp, fft)))
                nxt += 1
            if not pending:
                break
            finished, pending = wait(pending, return_when=FIRST_COMPLETED)
            for f in finished:
                done_audio += f.result()[1]
                done_n += 1
        dt = time.perf_counter() - t0
    return {"value": done_audio / dt, "unit": "audio-s/s", "cores": cores, "kind": "oracle",
            "sample": f"first {done_n} utterance(s) of the workload ({done_audio:.1f} audio-s), one per worker "
                      f"process at a time on {cores} cores, "
                      + ("fp64 FFT convolution + FFT front end" if fft else
                         "direct time-domain convolution + DFT-matrix front end") + f", {dt:.1f} s of wall time"}


# ---- GPU side ----

class DeviceBatch:
    """A workload's arrays in HBM, its output buffer and the step that the benchmark times."""

    def __init__(self, w, aug, vtlp="mel"):
        import torch
        dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
        self.w, self.aug, self.vtlp = w, aug, vtlp
        self.offsets = np.ascontiguousarray(w.offsets, dtype=np.int64)
        self.speech, self.noise, self.geom = dev(w.speech), dev(w.noise), dev(w.geom)
        self.snr, self.alpha = dev(w.snr_db), dev(w.alpha)
        self.foff = w.frame_offsets()
        self.feats = torch.empty((int(self.foff[-1]), w.frontend.n_mel), dtype=torch.float32, device="cuda")
        self.full = w.geom is not None
        self.warped = torch.empty_like(self.speech) if vtlp != "mel" else None
        self.ones = torch.ones_like(self.alpha)

    def step(self, aug=None):
        aug, w = aug or self.aug, self.w
        if self.vtlp == "waveform-only":
            aug.aug_vtlp_resynth_batch(self.offsets, self.speech, self.alpha, self.warped)
            return
        x, a = self.speech, self.alpha
        if self.vtlp == "waveform":
            aug.aug_vtlp_resynth_batch(self.offsets, self.speech, self.alpha, self.warped)
            x, a = self.warped, self.ones
        if self.full:
            aug.aug_pipeline_batch(self.offsets, x, self.noise, self.geom, w.rir_len, w.fs, w.c, self.snr, a,
                                   w.frontend, self.foff, self.feats)
        else:
            aug.aug_vtlp_mel_batch(self.offsets, x, a, w.frontend, self.foff, self.feats)

    def trimmed(self, k: int):
        """The same batch with every utterance 37 k samples shorter, repacked: other offsets, same rooms."""
        import copy
        import torch
        w = self.w
        cut = 37 * k
        lens = np.maximum(w.lengths() - cut, 0)
        off = np.zeros(w.n_utt + 1, dtype=np.int64)
        np.cumsum(lens, out=off[1:])
        idx = torch.from_numpy(np.concatenate([np.arange(w.offsets[u], w.offsets[u] + lens[u])
                                               for u in range(w.n_utt)])).cuda()
        b = copy.copy(self)
        b.offsets = off
        b.speech = self.speech[idx].contiguous()
        b.noise = None if self.noise is None else self.noise[:, idx].contiguous()
        fe = w.frontend
        t = np.where(lens >= fe.win, 1 + (lens - fe.win) // fe.hop, 0)
        b.foff = np.concatenate([[0], np.cumsum(t)]).astype(np.int64)
        b.feats = torch.empty((int(b.foff[-1]), fe.n_mel), dtype=torch.float32, device="cuda")
        b.warped = None if self.warped is None else torch.empty_like(b.speech)
        return b


def count_images(batch):
    """(images of the definition with tap < L, images the amplitude kernel walks), both counted by the
    library in untimed passes: tap_count_out summed, and the instrumented instantiation's counter."""
    import torch
    w, aug = batch.w, batch.aug
    if not batch.full or batch.vtlp == "waveform-only":
        return 0.0, 0.0
    n_rir = w.n_utt * (1 + w.n_noise)
    chunk = max(1, min(n_rir, (1 << 28) // w.rir_len))
    g2 = batch.geom.reshape(-1, 10)
    defined, visited = 0.0, 0.0
    for a in range(0, n_rir, chunk):
        b = min(n_rir, a + chunk)
        h = torch.empty((b - a, w.rir_len), dtype=torch.float32, device="cuda")
        cnt = torch.empty((b - a, w.rir_len), dtype=torch.int32, device="cuda")
        rows = g2[a:b].contiguous()
        aug.aug_rir_batch(rows, w.rir_len, w.fs, w.c, h, cnt)
        defined += float(cnt.sum(dtype=torch.int64).item())
        visited += float(aug.aug_rir_visited_images(rows, w.rir_len, w.fs, w.c, h))
        del h, cnt
    return defined, visited


def timed_run(batch, steps: int, warmup: int, rotate=None):
    """`warmup` untimed steps, then exactly `steps` timed ones between two synchronisations.  HIP events
    around every stage hold the stream up by a few microseconds each (about 3 % of a varlen step when every
    step carries them), so only every eighth timed step is instrumented (every step in short runs).
    `rotate`: batches taken in turn instead of `batch` (every call then brings other offsets)."""
    import torch
    aug = batch.aug
    seq = rotate or [batch]
    for i in range(max(warmup, len(seq) if rotate else 0)):
        seq[i % len(seq)].step()
    torch.cuda.synchronize()
    aug.aug_profile_read()
    period = 8 if steps >= 40 else 1
    timed_steps = len(range(0, steps, period))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        if i % period == 0:
            aug.aug_profile_enable(True)
            seq[i % len(seq)].step()
            aug.aug_profile_enable(False)
        else:
            seq[i % len(seq)].step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = aug.aug_profile_read()
    stages = {k: (ms / max(n, 1), n) for k, (ms, n) in prof.items() if n > 0}     # (ms per launch, launches)
    return dt * 1e3 / steps, stages, timed_steps


def summarise(batch, ms_per_step, stages, timed_steps, images, workload_name):
    """Dominant stage, its roofline, and every stage's time and fraction."""
    w = batch.w
    defined, visited = images
    work = stage_work(w, visited)
    if batch.vtlp == "waveform-only":
        work = {k: v for k, v in work.items() if k == "vtlp"}
    per_step = {k: v[0] * v[1] / timed_steps for k, v in stages.items()}
    dominant = max((k for k in stages if k in work), key=lambda k: per_step[k])
    roof = roofline_for(dominant, work, per_step[dominant])
    roof["kernel"] = KERNEL_OF_STAGE[dominant]
    roof["avg_launch_ms"] = stages[dominant][0]
    roof["traffic"] = recorded_traffic(workload_name, dominant)     # HBM bytes per launch, or null
    if work[dominant][0] == "alu32":
        roof["peak_note"] = "fp32 vector peak with packed FP32; this build issues plain FMAs only, which reach 78.6"
    fracs = {k: round(roofline_for(k, work, per_step[k])["frac"], 4) for k in stages if k in work}
    return dominant, roof, {k: round(v, 4) for k, v in per_step.items()}, fracs, work


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="varlen",
                    choices=["tiny", "features", "batch", "varlen", "throughput"])
    ap.add_argument("--vtlp", default="mel", choices=["mel", "waveform", "waveform-only"],
                    help="mel: the warp is applied to the mel bank inside the front end (the headline path); "
                         "waveform: aug_vtlp_resynth_batch on the speech first, then the same path with "
                         "alpha = 1 (the paper's own order); waveform-only: aug_vtlp_resynth_batch alone")
    ap.add_argument("--mics", type=int, default=0,
                    help="time aug_rir_mics_batch alone: the workload's rooms with this many microphones in each "
                         "(responses/s instead of the headline metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a HIP graph (extra object in the JSON line; matters for "
                         "small batches, whose dozen launches cost as much as their kernels)")
    ap.add_argument("--no-h2d", action="store_true",
                    help="skip the extra, untimed-for-the-headline loop that copies the waveforms from host memory")
    ap.add_argument("--rotate-batches", type=int, default=3,
                    help="also time the step when K batches with different utterance lengths take turns, so that "
                         "every call uploads new offsets and rebuilds its tables (0: skip)")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the figures for the other four workloads")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one untimed 1 GiB device-to-device copy, the known-size kernel that "
                         "FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU (utterances are independent; there is nothing to "
              "exchange), so --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_1912_11040_amd import workloads as W
    from paper_1912_11040_amd.binding import Augmenter

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    w = W.WORKLOADS[args.workload]()
    aug = Augmenter(0)
    if args.mics > 0:
        if w.geom is None:
            print("bench.py: --mics needs a workload with rooms", file=sys.stderr)
            return 2
        print(json.dumps(bench_mics(args, w, aug)))
        aug.close()
        return 0

    batch = DeviceBatch(w, aug, args.vtlp)
    images = count_images(batch)

    if args.copy_probe:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ms_per_step, stages, timed_steps = timed_run(batch, args.steps, args.warmup)
    dominant, roof, stage_ms, stage_frac, work = summarise(batch, ms_per_step, stages, timed_steps, images, args.workload)

    rotating = None
    if args.rotate_batches > 0 and args.vtlp == "mel":
        # the largest batch first, so that the workspace is sized once
        others = [batch] + [batch.trimmed(k) for k in range(1, args.rotate_batches)]
        r_steps = max(len(others), min(args.steps, 60))
        r_ms, _, _ = timed_run(batch, r_steps, args.warmup, rotate=others)
        audio = sum(int(b.offsets[-1]) for b in others) / len(others) / w.fs
        rotating = {"batches": len(others), "steps": r_steps, "ms_per_step": r_ms, "value": audio / (r_ms * 1e-3),
                    "vs_steady_state": r_ms / ms_per_step * (w.audio_seconds / audio),
                    "note": "the workload and copies of it with every utterance 37 k samples shorter take turns: "
                            "every call has other offsets than the one before"}
        del others

    ms_with_h2d = None
    if not args.no_h2d:
        # The same step when the waveforms start in pinned host memory (never `value`: the boundary takes
        # device pointers): host-to-device copies of speech and noise, then the call.
        h_speech = torch.from_numpy(np.ascontiguousarray(w.speech)).pin_memory()
        h_noise = None if w.noise is None else torch.from_numpy(np.ascontiguousarray(w.noise)).pin_memory()
        reps = max(3, min(10, args.steps))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            batch.speech.copy_(h_speech, non_blocking=True)
            if h_noise is not None:
                batch.noise.copy_(h_noise, non_blocking=True)
            batch.step()
        torch.cuda.synchronize()
        ms_with_h2d = (time.perf_counter() - t0) * 1e3 / reps
        del h_speech, h_noise
    graph_ms = None
    if args.graph:
        # the library's context runs on torch's current stream; capture needs a stream of its own
        side = torch.cuda.Stream()
        aug_g = Augmenter(0, side)
        with torch.cuda.stream(side):
            batch.step(aug_g)                            # sizes this context's workspace, uploads its tables
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                batch.step(aug_g)
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        del g
        aug_g.close()

    full = batch.full
    foff = batch.foff
    out = {
        "metric": METRIC_BY_VTLP[args.vtlp],
        "value": w.audio_seconds / (ms_per_step * 1e-3),
        "unit": "audio-s/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": describe(w),
                   "entry_point": {"mel": "", "waveform": "aug_vtlp_resynth_batch + ",
                                   "waveform-only": "aug_vtlp_resynth_batch"}[args.vtlp] +
                                  ("" if args.vtlp == "waveform-only" else
                                   "aug_pipeline_batch" if full else "aug_vtlp_mel_batch"),
                   "vtlp": args.vtlp, "images_defined": images[0], "images_visited": images[1]},
        "roofline": roof,
        "rotating": rotating,
        "with_h2d": None if ms_with_h2d is None else
                    {"ms_per_step": ms_with_h2d, "value": w.audio_seconds / (ms_with_h2d * 1e-3),
                     "note": "waveforms copied from pinned host memory before every call; not the headline"},
        "graph": None if graph_ms is None else
                 {"ms_per_step": graph_ms, "value": w.audio_seconds / (graph_ms * 1e-3),
                  "note": "the same step replayed from a HIP graph"},
        "stage_ms": stage_ms,
        "stage_timed_steps": timed_steps,
        "stage_roofline_frac": stage_frac,
    }
    # The whole step against the chip: all stages' algorithmic flops over the step time against the fp32
    # vector peak (the image sum's fp64 flops count once each, on the images it walks), and the bytes that
    # must cross HBM at least once (inputs in, features out) against the HBM peak.
    # front end: 2.5 K log2 K for the real transform + window + bin powers + sparse mel + power law, per frame
    front_flop_per_frame = 2.5 * 512 * 9 + 400 + 771 + 1028 + 80
    flops = sum(amount for k, (bound, amount) in work.items() if bound != "hbm" and k in stages)
    if "mel" in stages:
        flops += front_flop_per_frame * float(foff[-1])
    n_src_in = 1 + (w.n_noise if full and args.vtlp != "waveform-only" else 0)
    min_bytes = 4.0 * w.total * n_src_in + (4.0 * w.total if args.vtlp == "waveform-only"
                                             else 4.0 * w.frontend.feature_dim * float(foff[-1]))
    out["path_roofline"] = {
        "flops_per_step": flops, "achieved_tflops": flops / (ms_per_step * 1e-3) / 1e12,
        "frac_of_fp32_peak": flops / (ms_per_step * 1e-3) / 1e12 / PEAK_FP32_TFLOPS,
        "min_hbm_bytes_per_step": min_bytes, "achieved_gbs": min_bytes / (ms_per_step * 1e-3) / 1e9,
        "frac_of_hbm_peak": min_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
    }

    if not args.no_per_config and args.vtlp == "mel":
        per = {args.workload: {"workload": describe(w), "steps": args.steps, "ms_per_step": ms_per_step,
                               "value": out["value"], "dominant_kernel": roof["kernel"], "bound": roof["bound"],
                               "frac": roof["frac"], "stage_ms": stage_ms}}
        del batch
        torch.cuda.empty_cache()
        for name in ("tiny", "features", "batch", "varlen", "throughput"):
            if name in per:
                continue
            wn = W.WORKLOADS[name]()
            bn = DeviceBatch(wn, aug)
            img = count_images(bn)
            n_steps = PER_CONFIG_STEPS[name]
            ms, st, ts = timed_run(bn, n_steps, 3)
            _, rf, sms, _, _ = summarise(bn, ms, st, ts, img, name)
            per[name] = {"workload": describe(wn), "steps": n_steps, "ms_per_step": ms,
                         "value": wn.audio_seconds / (ms * 1e-3), "dominant_kernel": rf["kernel"],
                         "bound": rf["bound"], "frac": rf["frac"], "stage_ms": sms}
            del bn, wn
            torch.cuda.empty_cache()
        out["per_config"] = {k: per[k] for k in ("tiny", "features", "batch", "varlen", "throughput")}
    aug.close()

    if not args.no_cpu_baseline:
        # the oracle's direct sums (the definition), then, as context, its own FFT forms, which is what a
        # sensible CPU program would run; both on all host cores
        out["cpu_baseline"] = cpu_baseline(w, vtlp=args.vtlp)
        out["cpu_baseline_fft"] = cpu_baseline(w, budget_s=8.0, vtlp=args.vtlp, fft=True)
    print(json.dumps(out))
    return 0


def bench_mics(args, w, aug) -> dict:
    """aug_rir_mics_batch alone: every room of the workload with a line array of --mics microphones."""
    import torch
    from paper_1912_11040_amd import workloads as W
    K, L = args.mics, w.rir_len
    geom_h = np.asarray(w.geom, np.float32).reshape(-1, 10)
    mics_h = W.microphone_arrays(geom_h, K, 0.068, seed=17)
    geom, mics = torch.from_numpy(geom_h).cuda(), torch.from_numpy(mics_h).cuda()
    n_rir = len(geom_h)
    out_h = torch.empty((n_rir, K, L), dtype=torch.float32, device="cuda")
    cnt = torch.empty((n_rir, K, L), dtype=torch.int32, device="cuda")
    aug.aug_rir_mics_batch(geom, mics, L, w.fs, w.c, out_h, cnt)          # untimed: counts the images
    n_images = float(cnt.sum(dtype=torch.int64).item())
    del cnt
    for _ in range(args.warmup):
        aug.aug_rir_mics_batch(geom, mics, L, w.fs, w.c, out_h)
    torch.cuda.synchronize()
    aug.aug_profile_read()
    aug.aug_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        aug.aug_rir_mics_batch(geom, mics, L, w.fs, w.c, out_h)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = aug.aug_profile_read()
    aug.aug_profile_enable(False)
    ms_per_step = dt * 1e3 / args.steps
    rir_ms = prof["rir"][0] / max(prof["rir"][1], 1)
    # one-microphone time of the same rooms, for the ratio
    one = torch.empty((n_rir, L), dtype=torch.float32, device="cuda")
    for _ in range(args.warmup):
        aug.aug_rir_batch(geom, L, w.fs, w.c, one)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        aug.aug_rir_batch(geom, L, w.fs, w.c, one)
    torch.cuda.synchronize()
    one_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    res = {
        "metric": f"image-method responses/sec, {K} microphones per room, on 1 GPU",
        "value": n_rir * K / (ms_per_step * 1e-3), "unit": "responses/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"rooms and sources of {describe(w)}; {K} microphones 6.8 cm apart in each; "
                               f"{n_rir} x {K} responses of {L} taps", "entry_point": "aug_rir_mics_batch",
                   "images_defined": n_images},
        "one_microphone_ms_per_step": one_ms, "ratio_to_one_microphone": ms_per_step / one_ms,
        "rir_kernel_ms": rir_ms,
        "stage_ms": {k: round(ms / args.steps, 4) for k, (ms, n) in prof.items() if n > 0},
    }
    if not args.no_cpu_baseline:
        from oracle import aug_oracle as O
        t0, done = time.perf_counter(), 0
        while done < n_rir and time.perf_counter() - t0 < 15.0:
            O.rir_mics_batch(geom_h[done:done + 1], mics_h[done:done + 1], L, w.fs, w.c)
            done += 1
        dt = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": done * K / dt, "unit": "responses/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {done} room(s) of the workload, {K} microphones each, {dt:.1f} s"}
    return res


if __name__ == "__main__":
    sys.exit(main())
