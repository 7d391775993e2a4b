#!/usr/bin/env python3
"""Throughput of the augmentation + feature path on one MI355X.

A step is one aug_pipeline_batch call (impulse responses, reverberation, SNR mix,
warped power-mel features) over one batch of seeded synthetic utterances that is
already resident in HBM.  Prints one JSON line with the whole-call throughput in
audio-seconds per second, the roofline of the dominant kernel (timed with HIP
events on the library's stream inside the timed region) and the CPU oracle timed
on a bounded sample of the same workload.
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
PEAK_FP32_TFLOPS = 157.3
PEAK_FP64_TFLOPS = 78.6
RIR_FLOP_PER_IMAGE = 12.0     # 2 add, sqrt, mul, add, floor, table product, divide, scale, accumulate ...

# HBM bytes per launch (read + written) of each stage's kernel, from the rocprofv3 FETCH_SIZE / WRITE_SIZE
# runs summarised in profiles/hbm_traffic_<workload>.md, scaled there by a 1 GiB copy.  They describe the
# kernel sources with this digest only; for any other sources `traffic` is reported as null.
RECORDED_TRAFFIC = {
    "digest": "0cfbf2ec4f706c26",
    "varlen": {"rir": 124206024, "rir_spectrum": 202541643, "convolve": 1330361433, "mel": 627087549},
    "throughput": {"rir": 672419566, "rir_spectrum": 1220132549, "convolve": 5675457889, "mel": 2221217745},
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
    """Algorithmic work of each stage for one step: (bound, amount, unit of amount)."""
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
    return {"bound": b, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
            "traffic": None}


def cpu_baseline(w, budget_s: float = 15.0, vtlp: str = "mel", fft: bool = False):
    """The oracle as it stands, one thread, on the first utterances of the workload: utterances are
    fed to it one at a time until the time budget is used up.  fft=True times the oracle's own
    FFT forms (fp64 numpy FFT convolution and STFT) instead of the direct sums."""
    from oracle import aug_oracle as O
    try:
        from threadpoolctl import threadpool_limits
    except Exception:                                  # pragma: no cover
        threadpool_limits = None

    def run():
        elapsed, audio, count = 0.0, 0.0, 0
        for u in range(w.n_utt):
            s = w.slice([u])
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
            elapsed += time.perf_counter() - t0
            audio += s.audio_seconds
            count += 1
            if elapsed >= budget_s:
                break
        return elapsed, audio, count

    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            dt, audio, count = run()
    else:
        dt, audio, count = run()
    return {"value": audio / dt, "unit": "audio-s/s", "cores": 1, "kind": "oracle",
            "sample": f"first {count} utterance(s) of the workload ({audio:.1f} audio-s), one at a time, "
                      + ("fp64 FFT convolution + FFT front end" if fft else
                         "direct time-domain convolution + DFT-matrix front end") + f", {dt:.1f} s"}


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
    flops = RIR_FLOP_PER_IMAGE * n_images
    res = {
        "metric": f"image-method responses/sec, {K} microphones per room, on 1 GPU",
        "value": n_rir * K / (ms_per_step * 1e-3), "unit": "responses/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"rooms and sources of {describe(w)}; {K} microphones 6.8 cm apart in each; "
                               f"{n_rir} x {K} responses of {L} taps", "entry_point": "aug_rir_mics_batch",
                   "images_per_step": n_images},
        "roofline": {"bound": "alu", "achieved": flops / (rir_ms * 1e-3) / 1e12, "peak": PEAK_FP64_TFLOPS,
                     "unit": "TFLOP/s", "frac": flops / (rir_ms * 1e-3) / 1e12 / PEAK_FP64_TFLOPS, "traffic": None,
                     "kernel": "rir_image_kernel", "avg_launch_ms": rir_ms},
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
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    speech, noise, geom = dev(w.speech), dev(w.noise), dev(w.geom)
    snr, alpha = dev(w.snr_db), dev(w.alpha)
    foff = w.frame_offsets()
    feats = torch.empty((int(foff[-1]), w.frontend.n_mel), dtype=torch.float32, device="cuda")
    full = w.geom is not None

    aug = Augmenter(0)
    if args.mics > 0:
        if not full:
            print("bench.py: --mics needs a workload with rooms", file=sys.stderr)
            return 2
        print(json.dumps(bench_mics(args, w, aug)))
        aug.close()
        return 0
    warped = torch.empty_like(speech) if args.vtlp != "mel" else None
    ones = torch.ones_like(alpha)

    def step():
        if args.vtlp == "waveform-only":
            aug.aug_vtlp_resynth_batch(w.offsets, speech, alpha, warped)
            return
        x, a = speech, alpha
        if args.vtlp == "waveform":
            aug.aug_vtlp_resynth_batch(w.offsets, speech, alpha, warped)
            x, a = warped, ones
        if full:
            aug.aug_pipeline_batch(w.offsets, x, noise, geom, w.rir_len, w.fs, w.c, snr, a,
                                   w.frontend, foff, feats)
        else:
            aug.aug_vtlp_mel_batch(w.offsets, x, a, w.frontend, foff, feats)

    # images per step, for the image-sum kernel's algorithmic work (counted once, untimed)
    n_images = 0.0
    if full and args.vtlp != "waveform-only":
        n_rir = w.n_utt * (1 + w.n_noise)
        chunk = max(1, min(n_rir, (1 << 28) // w.rir_len))
        g2 = geom.reshape(-1, 10)
        for a in range(0, n_rir, chunk):
            b = min(n_rir, a + chunk)
            h = torch.empty((b - a, w.rir_len), dtype=torch.float32, device="cuda")
            cnt = torch.empty((b - a, w.rir_len), dtype=torch.int32, device="cuda")
            aug.aug_rir_batch(g2[a:b].contiguous(), w.rir_len, w.fs, w.c, h, cnt)
            n_images += float(cnt.sum(dtype=torch.int64).item())
            del h, cnt

    if args.copy_probe:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    aug.aug_profile_read()
    # HIP events around every stage hold the stream up by a few microseconds each (about 3 % of a varlen
    # step when every step carries them), so inside the timed region only every eighth step is
    # instrumented; runs too short for that instrument every step.
    period = 8 if args.steps >= 40 else 1
    timed_steps = len(range(0, args.steps, period))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % period == 0:
            aug.aug_profile_enable(True)
            step()
            aug.aug_profile_enable(False)
        else:
            step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = aug.aug_profile_read()

    ms_per_step = dt * 1e3 / args.steps

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
            speech.copy_(h_speech, non_blocking=True)
            if h_noise is not None:
                noise.copy_(h_noise, non_blocking=True)
            step()
        torch.cuda.synchronize()
        ms_with_h2d = (time.perf_counter() - t0) * 1e3 / reps
        del h_speech, h_noise
    graph_ms = None
    if args.graph:
        # the library's context runs on torch's current stream; capture needs a stream of its own
        side = torch.cuda.Stream()
        aug_g = Augmenter(0, side)
        with torch.cuda.stream(side):
            saved, aug = aug, aug_g
            try:
                step()                                   # sizes this context's workspace, uploads its tables
                side.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    step()
            finally:
                aug = saved
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
    stages = {k: (ms / max(n, 1), n) for k, (ms, n) in prof.items() if n > 0}
    work = stage_work(w, n_images)
    if args.vtlp == "waveform-only":
        work = {k: v for k, v in work.items() if k == "vtlp"}
    dominant = max((k for k in stages if k in work), key=lambda k: stages[k][0] * stages[k][1])
    per_step_launches = stages[dominant][1] / timed_steps
    roof = roofline_for(dominant, work, stages[dominant][0] * per_step_launches)
    roof["kernel"] = {"rir": "rir_image_kernel", "convolve": "convolve_kernel", "mel": "mel_kernel",
                      "mix": "mix_kernel", "rir_spectrum": "rir_spectrum_kernel",
                      "vtlp": "vtlp_resynth_kernel"}[dominant]
    roof["avg_launch_ms"] = stages[dominant][0]
    roof["traffic"] = recorded_traffic(args.workload, dominant)     # HBM bytes per launch, or null

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
                   "vtlp": args.vtlp, "images_per_step": n_images},
        "roofline": roof,
        "with_h2d": None if ms_with_h2d is None else
                    {"ms_per_step": ms_with_h2d, "value": w.audio_seconds / (ms_with_h2d * 1e-3),
                     "note": "waveforms copied from pinned host memory before every call; not the headline"},
        "graph": None if graph_ms is None else
                 {"ms_per_step": graph_ms, "value": w.audio_seconds / (graph_ms * 1e-3),
                  "note": "the same step replayed from a HIP graph"},
        "stage_ms": {k: round(v[0] * v[1] / timed_steps, 4) for k, v in stages.items()},
        "stage_timed_steps": timed_steps,
        "stage_roofline_frac": {k: round(roofline_for(k, work, stages[k][0] * stages[k][1] / timed_steps)["frac"], 4)
                                for k in stages if k in work},
    }
    # The whole step against the chip: all stages' algorithmic flops over the step time against the fp32
    # vector peak (the image sum's fp64 flops count once each), and the bytes that must cross HBM at least
    # once (inputs in, features out) against the HBM peak.
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
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, vtlp=args.vtlp)
        # context only: the same oracle with its FFT forms, which is what a sensible CPU program would run
        out["cpu_baseline_fft"] = cpu_baseline(w, budget_s=8.0, vtlp=args.vtlp, fft=True)
    aug.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
