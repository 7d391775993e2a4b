"""aug_pipeline_batch (the fused path) against the oracle, small and sampled-at-scale."""
import numpy as np
import pytest

from oracle import aug_oracle as O
from paper_1912_11040_amd import binding
from paper_1912_11040_amd import workloads as W
from tests.parity import FEAT_TOL, GAIN_TOL, RIR_TOL, WAVE_TOL, DeviceWorkload, feat_err, rir_err, wave_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def aug():
    from paper_1912_11040_amd.binding import Augmenter
    a = Augmenter(0)
    yield a
    a.close()


def _run(aug, w, want_rir=True, want_mixed=True):
    import torch
    d = DeviceWorkload(w)
    feats = d.empty_feats()
    n_src = 1 + w.n_noise
    rir = torch.full((w.n_utt, n_src, w.rir_len), float("nan"), dtype=torch.float32, device="cuda") \
        if want_rir else None
    mixed = torch.full((w.total,), float("nan"), dtype=torch.float32, device="cuda") if want_mixed else None
    gains = torch.full((w.n_utt, max(w.n_noise, 1)), float("nan"), dtype=torch.float32, device="cuda")
    aug.aug_pipeline_batch(w.offsets, d.speech, d.noise, d.geom, w.rir_len, w.fs, w.c, d.snr_db, d.alpha,
                           w.frontend, d.frame_offsets, feats, rir, mixed, gains if w.n_noise else None)
    torch.cuda.synchronize()
    return dict(feats=feats.cpu().numpy(), rir=None if rir is None else rir.cpu().numpy(),
                mixed=None if mixed is None else mixed.cpu().numpy(),
                gains=gains.cpu().numpy()[:, :w.n_noise])


def _oracle(w, conv="direct"):
    return O.pipeline_batch(w.offsets, w.speech, w.noise, w.geom, w.rir_len, w.fs, w.c, w.snr_db,
                            w.alpha, w.frontend, conv_method=conv)


def _compare(got, ref, w):
    w_err = wave_err(got["mixed"], ref["mixed"], w.offsets, silent_scale=w.speech)
    print(f"  rir err {rir_err(got['rir'], ref['rir']):.2e}  wave err {w_err:.2e}"
          f"  feat err {feat_err(got['feats'], ref['feats']):.2e}", flush=True)
    assert rir_err(got["rir"], ref["rir"]) <= RIR_TOL
    assert w_err <= WAVE_TOL
    np.testing.assert_allclose(got["gains"], ref["gains"], rtol=GAIN_TOL)
    assert got["feats"].shape == ref["feats"].shape
    assert feat_err(got["feats"], ref["feats"]) <= FEAT_TOL


def _compare_unmaterialised(aug, w, ref):
    # without mixed_out the front end mixes the reverberated signals while it loads its frames:
    # a different kernel instantiation, held to the same bar against the oracle
    got = _run(aug, w, want_rir=False, want_mixed=False)
    print(f"  mixture not materialised: feat err {feat_err(got['feats'], ref['feats']):.2e}", flush=True)
    assert got["feats"].shape == ref["feats"].shape
    assert feat_err(got["feats"], ref["feats"]) <= FEAT_TOL
    if w.n_noise:
        np.testing.assert_allclose(got["gains"], ref["gains"], rtol=GAIN_TOL)
    return got


def test_tiny_config_end_to_end(aug):
    w = W.tiny()
    print("case: tiny pipeline, direct convolution + DFT-matrix oracle", flush=True)
    got = _run(aug, w)
    ref = _oracle(w)
    _compare(got, ref, w)
    # internal buffers instead of caller outputs give the same features
    again = _compare_unmaterialised(aug, w, ref)
    assert feat_err(again["feats"], got["feats"].astype(np.float64)) <= 1e-5


def test_batch_config_subset(aug):
    w = W.batch(n_utt=4, seconds=4.0)
    print("case: batch config, 4 utterances, L=8000, direct oracle", flush=True)
    ref = _oracle(w)
    _compare(_run(aug, w), ref, w)
    _compare_unmaterialised(aug, w, ref)


def test_batch_config_full_size(aug):
    # all 64 utterances in one call; the direct-convolution oracle checks eight of them
    w = W.batch()
    print(f"case: batch config full, {w.n_utt} utterances, L={w.rir_len}", flush=True)
    got = _run(aug, w)
    lean = _run(aug, w, want_rir=False, want_mixed=False)
    foff = w.frame_offsets()
    # all 128 responses of the configuration: amplitudes from the pipeline, tap counts from aug_rir_batch
    import torch
    from tests.parity import dev, oracle_rirs
    h_ref, cnt_ref = oracle_rirs(w.geom, w.rir_len, w.fs, w.c)
    cnt = torch.full((len(h_ref), w.rir_len), -7, dtype=torch.int32, device="cuda")
    h = torch.empty((len(h_ref), w.rir_len), dtype=torch.float32, device="cuda")
    aug.aug_rir_batch(dev(w.geom.reshape(-1, 10)), w.rir_len, w.fs, w.c, h, cnt)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(cnt.cpu().numpy(), cnt_ref)
    assert rir_err(got["rir"].reshape(-1, w.rir_len), h_ref) <= RIR_TOL
    for u in range(0, w.n_utt, 8):
        s = w.slice([u])
        ref = _oracle(s)
        sub = dict(rir=got["rir"][u:u + 1], mixed=got["mixed"][w.offsets[u]:w.offsets[u + 1]],
                   gains=got["gains"][u:u + 1], feats=got["feats"][foff[u]:foff[u + 1]])
        _compare(sub, ref, s)
        assert feat_err(lean["feats"][foff[u]:foff[u + 1]], ref["feats"]) <= FEAT_TOL


def test_varlen_config_small(aug):
    w = W.varlen(n_utt=5, rir_len=2000, min_s=0.02, max_s=1.5)
    print("case: varlen small, 3 noises", flush=True)
    ref = _oracle(w)
    _compare(_run(aug, w), ref, w)
    _compare_unmaterialised(aug, w, ref)


def _full_size_sampled(aug, w, picks):
    """The whole workload in one call, as the benchmark launches it; the listed utterances against the oracle:
    their responses (amplitudes of the pipeline's image sums, and tap counts from aug_rir_batch on the same
    rows), gains, the whole mixture (fp64 FFT form, itself tied to direct sums at sampled positions) and all
    their frames, for both forms of the call."""
    import torch
    from tests.parity import dev, oracle_utterances
    got = _run(aug, w, want_rir=True, want_mixed=True)
    assert not np.isnan(got["feats"]).any() and not np.isnan(got["mixed"]).any()
    lean = _run(aug, w, want_rir=False, want_mixed=False)       # the call the benchmark times
    assert not np.isnan(lean["feats"]).any()
    np.testing.assert_array_equal(lean["gains"], got["gains"])
    foff = w.frame_offsets()
    lens = w.lengths()
    refs = oracle_utterances(w, picks, conv="fft")
    # tap counts of the picked utterances' responses, on the workload's own rooms
    rows = np.ascontiguousarray(w.geom[picks]).reshape(-1, 10)
    h = torch.full((len(rows), w.rir_len), float("nan"), dtype=torch.float32, device="cuda")
    cnt = torch.full((len(rows), w.rir_len), -7, dtype=torch.int32, device="cuda")
    aug.aug_rir_batch(dev(rows), w.rir_len, w.fs, w.c, h, cnt)
    torch.cuda.synchronize()
    cnt = cnt.cpu().numpy().reshape(len(picks), -1, w.rir_len)
    h = h.cpu().numpy().reshape(len(picks), -1, w.rir_len)
    rng = np.random.default_rng(0)
    for i, (u, ref) in enumerate(zip(picks, refs)):
        print(f"  utterance {u}: {lens[u]} samples", flush=True)
        s = w.slice([u])
        np.testing.assert_array_equal(cnt[i], ref["tap_count"][0])           # integer work: bit exact
        assert rir_err(h[i], ref["rir"][0]) <= RIR_TOL
        np.testing.assert_array_equal(h[i], got["rir"][u])                    # one image sum, whoever asks for it
        sub = dict(rir=got["rir"][u:u + 1], mixed=got["mixed"][w.offsets[u]:w.offsets[u + 1]],
                   gains=got["gains"][u:u + 1], feats=got["feats"][foff[u]:foff[u + 1]])
        _compare(sub, ref, s)
        assert feat_err(lean["feats"][foff[u]:foff[u + 1]], ref["feats"]) <= FEAT_TOL
        if i % 4 == 0:                                                         # the FFT form of the oracle itself
            pos = rng.integers(0, lens[u], 32)
            for j in range(1 + w.n_noise):
                x = s.speech if j == 0 else s.noise[j - 1]
                direct = O.convolve_at(x, ref["rir"][0, j], pos)
                np.testing.assert_allclose(O.convolve_fft(x, ref["rir"][0, j])[pos], direct, atol=1e-9)


def test_varlen_full_size_sampled(aug):
    # the benchmark's configuration and launch shape; 18 of its 256 utterances (first, last, shortest,
    # longest and a spread in between): 72 responses of 16000 taps
    from tests.parity import spread
    w = W.varlen()
    print(f"case: varlen full size, {w.n_utt} utterances, {w.total} samples, L={w.rir_len}", flush=True)
    lens = w.lengths()
    _full_size_sampled(aug, w, spread(w.n_utt, 16, extra=[np.argmin(lens), np.argmax(lens)]))


def test_throughput_full_size_sampled(aug):
    # the largest configuration (32768-tap responses in two partitions), as the benchmark launches it with
    # --workload throughput; 16 of its 1024 utterances: 48 responses of 32768 taps
    from tests.parity import spread
    w = W.throughput()
    print(f"case: throughput full size, {w.n_utt} utterances, {w.total} samples, L={w.rir_len}", flush=True)
    _full_size_sampled(aug, w, spread(w.n_utt, 16))


@pytest.mark.parametrize("want_mixed", [False, True])
def test_padded_batch_layout(aug, want_mixed):
    # the padded [n_utt][Tmax][n_mel] output through the fused call, with and without the mixture as an output
    import torch
    w = W.varlen(n_utt=4, rir_len=1500, min_s=0.01, max_s=1.2)
    d = DeviceWorkload(w)
    t = np.diff(w.frame_offsets())
    t_max = int(t.max()) + 2
    foff = (np.arange(w.n_utt + 1) * t_max).astype(np.int64)
    feats = torch.full((w.n_utt, t_max, w.frontend.n_mel), float("nan"), dtype=torch.float32, device="cuda")
    mixed = torch.empty((w.total,), dtype=torch.float32, device="cuda") if want_mixed else None
    aug.aug_pipeline_batch(w.offsets, d.speech, d.noise, d.geom, w.rir_len, w.fs, w.c, d.snr_db, d.alpha,
                           w.frontend, foff, feats, None, mixed, None)
    torch.cuda.synchronize()
    got = feats.cpu().numpy()
    ref = _oracle(w)["feats"]
    packed = w.frame_offsets()
    for u in range(w.n_utt):
        assert np.all(got[u, t[u]:] == 0.0)
        if t[u]:
            assert feat_err(got[u, :t[u]], ref[packed[u]:packed[u + 1]]) <= FEAT_TOL


def test_two_contexts_on_two_streams(aug):
    # double buffering: batches alternate between two contexts, each on a stream of its own with its own
    # workspace; every batch must come out as it does on a single stream
    import torch
    from paper_1912_11040_amd.binding import Augmenter
    ws = [W.varlen(n_utt=3, rir_len=1200, min_s=0.05, max_s=0.8, seed=s) for s in (7, 8, 9, 10)]
    want = [_run(aug, w, want_rir=False, want_mixed=False)["feats"] for w in ws]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ctxs = [Augmenter(0, s) for s in streams]
    keep = []
    for k, w in enumerate(ws):
        with torch.cuda.stream(streams[k % 2]):
            d = DeviceWorkload(w)
            feats = d.empty_feats()
            ctxs[k % 2].aug_pipeline_batch(w.offsets, d.speech, d.noise, d.geom, w.rir_len, w.fs, w.c, d.snr_db,
                                           d.alpha, w.frontend, d.frame_offsets, feats)
        keep.append((d, feats))
    torch.cuda.synchronize()
    for (d, feats), ref in zip(keep, want):
        assert feat_err(feats.cpu().numpy(), ref.astype(np.float64)) <= 1e-6
    for c in ctxs:
        c.close()


def test_many_short_utterances(aug):
    # a thousand utterances of 0 .. 0.25 s (some shorter than one analysis window, some empty):
    # the work-item tables, not the arithmetic, are what this stresses
    w = W.varlen(n_utt=1000, rir_len=300, min_s=0.0, max_s=0.25, seed=77)
    print(f"case: {w.n_utt} short utterances, {w.total} samples, L={w.rir_len}", flush=True)
    got = _run(aug, w)
    lean = _run(aug, w, want_rir=False, want_mixed=False)
    ref = _oracle(w)
    _compare(got, ref, w)
    assert feat_err(lean["feats"], ref["feats"]) <= FEAT_TOL
    assert int(np.sum(w.lengths() == 0)) >= 0 and int(np.sum(w.lengths() < 400)) > 50


def test_frames_before_any_sound_arrives(aug):
    # every source is more than 400 samples of travel away from the microphone, so the first analysis frame
    # of the mixture is exactly zero and its features must be zero, not the power law of rounding noise
    import dataclasses
    w = W.tiny(n_utt=2)
    geom = np.array(w.geom, np.float32)
    geom[:, :, 0:3] = [10.0, 8.0, 4.0]
    geom[:, 0, 3:6] = [0.6, 0.7, 0.5]
    geom[:, 1, 3:6] = [0.5, 7.4, 3.4]
    geom[:, :, 6:9] = [9.4, 4.0, 2.0]
    w = dataclasses.replace(w, geom=geom)
    ref = _oracle(w)
    foff = w.frame_offsets()
    assert np.all(ref["feats"][foff[0]] == 0.0) and np.all(ref["mixed"][:440] == 0.0)
    got = _run(aug, w)
    _compare(got, ref, w)
    _compare_unmaterialised(aug, w, ref)
    assert np.all(got["mixed"][:440] == 0.0) and np.all(got["feats"][foff[0]] == 0.0)


def test_steady_state_call_can_be_captured_in_a_graph():
    # Once the workspace has its size and the offsets are known, a call is kernel launches only (clears are
    # fill kernels, not memsets), so it can be recorded into a HIP graph.  Replays are interleaved with eager
    # work and synchronisations and each one is checked against the eager result.
    import torch
    from paper_1912_11040_amd.binding import Augmenter
    w = W.tiny(n_utt=4, rir_len=1500)
    stream = torch.cuda.Stream()
    ctx = Augmenter(0, stream)
    with torch.cuda.stream(stream):
        d = DeviceWorkload(w)
        eager = d.empty_feats()
        ctx.aug_pipeline_batch(w.offsets, d.speech, d.noise, d.geom, w.rir_len, w.fs, w.c, d.snr_db, d.alpha,
                               w.frontend, d.frame_offsets, eager)          # sizes the workspace, uploads the tables
        stream.synchronize()
        out = d.empty_feats()
        w2 = w.slice([0, 1])
        d2 = DeviceWorkload(w2)
        out2 = d2.empty_feats()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            # a batch with other offsets would need copies and new tables: refused while the stream is captured
            with pytest.raises(binding.AugError) as refused:
                ctx.aug_pipeline_batch(w2.offsets, d2.speech, d2.noise, d2.geom, w2.rir_len, w2.fs, w2.c, d2.snr_db,
                                       d2.alpha, w2.frontend, d2.frame_offsets, out2)
            assert refused.value.code == binding.AUG_ERR_UNSUPPORTED
            ctx.aug_pipeline_batch(w.offsets, d.speech, d.noise, d.geom, w.rir_len, w.fs, w.c, d.snr_db, d.alpha,
                                   w.frontend, d.frame_offsets, out)
    want = eager.cpu().numpy()
    for k in range(4):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out.cpu().numpy(), want)
        # eager work of the same context between replays
        with torch.cuda.stream(stream):
            again = d.empty_feats()
            ctx.aug_pipeline_batch(w.offsets, d.speech, d.noise, d.geom, w.rir_len, w.fs, w.c, d.snr_db, d.alpha,
                                   w.frontend, d.frame_offsets, again)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(again.cpu().numpy(), want)
    ref = _oracle(w)["feats"]
    assert feat_err(want, ref) <= FEAT_TOL
    del graph
    ctx.close()


def test_no_noise_pipeline(aug):
    import dataclasses
    w = W.tiny(n_utt=2)
    w = dataclasses.replace(w, noise=None, snr_db=None, geom=np.ascontiguousarray(w.geom[:, :1]))
    got = _run(aug, w)
    ref = _oracle(w)
    _compare(got, ref, w)
    _compare_unmaterialised(aug, w, ref)


def test_batch_with_no_frames_and_batch_with_no_samples(aug):
    # Every utterance shorter than one analysis window: the feature output has no rows, and an array with no
    # elements may be passed as a null pointer (torch's empty tensors are).  The waveform side still runs.
    import dataclasses
    import torch
    w = W.varlen(n_utt=3, rir_len=1024, min_s=0.0, max_s=0.02, seed=5)
    assert 0 < w.total and int(w.frame_offsets()[-1]) == 0
    got = _run(aug, w)
    ref = _oracle(w)
    assert got["feats"].shape == ref["feats"].shape == (0, w.frontend.n_mel)
    assert rir_err(got["rir"], ref["rir"]) <= RIR_TOL
    assert wave_err(got["mixed"], ref["mixed"], w.offsets, silent_scale=w.speech) <= WAVE_TOL
    np.testing.assert_allclose(got["gains"], ref["gains"], rtol=GAIN_TOL)
    _run(aug, w, want_rir=False, want_mixed=False)
    # no samples at all: responses are still produced, every gain is zero (zero energies)
    empty = dataclasses.replace(w, offsets=np.zeros(w.n_utt + 1, np.int64), speech=np.zeros(0, np.float32),
                                noise=np.zeros((w.n_noise, 0), np.float32))
    got = _run(aug, empty)
    assert got["feats"].shape[0] == 0 and got["mixed"].size == 0
    assert rir_err(got["rir"], ref["rir"]) <= RIR_TOL
    assert np.all(got["gains"] == 0.0)
    gains = torch.full((w.n_utt, w.n_noise), float("nan"), device="cuda")
    d = DeviceWorkload(empty)
    aug.aug_convolve_mix_batch(empty.offsets, d.speech, d.noise, torch.from_numpy(ref["rir"].astype(np.float32)).cuda(),
                               w.rir_len, d.snr_db, torch.zeros(0, device="cuda"), gains)
    torch.cuda.synchronize()
    assert np.all(gains.cpu().numpy() == 0.0)


def test_batches_with_new_lengths_every_call(aug):
    # The example queue hands over a batch with new lengths at every step (Sec. 2.2): batches that differ in
    # utterance count, lengths and response length alternate on one context with no synchronisation between
    # the calls (nine calls, so the four staging slots for the offsets are reused twice); every call's
    # features and gains against the oracle.
    import torch
    ws = [W.varlen(n_utt=3, rir_len=1200, min_s=0.05, max_s=0.9, seed=21),
          W.varlen(n_utt=6, rir_len=700, min_s=0.02, max_s=0.5, seed=22),
          W.varlen(n_utt=4, rir_len=1200, min_s=0.3, max_s=1.4, seed=23)]
    refs = [_oracle(w) for w in ws]
    devs = [DeviceWorkload(w) for w in ws]
    outs = []
    for k in range(9):
        w, d = ws[k % 3], devs[k % 3]
        feats = d.empty_feats()
        gains = torch.full((w.n_utt, w.n_noise), float("nan"), dtype=torch.float32, device="cuda")
        mixed = torch.full((w.total,), float("nan"), dtype=torch.float32, device="cuda") if k % 2 else None
        aug.aug_pipeline_batch(w.offsets, d.speech, d.noise, d.geom, w.rir_len, w.fs, w.c, d.snr_db, d.alpha,
                               w.frontend, d.frame_offsets, feats, None, mixed, gains)
        outs.append((feats, gains, mixed))
    torch.cuda.synchronize()
    for k, (feats, gains, mixed) in enumerate(outs):
        w, ref = ws[k % 3], refs[k % 3]
        fe = feat_err(feats.cpu().numpy(), ref["feats"])
        print(f"  call {k}: batch {k % 3}, feat err {fe:.2e}", flush=True)
        assert fe <= FEAT_TOL
        np.testing.assert_allclose(gains.cpu().numpy(), ref["gains"], rtol=GAIN_TOL)
        if mixed is not None:
            assert wave_err(mixed.cpu().numpy(), ref["mixed"], w.offsets, silent_scale=w.speech) <= WAVE_TOL
