"""The oracle against the closed-form fixtures of tests/golden/closed_forms.txt."""
import os

import numpy as np

from oracle import aug_oracle as O

PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "closed_forms.txt")


def _rows(kind):
    with open(PATH) as fh:
        return [line.split()[1:] for line in fh if line.startswith(kind + " ")]


def test_eq1_special_points():
    rows = _rows("warp")
    assert len(rows) == 20
    for alpha, w, w_out in rows:
        assert abs(float(O.bilinear_warp(float(w), float(alpha))) - float(w_out)) < 1e-14


def test_direct_path_only():
    rows = _rows("direct")
    assert len(rows) == 4
    for r, fs, c, tap, amp in rows:
        r, fs, c, tap, amp = float(r), float(fs), float(c), int(tap), float(amp)
        # source and microphone r apart along x in a large room, no reflections
        geom = np.array([30.0, 20.0, 10.0, 5.0, 7.0, 3.0, 5.0 + r, 7.0, 3.0, 0.0], np.float32)
        h, cnt = O.rir_single(geom, 2048, fs, c)
        r32 = float(np.float32(5.0 + r)) - 5.0                   # the geometry is held in fp32
        assert np.count_nonzero(h) == 1
        assert int(np.argmax(h)) == int(np.floor(r32 * fs / c + 0.5)) and abs(int(np.argmax(h)) - tap) <= 1
        assert abs(h.max() - 1.0 / (4.0 * np.pi * r32)) < 1e-12 and abs(h.max() - amp) < 1e-6 * amp
        assert cnt[int(np.argmax(h))] >= 1


def test_mel_anchor_points():
    rows = _rows("mel")
    assert len(rows) == 3
    for f, m in rows:
        assert abs(float(O._hz_to_mel(float(f))) - float(m)) < 1e-9
        assert abs(float(O._mel_to_hz(float(m))) - float(f)) < 1e-9
    # the band edges are equally spaced in mel: on [0, 6300] Hz = [0, 2595] mel they sit at 2595 i / 41 mel
    edges = O.mel_edges_hz(40, 0.0, 6300.0)
    assert edges[0] == 0.0 and abs(edges[-1] - 6300.0) < 1e-9
    np.testing.assert_allclose(O._hz_to_mel(edges), 2595.0 * np.arange(42) / 41.0, atol=1e-9)
