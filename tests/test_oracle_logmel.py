"""Pins of the fp64 log-mel oracle (feature type named in Sec. 2.2, used with 40 bins in
Sec. 4.1; the paper fixes no constant, so the recipe is a stated reading).  Checked against what
the mathematics fixes, by means other than the oracle's own routine: a brute-force DFT, closed
forms for tones and impulses, Parseval's identity, the partition-of-unity property of adjacent
triangles, known points of the mel scale, and shift behaviour."""
import math

import numpy as np

import oracle


def test_frame_count():
    assert oracle.logmel_num_frames(399, 400, 160) == 0
    assert oracle.logmel_num_frames(400, 400, 160) == 1
    assert oracle.logmel_num_frames(559, 400, 160) == 1
    assert oracle.logmel_num_frames(560, 400, 160) == 2
    assert oracle.logmel_num_frames(16000, 400, 160) == 98
    assert oracle.logmel_num_frames(0, 400, 160) == 0


def test_mel_scale_known_points_and_inverse():
    assert abs(oracle.mel_of_hz(0.0)) < 1e-12
    assert abs(oracle.mel_of_hz(700.0) - 2595.0 * math.log10(2.0)) < 1e-9
    assert abs(oracle.mel_of_hz(1000.0) - 1000.0) < 0.05          # the scale is anchored at 1 kHz = 1000 mel
    f = np.linspace(0, 8000, 50)
    assert np.allclose(oracle.hz_of_mel(oracle.mel_of_hz(f)), f, atol=1e-9)
    assert np.all(np.diff(oracle.mel_of_hz(f)) > 0)


def test_filterbank_shape_properties():
    F, nfft, sr = 40, 512, 16000
    fb = oracle.mel_filterbank(F, nfft, sr, 0.0, 8000.0)
    assert fb.shape == (F, nfft // 2 + 1)
    assert np.all(fb >= 0) and np.all(fb <= 1 + 1e-12)
    pts = oracle.hz_of_mel(np.linspace(oracle.mel_of_hz(0.0), oracle.mel_of_hz(8000.0), F + 2))
    freqs = np.arange(nfft // 2 + 1) * sr / nfft
    # adjacent triangles partition unity between the first and the last centre
    inside = (freqs >= pts[1]) & (freqs <= pts[F])
    assert np.allclose(fb[:, inside].sum(0), 1.0, atol=1e-12)
    # support of filter f is (pts[f], pts[f+2]); widths grow with frequency
    for f in (0, 7, 20, 39):
        nz = freqs[fb[f] > 0]
        assert nz.min() > pts[f] and nz.max() < pts[f + 2]
    assert np.all(np.diff(pts, 2) > 0)
    # a filter evaluated half way up its rising edge is 1/2
    fb2 = oracle.mel_filterbank(4, 4096, sr, 0.0, 8000.0)
    p2 = oracle.hz_of_mel(np.linspace(0, oracle.mel_of_hz(8000.0), 6))
    fr2 = np.arange(2049) * sr / 4096
    k = np.argmin(np.abs(fr2 - 0.5 * (p2[1] + p2[2])))
    assert abs(fb2[1, k] - (fr2[k] - p2[1]) / (p2[2] - p2[1])) < 1e-12


def brute_logmel_frame(seg, nfft, fb, floor):
    """One frame by the DFT definition, term by term."""
    win = len(seg)
    w = np.array([0.54 - 0.46 * math.cos(2 * math.pi * n / (win - 1)) for n in range(win)])
    x = seg * w
    power = np.zeros(nfft // 2 + 1)
    n = np.arange(win)
    for k in range(nfft // 2 + 1):
        re = np.sum(x * np.cos(2 * math.pi * k * n / nfft))
        im = -np.sum(x * np.sin(2 * math.pi * k * n / nfft))
        power[k] = re * re + im * im
    return np.log(np.maximum(fb @ power, floor))


def test_logmel_matches_brute_force_dft():
    rng = np.random.default_rng(3)
    wav = rng.standard_normal((2, 1000))
    lens = np.array([1000, 730])
    feat, flen = oracle.logmel(wav, lens, n_mels=23, sample_rate=16000, win=400, hop=160, nfft=512)
    assert list(flen) == [4, 3] and feat.shape == (2, 4, 23)
    fb = oracle.mel_filterbank(23, 512, 16000, 0.0, 8000.0)
    for b, t in [(0, 0), (0, 3), (1, 2)]:
        want = brute_logmel_frame(wav[b, t * 160:t * 160 + 400], 512, fb, 1e-10)
        assert np.allclose(feat[b, t], want, atol=1e-10)
    assert np.all(feat[1, 3] == 0)                       # beyond the utterance's frames


def test_logmel_closed_forms():
    sr, win, hop, nfft, F = 16000, 400, 160, 512, 40
    fb = oracle.mel_filterbank(F, nfft, sr, 0.0, 8000.0)
    w = 0.54 - 0.46 * np.cos(2 * np.pi * np.arange(win) / (win - 1))
    # an impulse inside the frame: flat power spectrum w[n0]^2, so every mel energy is w[n0]^2 * sum of the filter
    x = np.zeros((1, win))
    x[0, 123] = 2.5
    feat, _ = oracle.logmel(x, [win], n_mels=F, win=win, hop=hop, nfft=nfft)
    assert np.allclose(feat[0, 0], np.log((2.5 * w[123]) ** 2 * fb.sum(1)), atol=1e-10)
    # silence: the floor
    feat, _ = oracle.logmel(np.zeros((1, 900)), [900], n_mels=F)
    assert np.allclose(feat[0, :4], math.log(1e-10))
    # Parseval with a filterbank of all-ones would need the full spectrum; check it on the power spectrum itself
    rng = np.random.default_rng(5)
    seg = rng.standard_normal(win)
    spec = np.fft.fft(seg * w, n=nfft)
    assert abs(np.sum(np.abs(spec) ** 2) / nfft - np.sum((seg * w) ** 2)) < 1e-9
    # a tone exactly on DFT bin k0 with a rectangular stretch of the Hamming window: the bin's power is (A/2 * sum(w))^2
    # up to the leakage of the negative-frequency image, which is far below it for k0 in mid band
    k0, A = 100, 0.7
    tone = A * np.cos(2 * np.pi * k0 * np.arange(win) / nfft)
    power = np.abs(np.fft.rfft(tone * w, n=nfft)) ** 2
    assert abs(power[k0] / (A / 2 * w.sum()) ** 2 - 1) < 1e-3
    feat, _ = oracle.logmel(tone[None], [win], n_mels=F)
    assert np.argmax(feat[0, 0]) == np.argmax(fb[:, k0])  # the brightest band is the one whose filter peaks at that bin
    # gain: scaling the signal by g adds 2 log g to every band
    feat2, _ = oracle.logmel(3.0 * tone[None], [win], n_mels=F)
    assert np.allclose(feat2 - feat, 2 * math.log(3.0), atol=1e-9)


def test_logmel_shift_by_one_hop_shifts_frames():
    rng = np.random.default_rng(8)
    x = rng.standard_normal(4000)
    a, la = oracle.logmel(x[None], [4000], n_mels=40)
    b, lb = oracle.logmel(x[None, 160:], [3840], n_mels=40)
    assert la[0] == lb[0] + 1
    assert np.allclose(a[0, 1:la[0]], b[0, :lb[0]], atol=1e-12)
    # Tmax smaller than the frame count truncates; larger pads with zeros
    c, lc = oracle.logmel(x[None], [4000], n_mels=40, Tmax=5)
    assert lc[0] == 5 and np.allclose(c[0], a[0, :5])
    d, ld = oracle.logmel(x[None], [4000], n_mels=40, Tmax=40)
    assert ld[0] == la[0] and np.all(d[0, la[0]:] == 0)
