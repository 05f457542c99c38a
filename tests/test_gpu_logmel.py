"""GPU-vs-oracle parity of the log-mel feature kernel (w2l_logmel_fwd), through the C ABI, on the
same seeded waveforms.

Tolerance (fp32 FFT and filterbank against the fp64 oracle): a 512-point fp32 FFT carries an
error of about 2^-24 * log2(512) * |largest bin|; a band whose energy lies D dB below the
strongest band of its frame therefore has a relative amplitude error of about 6e-7 * 10^(D/20),
i.e. |error of the log energy| <= 1.2e-6 * 10^(D/20) + 1e-5.  The test allows four times that,
per element, and additionally requires relative L2 <= 2e-5 over everything.  bf16 output: the
fp32 result rounded to nearest even, compared after rounding the oracle the same way (one bf16 ulp)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import empty, rel_l2, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_1812_07625_amd as P
    return P


def run_logmel(P, wav, wav_len, Tmax, n_mels, dtype="f32", **kw):
    B = wav.shape[0]
    wd, ld = to_dev(wav.astype(np.float32)), to_dev(np.asarray(wav_len, np.int32))
    feat = empty((B, Tmax, n_mels), dtype)
    flen = torch.full((B,), -7, dtype=torch.int32, device="cuda:0")
    feat.fill_(float("nan"))
    P.w2l_logmel_fwd(wd, ld, feat, flen, **kw)
    torch.cuda.synchronize()
    return to_host(feat), flen.cpu().numpy()


def check(feat, flen, wav, wav_len, n_mels, **kw):
    ref, rlen = oracle.logmel(wav.astype(np.float64), wav_len, n_mels=n_mels, Tmax=feat.shape[1], **kw)
    assert np.array_equal(flen, rlen)
    assert np.all(np.isfinite(feat))
    for b in range(len(rlen)):
        assert np.all(feat[b, rlen[b]:] == 0)
        if rlen[b] == 0:
            continue
        r, g = ref[b, :rlen[b]], feat[b, :rlen[b]]
        depth_db = (r.max(axis=1, keepdims=True) - r) * (10.0 / np.log(10.0))       # dB below the frame's strongest band
        allowed = 4 * (1.2e-6 * 10 ** (depth_db / 20.0) + 1e-5)
        assert np.all(np.abs(g - r) <= allowed), (b, float(np.max(np.abs(g - r) / allowed)))
    assert rel_l2(feat, ref) <= 2e-5


@pytest.mark.parametrize("kw", [
    dict(B=3, n_lo=2000, n_hi=9000, n_mels=40),
    dict(B=2, n_lo=30000, n_hi=40000, n_mels=80),
    dict(B=4, n_lo=300, n_hi=1200, n_mels=23),                       # utterances shorter than a window
    dict(B=2, n_lo=5000, n_hi=6000, n_mels=40, win=200, hop=80, nfft=256, sample_rate=8000),
    dict(B=2, n_lo=9000, n_hi=9900, n_mels=64, win=1000, hop=250, nfft=1024, fmin=60.0, fmax=7600.0),
    dict(B=1, n_lo=4000, n_hi=4000, n_mels=130, win=401, hop=77, nfft=512),   # odd window, more bands than lanes
])
def test_logmel_matches_oracle(P, kw):
    kw = dict(kw)
    n_mels = kw.pop("n_mels")
    sr = kw.get("sample_rate", 16000)
    cfg = W.waveforms(seed=13, B=kw.pop("B"), n_lo=kw.pop("n_lo"), n_hi=kw.pop("n_hi"), sample_rate=sr)
    win, hop = kw.get("win", 400), kw.get("hop", 160)
    Tmax = max(1, max(oracle.logmel_num_frames(int(n), win, hop) for n in cfg["wav_len"])) + 3   # a few all-padding frames
    feat, flen = run_logmel(P, cfg["wav"], cfg["wav_len"], Tmax, n_mels, **kw)
    check(feat, flen, cfg["wav"], cfg["wav_len"], n_mels, **kw)


def test_logmel_benchmark_shape_and_bf16(P):
    """The shape bench.py times (B=8, up to 240240 samples -> 1500 frames of 80 bands): every
    element against the oracle; then the bf16 output the train step would read."""
    cfg = W.waveforms()
    feat, flen = run_logmel(P, cfg["wav"], cfg["wav_len"], 1500, 80)
    check(feat, flen, cfg["wav"], cfg["wav_len"], 80)
    fb, flb = run_logmel(P, cfg["wav"], cfg["wav_len"], 1500, 80, dtype="bf16")
    assert np.array_equal(flb, flen)
    # the kernel rounds its own fp32 value: at most one bf16 step from the rounded fp32 run
    assert np.all(np.abs(fb - W.round_to_bf16(feat)) <= np.abs(feat) * 2.0 ** -7)
    assert np.mean(fb == W.round_to_bf16(feat)) > 0.999


def test_logmel_truncates_to_tmax_and_handles_silence(P):
    cfg = W.waveforms(seed=4, B=2, n_lo=8000, n_hi=9000)
    feat, flen = run_logmel(P, cfg["wav"], cfg["wav_len"], 10, 40)
    assert list(flen) == [10, 10]
    check(feat, flen, cfg["wav"], cfg["wav_len"], 40)
    wav = np.zeros((1, 2000), np.float32)
    feat, flen = run_logmel(P, wav, [2000], 12, 40)
    assert flen[0] == 11 and np.allclose(feat[0, :11], np.log(1e-10), atol=1e-5) and np.all(feat[0, 11:] == 0)
    assert P.w2l_logmel_num_frames(16000) == 98 and P.w2l_logmel_num_frames(399) == 0


def test_logmel_is_deterministic(P):
    cfg = W.waveforms(seed=6, B=2, n_lo=20000, n_hi=30000)
    a = run_logmel(P, cfg["wav"], cfg["wav_len"], 200, 80)
    b = run_logmel(P, cfg["wav"], cfg["wav_len"], 200, 80)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_features_feed_the_train_step(P):
    """Waveforms -> log-mel -> network forward, CTC, backward -> SGD with momentum, all through the
    C ABI with no host round trip in between (feat / feat_len are handed to w2l_train_step as x /
    in_len as they are), against the same chain of oracle functions.  fp32 model; the tolerance is
    1e-3 because the feature error (above) goes through the whole network."""
    from test_gpu_parity import rel_l2 as _rel
    cfg = W.waveforms(seed=21, B=3, n_lo=20000, n_hi=32000)
    layers = [dict(k=5, stride=2, cin=40, cout=64, glu=1), dict(k=3, stride=1, cin=32, cout=48, glu=1),
              dict(k=1, stride=1, cin=24, cout=W.NUM_CLASSES, glu=0)]
    model = W.small_model(22, 3, 10, 10, 40, layers, False, 4, 12)     # only its weights, biases and targets are used
    Tmax = max(oracle.logmel_num_frames(int(n), 400, 160) for n in cfg["wav_len"])
    # ---- GPU chain
    wd, ld = to_dev(cfg["wav"]), to_dev(cfg["wav_len"])
    feat = empty((3, Tmax, 40))
    flen = torch.zeros(3, dtype=torch.int32, device="cuda:0")
    P.w2l_logmel_fwd(wd, ld, feat, flen)
    wts = [to_dev(w) for w in model["weights"]]
    bss = [to_dev(b) for b in model["biases"]]
    dws = [empty(w.shape) for w in model["weights"]]
    dbs = [empty(b.shape) for b in model["biases"]]
    tg, tl = to_dev(model["targets"]), to_dev(model["tgt_len"])
    Lmax = model["targets"].shape[1]
    ws = P.workspace(P.w2l_train_step_workspace_bytes(layers, 3, Tmax, Lmax, P.W2L_F32))
    loss = empty((3,))
    P.w2l_train_step(layers, wts, bss, dws, dbs, feat, flen, tg, tl, loss, None, 0, 1.0, ws)
    vel = [torch.zeros_like(w) for w in wts]
    for w, v, g in zip(wts, vel, dws):
        P.w2l_sgd_momentum_step(w, v, g, None, 0.01, 0.9)
    torch.cuda.synchronize()
    # ---- oracle chain
    f_o, l_o = oracle.logmel(cfg["wav"].astype(np.float64), cfg["wav_len"], n_mels=40)
    assert np.array_equal(flen.cpu().numpy(), l_o)
    ref = oracle.train_step(layers, [w.astype(np.float64) for w in model["weights"]],
                            [b.astype(np.float64) for b in model["biases"]], f_o, l_o, model["targets"],
                            model["tgt_len"])
    assert np.all(np.abs(to_host(loss) - ref["loss"]) <= 1e-3 * np.abs(ref["loss"]))
    for i, (g, r) in enumerate(zip(dws, ref["dw"])):
        assert _rel(to_host(g), r) <= 1e-3, i
    for w, w0, r in zip(wts, model["weights"], ref["dw"]):
        w_o, _ = oracle.sgd_momentum(w0.astype(np.float64), np.zeros_like(r), r, 0.01, 0.9)
        assert _rel(to_host(w), w_o) <= 1e-5
