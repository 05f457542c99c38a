"""Seeded synthetic inputs for the five benchmark/parity configurations.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic (no convolution, GLU, softmax, CTC, ASG or feature computation) and is the one piece
shared by the oracle-side and the GPU-side callers.  Everything is numpy on the
host.  Shapes follow the paper's workload (Sec. 4.1: log-mel feature frames at
10 ms, grapheme targets, length-sorted -- hence narrow -- utterance lengths, an
all-convolutional network of ~100M parameters); no corpus item is used.

Draw order for every config, from ``numpy.random.default_rng(seed)``:
input lengths -> features -> per layer (weights, then bias) -> target lengths ->
targets.  For bf16 configs the features and weights are rounded to the nearest
bf16 value (ties to even) *here*, so both sides start from identical numbers.
"""
from __future__ import annotations

import numpy as np

BLANK = 0
NUM_CLASSES = 29


# ----------------------------------------------------------------------------- bf16 plumbing
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Nearest-even rounding of float32 values onto the bf16 grid (returned as float32)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    r = ((u + bias) >> 16) << 16
    out = r.astype(np.uint32).view(np.float32).reshape(a.shape)
    return np.where(np.isfinite(a), out, a)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values already on the bf16 grid."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16).reshape(a.shape)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """float32 values of uint16 bf16 bit patterns."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------- layer tables
def _L(k, stride, cin, cout, glu):
    return dict(k=k, stride=stride, cin=cin, cout=cout, glu=int(glu))


def layers_tiny():
    return [_L(5, 1, 40, 128, 1), _L(5, 1, 64, 128, 1), _L(1, 1, 64, NUM_CLASSES, 0)]


def layers_10m():
    return ([_L(13, 2, 40, 512, 1)] + [_L(11, 1, 256, 512, 1) for _ in range(6)]
            + [_L(1, 1, 256, 1024, 1), _L(1, 1, 512, NUM_CLASSES, 0)])


def layers_105m():
    return ([_L(13, 2, 80, 1536, 1)] + [_L(11, 1, 768, 1536, 1) for _ in range(8)]
            + [_L(1, 1, 768, 2048, 1), _L(1, 1, 1024, NUM_CLASSES, 0)])


def num_params(layers) -> int:
    return sum(L["k"] * L["cin"] * L["cout"] + L["cout"] for L in layers)


def total_stride(layers) -> int:
    s = 1
    for L in layers:
        s *= L["stride"]
    return s


def step_flops(layers, B, T) -> float:
    """2*M*K*N per GEMM-shaped pass: forward, wgrad for every layer, dgrad for all but the first."""
    f, t = 0.0, T
    for i, L in enumerate(layers):
        tp = (t + L["stride"] - 1) // L["stride"]
        g = 2.0 * B * tp * L["k"] * L["cin"] * L["cout"]
        f += g * (3 if i > 0 else 2)
        t = tp
    return f


# ----------------------------------------------------------------------------- generators
def _weights(rng, layers, bf16, zero_bias=True):
    ws, bs = [], []
    for L in layers:
        bound = 1.0 / np.sqrt(L["k"] * L["cin"])
        w = rng.uniform(-bound, bound, size=(L["cout"], L["k"], L["cin"])).astype(np.float32)
        if zero_bias:
            b = np.zeros(L["cout"], dtype=np.float32)
        else:
            b = rng.uniform(-bound, bound, size=L["cout"]).astype(np.float32)
        if bf16:
            w = round_to_bf16(w)
        ws.append(w)
        bs.append(b)
    return ws, bs


def _model_batch(seed, layers, B, Tmin, Tmax, feat, bf16, tgt_len_fn, zero_bias=True):
    rng = np.random.default_rng(seed)
    in_len = rng.integers(Tmin, Tmax + 1, size=B).astype(np.int32)
    T = int(Tmax)
    x = rng.standard_normal(size=(B, T, feat)).astype(np.float32)
    for b in range(B):
        x[b, in_len[b]:, :] = 0.0
    if bf16:
        x = round_to_bf16(x)
    ws, bs = _weights(rng, layers, bf16, zero_bias)
    tgt_len = np.asarray(tgt_len_fn(rng, in_len), dtype=np.int32)
    Lmax = int(max(1, tgt_len.max()))
    targets = np.zeros((B, Lmax), dtype=np.int32)
    for b in range(B):
        targets[b, :tgt_len[b]] = rng.integers(1, NUM_CLASSES, size=tgt_len[b])
    return dict(layers=layers, x=x, in_len=in_len, weights=ws, biases=bs, targets=targets,
                tgt_len=tgt_len, B=B, T=T, dtype="bf16" if bf16 else "f32", blank=BLANK,
                C=NUM_CLASSES)


def config0(seed=0, zero_bias=True):
    """Tiny fp32 model: B=2, T=100, 40-dim features, target lengths 10 and 7."""
    return _model_batch(seed, layers_tiny(), 2, 100, 100, 40, False,
                        lambda rng, n: [10, 7], zero_bias)


def config1(seed=1, B=16, T=800, Cin=512, Cout=1024, k=11, stride=1):
    """Single conv layer, bf16 operands: x ~ N(0,1), w ~ N(0, var 1/(Cin k)), dy ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    x = round_to_bf16(rng.standard_normal(size=(B, T, Cin)).astype(np.float32))
    w = round_to_bf16((rng.standard_normal(size=(Cout, k, Cin)) / np.sqrt(Cin * k)).astype(np.float32))
    Tp = (T + stride - 1) // stride
    dy = round_to_bf16(rng.standard_normal(size=(B, Tp, Cout)).astype(np.float32))
    return dict(x=x, w=w, dy=dy, B=B, T=T, Cin=Cin, Cout=Cout, k=k, stride=stride, dtype="bf16")


def config2(seed=2, B=32, T=750, Cc=NUM_CLASSES, in_lo=600, in_hi=750, l_lo=50, l_hi=200):
    """CTC alone, fp32: logits ~ N(0, var 2); input lengths U[in_lo,in_hi]; target lengths
    U[l_lo,l_hi], labels U[1,C-1]; a target is redrawn until in_len >= L + adjacent repeats."""
    rng = np.random.default_rng(seed)
    in_len = rng.integers(in_lo, in_hi + 1, size=B).astype(np.int32)
    logits = (rng.standard_normal(size=(B, T, Cc)) * np.sqrt(2.0)).astype(np.float32)
    tgt_len = rng.integers(l_lo, l_hi + 1, size=B).astype(np.int32)
    Lmax = int(max(1, tgt_len.max()))
    targets = np.zeros((B, Lmax), dtype=np.int32)
    for b in range(B):
        while True:
            lab = rng.integers(1, Cc, size=tgt_len[b])
            rep = int(np.sum(lab[1:] == lab[:-1]))
            if in_len[b] >= tgt_len[b] + rep:
                break
        targets[b, :tgt_len[b]] = lab
    return dict(logits=logits, in_len=in_len, targets=targets, tgt_len=tgt_len, B=B, T=T, C=Cc,
                blank=BLANK)


def asg_batch(seed=12, B=32, T=750, Cc=NUM_CLASSES - 1, in_lo=600, in_hi=750, l_lo=50, l_hi=200, em_std=np.sqrt(2.0),
              trans_std=0.5, allow_repeats=False):
    """ASG criterion alone, fp32, in the shape of config 2 without the blank class: emissions ~
    N(0, em_std^2); transitions ~ N(0, trans_std^2); input lengths U[in_lo,in_hi]; target lengths
    U[l_lo,l_hi] clipped to the input length; labels U[0,C-1], redrawn where equal to the label
    before them unless ``allow_repeats`` (the criterion's own preprocessing replaces letter repeats
    by repetition symbols, so neighbours differ).  Draw order: input lengths, emissions,
    transitions, target lengths, targets."""
    rng = np.random.default_rng(seed)
    in_len = rng.integers(in_lo, in_hi + 1, size=B).astype(np.int32)
    em = (rng.standard_normal(size=(B, T, Cc)) * em_std).astype(np.float32)
    trans = (rng.standard_normal(size=(Cc, Cc)) * trans_std).astype(np.float32)
    tgt_len = np.minimum(rng.integers(l_lo, l_hi + 1, size=B), np.maximum(in_len, 1)).astype(np.int32)
    Lmax = int(max(1, tgt_len.max()))
    targets = np.zeros((B, Lmax), dtype=np.int32)
    for b in range(B):
        lab = rng.integers(0, Cc, size=tgt_len[b])
        if not allow_repeats and Cc > 1:
            for i in range(1, len(lab)):
                while lab[i] == lab[i - 1]:
                    lab[i] = rng.integers(0, Cc)
        targets[b, :tgt_len[b]] = lab
    return dict(emissions=em, trans=trans, in_len=in_len, targets=targets, tgt_len=tgt_len, B=B, T=T, C=Cc)


def waveforms(seed=13, B=8, n_lo=160000, n_hi=240240, sample_rate=16000):
    """Speech-shaped synthetic audio for the feature kernel (no recording is used): per utterance a
    harmonic source -- fundamental wandering between 90 and 250 Hz, 12 harmonics with a 1/h roll-off
    and random phases -- under a slow amplitude envelope with pauses, plus white noise 30 dB below
    the peak; fp32 samples in about [-1, 1], zeros beyond each utterance's length U[n_lo, n_hi]
    (n_hi = 240240 samples = 1500 frames of 25 ms every 10 ms).  Draw order: lengths, then per
    utterance: pitch track, phases, envelope, noise."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(n_lo, n_hi + 1, size=B).astype(np.int32)
    Nmax = int(lens.max())
    wav = np.zeros((B, Nmax), dtype=np.float32)
    t = np.arange(Nmax) / sample_rate
    for b in range(B):
        knots = rng.uniform(90.0, 250.0, size=Nmax // 8000 + 2)
        f0 = np.interp(np.arange(Nmax) / 8000.0, np.arange(len(knots)), knots)
        phase = 2 * np.pi * np.cumsum(f0) / sample_rate
        ph0 = rng.uniform(0, 2 * np.pi, size=12)
        sig = sum(np.sin(h * phase + ph0[h - 1]) / h for h in range(1, 13))
        env_knots = np.clip(rng.uniform(-0.3, 1.0, size=Nmax // 4000 + 2), 0.0, 1.0)
        env = np.interp(np.arange(Nmax) / 4000.0, np.arange(len(env_knots)), env_knots)
        x = 0.5 * env * sig / np.max(np.abs(sig)) + 0.5 * 10 ** (-30 / 20) * rng.standard_normal(Nmax)
        x[lens[b]:] = 0.0
        wav[b] = x.astype(np.float32)
    del t
    return dict(wav=wav, wav_len=lens, B=B, sample_rate=sample_rate)


def config3(seed=3, B=16):
    """~10M-parameter bf16 model: T_b ~ U[800,1600] padded to 1600, L_b = floor(T_b/16)."""
    return _model_batch(seed, layers_10m(), B, 800, 1600, 40, True,
                        lambda rng, n: [int(v) // 16 for v in n])


def config4(seed=4, B=8):
    """~105M-parameter bf16 model: T_b ~ U[1000,1500] padded to 1500, L_b ~ U[60,150]."""
    return _model_batch(seed, layers_105m(), B, 1000, 1500, 80, True,
                        lambda rng, n: rng.integers(60, 151, size=len(n)))


def small_model(seed, B, Tmin, Tmax, feat, layers, bf16, l_lo, l_hi, zero_bias=False):
    """A free-form model batch for parity cases (ragged lengths, odd shapes, non-zero bias)."""
    return _model_batch(seed, layers, B, Tmin, Tmax, feat, bf16,
                        lambda rng, n: rng.integers(l_lo, l_hi + 1, size=len(n)), zero_bias)
