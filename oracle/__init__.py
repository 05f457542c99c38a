"""fp64 CPU oracle for the conv-GLU + CTC training path (and the ASG criterion) -- TEST INFRASTRUCTURE ONLY.

Thin ctypes marshalling around ``w2l_oracle.c`` (plain C loops, double precision)
plus :func:`train_step`, which strings those definitions together in the order of
the paper's training loop (Sec. 2.3: network forward, criterion, backward), and
:func:`logmel`, the log-mel feature recipe (Sec. 2.2) in numpy, fp64.

Parity status: :func:`asg` and :func:`logmel` follow definitions the paper only names (it
cites the criterion's source and fixes no feature constant), so both are "parity unpinned" with
respect to the paper's text; each is pinned to its stated definition by brute force, closed
forms and invariants in ``tests/test_oracle_asg.py`` / ``tests/test_oracle_logmel.py``.

Only tests, the smoke check and the bench's ``cpu_baseline`` leg may import this
package.  It shares nothing with the HIP library and never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "w2l_oracle.c")
_LIB = os.path.join(_HERE, "libw2l_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over independent outputs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # W2L_ORACLE_LIB: a build of w2l_oracle.c made elsewhere (the sanitizer run of the tests uses this)
        _lib = C.CDLL(os.environ.get("W2L_ORACLE_LIB") or build())
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def _i(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int))


def _ll(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(C.POINTER(C.c_longlong))


def out_len(T: int, stride: int) -> int:
    return (T + stride - 1) // stride


def num_threads() -> int:
    return int(_load().orc_num_threads())


# ----------------------------------------------------------------------------- conv
def conv1d_fwd(x, w, bias, stride=1):
    """y[b,t',co] = bias[co] + sum_{j,ci} w[co,j,ci] x[b, s t' + j - p, ci]."""
    B, T, Cin = x.shape
    Cout, k, Cin2 = w.shape
    assert Cin2 == Cin and k % 2 == 1
    x, px = _d(x)
    w, pw = _d(w)
    pb = None
    if bias is not None:
        bias, pb = _d(bias)
    y = np.empty((B, out_len(T, stride), Cout))
    _load().orc_conv1d_fwd(px, pw, pb, y.ctypes.data_as(C.POINTER(C.c_double)),
                           B, T, Cin, Cout, k, stride)
    return y


def conv1d_fwd_at(x, w, bias, idx, stride=1):
    B, T, Cin = x.shape
    Cout, k, _ = w.shape
    x, px = _d(x)
    w, pw = _d(w)
    pb = None
    if bias is not None:
        bias, pb = _d(bias)
    idx, pi = _ll(idx)
    out = np.empty(idx.size)
    _load().orc_conv1d_fwd_at(px, pw, pb, pi, idx.size, out.ctypes.data_as(C.POINTER(C.c_double)),
                              B, T, Cin, Cout, k, stride)
    return out


def conv1d_bwd_data(dy, w, T, stride=1):
    """dx = transpose of x -> conv(x, w) applied to dy; T is the input length."""
    B, Tp, Cout = dy.shape
    Cout2, k, Cin = w.shape
    assert Cout2 == Cout and Tp == out_len(T, stride)
    dy, pdy = _d(dy)
    w, pw = _d(w)
    dx = np.empty((B, T, Cin))
    _load().orc_conv1d_bwd_data(pdy, pw, dx.ctypes.data_as(C.POINTER(C.c_double)),
                                B, T, Cin, Cout, k, stride)
    return dx


def conv1d_bwd_data_at(dy, w, T, idx, stride=1):
    B, Tp, Cout = dy.shape
    _, k, Cin = w.shape
    dy, pdy = _d(dy)
    w, pw = _d(w)
    idx, pi = _ll(idx)
    out = np.empty(idx.size)
    _load().orc_conv1d_bwd_data_at(pdy, pw, pi, idx.size, out.ctypes.data_as(C.POINTER(C.c_double)),
                                   B, T, Cin, Cout, k, stride)
    return out


def conv1d_bwd_weight(x, dy, k, stride=1, want_dbias=True):
    B, T, Cin = x.shape
    B2, Tp, Cout = dy.shape
    assert B2 == B and Tp == out_len(T, stride)
    x, px = _d(x)
    dy, pdy = _d(dy)
    dw = np.empty((Cout, k, Cin))
    db = np.empty(Cout) if want_dbias else None
    _load().orc_conv1d_bwd_weight(px, pdy, dw.ctypes.data_as(C.POINTER(C.c_double)),
                                  db.ctypes.data_as(C.POINTER(C.c_double)) if want_dbias else None,
                                  B, T, Cin, Cout, k, stride)
    return dw, db


def conv1d_bwd_weight_at(x, dy, k, idx, stride=1):
    B, T, Cin = x.shape
    _, _, Cout = dy.shape
    x, px = _d(x)
    dy, pdy = _d(dy)
    idx, pi = _ll(idx)
    out = np.empty(idx.size)
    _load().orc_conv1d_bwd_weight_at(px, pdy, pi, idx.size, out.ctypes.data_as(C.POINTER(C.c_double)),
                                     B, T, Cin, Cout, k, stride)
    return out


# ----------------------------------------------------------------------------- elementwise
def glu_fwd(y):
    """h = y[..., :C/2] * sigmoid(y[..., C/2:])."""
    Cout = y.shape[-1]
    assert Cout % 2 == 0
    y, py = _d(y)
    h = np.empty(y.shape[:-1] + (Cout // 2,))
    _load().orc_glu_fwd(py, h.ctypes.data_as(C.POINTER(C.c_double)),
                        C.c_longlong(y.size // Cout), Cout)
    return h


def glu_bwd(y, dh):
    Cout = y.shape[-1]
    y, py = _d(y)
    dh, pdh = _d(dh)
    dy = np.empty(y.shape)
    _load().orc_glu_bwd(py, pdh, dy.ctypes.data_as(C.POINTER(C.c_double)),
                        C.c_longlong(y.size // Cout), Cout)
    return dy


def logsoftmax_fwd(z):
    Cc = z.shape[-1]
    z, pz = _d(z)
    lp = np.empty(z.shape)
    _load().orc_logsoftmax_fwd(pz, lp.ctypes.data_as(C.POINTER(C.c_double)),
                               C.c_longlong(z.size // Cc), Cc)
    return lp


def logsoftmax_bwd(lp, dlp):
    Cc = lp.shape[-1]
    lp, plp = _d(lp)
    dlp, pd = _d(dlp)
    dz = np.empty(lp.shape)
    _load().orc_logsoftmax_bwd(plp, pd, dz.ctypes.data_as(C.POINTER(C.c_double)),
                               C.c_longlong(lp.size // Cc), Cc)
    return dz


# ----------------------------------------------------------------------------- optimiser
def sgd_momentum(w, v, g, lr, momentum, weight_decay=0.0):
    """One SGD-with-momentum update (Sec. 4.1; heavy-ball form): returns (w', v') with
    v' = momentum * v + (g + weight_decay * w),  w' = w - lr * v'.  Inputs are not modified."""
    w2 = np.array(w, dtype=np.float64, copy=True).ravel()
    v2 = np.array(v, dtype=np.float64, copy=True).ravel()
    g2, pg = _d(np.asarray(g).ravel())
    assert w2.size == v2.size == g2.size
    _load().orc_sgd_momentum(w2.ctypes.data_as(C.POINTER(C.c_double)), v2.ctypes.data_as(C.POINTER(C.c_double)), pg,
                             C.c_longlong(w2.size), C.c_double(lr), C.c_double(momentum), C.c_double(weight_decay))
    return w2.reshape(np.shape(w)), v2.reshape(np.shape(v))


# ----------------------------------------------------------------------------- CTC
def ctc(lp, targets, in_len, tgt_len, blank=0, want_lattice=False):
    """Per-utterance CTC loss and d(sum_b loss_b)/d lp (= -G), from log-probabilities.

    Returns (loss[B], grad_lp[B,Tp,C]) and, if ``want_lattice``, also the alpha
    and beta lattices [B,Tp,2*Lmax+1] (-inf where unused).
    """
    B, Tp, Cc = lp.shape
    targets = np.asarray(targets, dtype=np.int32).reshape(B, -1)
    Lmax = targets.shape[1]
    if Lmax == 0:
        targets = np.zeros((B, 1), dtype=np.int32)
        Lmax = 1
    lp, plp = _d(lp)
    targets, pt = _i(targets)
    in_len, pil = _i(in_len)
    tgt_len, ptl = _i(tgt_len)
    loss = np.empty(B)
    grad = np.empty((B, Tp, Cc))
    al = be = None
    pal = pbe = None
    if want_lattice:
        al = np.empty((B, Tp, 2 * Lmax + 1))
        be = np.empty((B, Tp, 2 * Lmax + 1))
        pal = al.ctypes.data_as(C.POINTER(C.c_double))
        pbe = be.ctypes.data_as(C.POINTER(C.c_double))
    rc = _load().orc_ctc(plp, pt, pil, ptl, loss.ctypes.data_as(C.POINTER(C.c_double)),
                         grad.ctypes.data_as(C.POINTER(C.c_double)), pal, pbe,
                         B, Tp, Cc, Lmax, blank)
    if rc != 0:
        raise ValueError("invalid CTC target or length")
    if want_lattice:
        return loss, grad, al, be
    return loss, grad


def ctc_from_logits(z, targets, in_len, tgt_len, blank=0, grad_scale=1.0):
    """log-softmax then CTC; returns (loss[B], lp, d(grad_scale * sum_b loss_b)/dz)."""
    lp = logsoftmax_fwd(z)
    loss, dlp = ctc(lp, targets, in_len, tgt_len, blank)
    dz = logsoftmax_bwd(lp, dlp) * grad_scale
    return loss, lp, dz


# ----------------------------------------------------------------------------- ASG
def asg(em, trans, targets, in_len, tgt_len, grad_scale=1.0, want_terms=False):
    """ASG criterion (Sec. 2.3 names it; definition: see ``orc_asg``): loss[b] = FCC_b - FAL_b from
    unnormalised emissions em[B,Tp,C] and transitions trans[C,C] (trans[i,j]: class j followed by
    class i).  Returns (loss[B], d em [B,Tp,C], d trans [C,C]) with both gradients of
    grad_scale * sum_b loss_b, and with ``want_terms`` also (FCC[B], FAL[B])."""
    B, Tp, Cc = em.shape
    targets = np.asarray(targets, dtype=np.int32).reshape(B, -1)
    Lmax = targets.shape[1]
    if Lmax == 0:
        targets = np.zeros((B, 1), dtype=np.int32)
        Lmax = 1
    em, pe = _d(em)
    trans, ptr = _d(trans)
    assert trans.shape == (Cc, Cc)
    targets, pt = _i(targets)
    in_len, pil = _i(in_len)
    tgt_len, ptl = _i(tgt_len)
    dp = lambda a: a.ctypes.data_as(C.POINTER(C.c_double))
    loss, ge, gt, fcc, fal = np.empty(B), np.empty((B, Tp, Cc)), np.empty((Cc, Cc)), np.empty(B), np.empty(B)
    rc = _load().orc_asg(pe, ptr, pt, pil, ptl, dp(loss), dp(ge), dp(gt), dp(fcc), dp(fal), B, Tp, Cc, Lmax)
    if rc != 0:
        raise ValueError("invalid ASG target or length")
    ge *= grad_scale
    gt *= grad_scale
    if want_terms:
        return loss, ge, gt, fcc, fal
    return loss, ge, gt


# ----------------------------------------------------------------------------- log-mel features
def logmel_num_frames(n_samples: int, win: int, hop: int) -> int:
    """Frames that lie wholly inside the signal: 1 + floor((n - win) / hop), or 0 if n < win."""
    return 0 if n_samples < win else 1 + (n_samples - win) // hop


def mel_of_hz(f):
    """The mel scale m = 2595 log10(1 + f / 700)."""
    return 2595.0 * np.log10(1.0 + np.asarray(f, dtype=np.float64) / 700.0)


def hz_of_mel(m):
    return 700.0 * (10.0 ** (np.asarray(m, dtype=np.float64) / 2595.0) - 1.0)


def mel_filterbank(n_mels, nfft, sample_rate, fmin, fmax):
    """[n_mels, nfft/2+1] triangular filters, peak 1: n_mels + 2 points equally spaced on the mel
    scale between fmin and fmax; filter f rises linearly (in Hz) from point f to point f+1 and falls
    to point f+2, evaluated at the DFT bin frequencies k * sample_rate / nfft."""
    pts = hz_of_mel(np.linspace(mel_of_hz(fmin), mel_of_hz(fmax), n_mels + 2))
    freqs = np.arange(nfft // 2 + 1, dtype=np.float64) * sample_rate / nfft
    fb = np.zeros((n_mels, nfft // 2 + 1))
    for f in range(n_mels):
        lo, ce, hi = pts[f], pts[f + 1], pts[f + 2]
        up = (freqs - lo) / (ce - lo)
        down = (hi - freqs) / (hi - ce)
        fb[f] = np.maximum(0.0, np.minimum(up, down))
    return fb


def logmel(wav, wav_len, n_mels=40, sample_rate=16000, win=400, hop=160, nfft=512, fmin=0.0, fmax=None,
           floor=1e-10, Tmax=None):
    """Log-mel filterbank features (Sec. 2.2 lists them among the feature types, Sec. 4.1 uses 40 of
    them per frame; the paper gives no constant or formula -- the steps below are a stated reading):
    frames of ``win`` samples every ``hop`` samples, only frames wholly inside the signal;
    Hamming window 0.54 - 0.46 cos(2 pi n / (win - 1)); zero-padded DFT of size nfft; power
    spectrum |X_k|^2, k = 0..nfft/2; triangular mel filterbank; natural log of max(energy, floor).
    wav: [B, Nmax]; wav_len: [B].  Returns (feat [B, Tmax, n_mels] with zeros beyond each
    utterance's frames, feat_len [B])."""
    wav = np.asarray(wav, dtype=np.float64)
    B = wav.shape[0]
    fmax = sample_rate / 2.0 if fmax is None else fmax
    nfr = [logmel_num_frames(int(n), win, hop) for n in wav_len]
    if Tmax is None:
        Tmax = max(nfr + [0])
    fb = mel_filterbank(n_mels, nfft, sample_rate, fmin, fmax)
    window = 0.54 - 0.46 * np.cos(2.0 * np.pi * np.arange(win) / (win - 1))
    feat = np.zeros((B, Tmax, n_mels))
    out_len = np.zeros(B, dtype=np.int32)
    for b in range(B):
        T = min(nfr[b], Tmax)
        out_len[b] = T
        for t in range(T):
            seg = wav[b, t * hop:t * hop + win] * window
            spec = np.fft.rfft(seg, n=nfft)
            power = spec.real ** 2 + spec.imag ** 2
            feat[b, t] = np.log(np.maximum(fb @ power, floor))
    return feat, out_len


# ----------------------------------------------------------------------------- train step
def train_step(layers, weights, biases, x, in_len, targets, tgt_len, grad_scale=1.0, blank=0,
               keep_activations=False, trans=None):
    """Forward + backward of the conv-GLU network with the CTC criterion, or -- if a transition
    matrix ``trans`` is given -- with the ASG criterion on the network output as emissions (then
    the result also holds dtrans, and lp is None).

    ``layers`` is a list of dicts {k, stride, cin, cout, glu}.  ``in_len`` counts
    valid input frames per utterance (frames beyond it are expected to be zero in
    ``x``); the criterion sees ceil(in_len / total stride) frames.  Returns a dict
    with loss[B], logits, lp, dlogits, dw (list), db (list) and optionally the
    per-layer activations.  Gradients are those of grad_scale * sum_b loss_b.
    """
    h = np.asarray(x, dtype=np.float64)
    saved_in, saved_pre = [], []
    tot_stride = 1
    for L, w, b in zip(layers, weights, biases):
        saved_in.append(h)
        y = conv1d_fwd(h, w, b, L["stride"])
        saved_pre.append(y)
        h = glu_fwd(y) if L["glu"] else y
        tot_stride *= L["stride"]
    logits = h
    crit_len = np.array([out_len(int(n), tot_stride) for n in in_len], dtype=np.int32)
    dtrans = None
    if trans is None:
        loss, lp, dz = ctc_from_logits(logits, targets, crit_len, tgt_len, blank, grad_scale)
    else:
        loss, dz, dtrans = asg(logits, trans, targets, crit_len, tgt_len, grad_scale)
        lp = None
    dws, dbs = [None] * len(layers), [None] * len(layers)
    dh = dz
    for i in range(len(layers) - 1, -1, -1):
        L = layers[i]
        dy = glu_bwd(saved_pre[i], dh) if L["glu"] else dh
        dws[i], dbs[i] = conv1d_bwd_weight(saved_in[i], dy, L["k"], L["stride"])
        if i > 0:
            dh = conv1d_bwd_data(dy, weights[i], saved_in[i].shape[1], L["stride"])
    out = dict(loss=loss, logits=logits, lp=lp, dlogits=dz, dw=dws, db=dbs, crit_len=crit_len, dtrans=dtrans)
    if keep_activations:
        out["inputs"] = saved_in
        out["pre"] = saved_pre
    return out
