"""ctypes binding of libw2l.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA tensors used purely as device buffers (``data_ptr()``); every
step of the path runs inside the library's kernels on ``stream`` (default: torch's
current stream).  A non-zero status raises :class:`W2LError`.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

W2L_F32, W2L_BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
# W2L_LIB: another build of the same sources (the sanitizer run of the host-side tests uses this)
_LIB_PATH = os.environ.get("W2L_LIB") or os.path.join(_HERE, "libw2l.so")

__all__ = [
    "W2L_F32", "W2L_BF16", "W2LError", "w2l_layer", "w2l_version", "w2l_status_str", "w2l_last_hip_error",
    "w2l_conv1d_fwd", "w2l_conv1d_bwd_data", "w2l_conv1d_bwd_weight", "w2l_conv1d_fwd_workspace_bytes",
    "w2l_conv1d_bwd_data_workspace_bytes", "w2l_conv1d_bwd_weight_workspace_bytes", "w2l_glu_fwd", "w2l_glu_bwd",
    "w2l_logsoftmax_fwd", "w2l_logsoftmax_bwd", "w2l_ctc_workspace_bytes", "w2l_ctc_fwd_bwd", "w2l_ctc_fwd_bwd_noalloc",
    "w2l_ctc_check_targets_host", "w2l_ctc_launch_config", "w2l_asg_launch_config", "w2l_asg_workspace_bytes", "w2l_asg_fwd_bwd", "w2l_asg_check_targets_host",
    "w2l_logmel_num_frames", "w2l_logmel_fwd",
    "w2l_train_step_workspace_bytes", "w2l_train_step", "w2l_train_step_asg_workspace_bytes", "w2l_train_step_asg",
    "w2l_sgd_momentum_step",
    "w2l_probe_mfma", "raw",
    "workspace",
]


class W2LError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, w2l_status_str(status)))


class w2l_layer(C.Structure):
    _fields_ = [("k", C.c_int), ("stride", C.c_int), ("cin", C.c_int), ("cout", C.c_int), ("glu", C.c_int)]


def lib_path() -> str:
    return _LIB_PATH


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "libw2l.so is not built (%s). Run `python -m paper_1812_07625_amd.build`; there is no "
            "fallback path." % _LIB_PATH)
    lib = C.CDLL(_LIB_PATH)
    vp, i, ll, sz, f = C.c_void_p, C.c_int, C.c_longlong, C.c_size_t, C.c_float
    sig = {
        "w2l_version": (i, []),
        "w2l_status_str": (C.c_char_p, [i]),
        "w2l_last_hip_error": (i, []),
        "w2l_conv1d_fwd_workspace_bytes": (sz, [i] * 7),
        "w2l_conv1d_bwd_data_workspace_bytes": (sz, [i] * 7),
        "w2l_conv1d_bwd_weight_workspace_bytes": (sz, [i] * 7),
        "w2l_conv1d_fwd": (i, [vp, vp, vp, vp] + [i] * 8 + [vp, sz, vp]),
        "w2l_conv1d_bwd_data": (i, [vp, vp, vp] + [i] * 8 + [vp, sz, vp]),
        "w2l_conv1d_bwd_weight": (i, [vp, vp, vp, vp] + [i] * 9 + [vp, sz, vp]),
        "w2l_glu_fwd": (i, [vp, vp, ll, i, i, vp]),
        "w2l_glu_bwd": (i, [vp, vp, vp, ll, i, i, vp]),
        "w2l_logsoftmax_fwd": (i, [vp, vp, ll, i, i, vp]),
        "w2l_logsoftmax_bwd": (i, [vp, vp, vp, ll, i, vp]),
        "w2l_ctc_workspace_bytes": (sz, [i] * 4),
        "w2l_ctc_fwd_bwd": (i, [vp, i, vp, vp, vp, vp, vp, i, i, i, i, i, f, vp, sz, vp]),
        "w2l_ctc_fwd_bwd_noalloc": (i, [vp, i, vp, vp, vp, vp, vp, i, i, i, i, i, f, vp]),
        "w2l_ctc_check_targets_host": (i, [vp, vp, vp, i, i, i, i, i]),
        "w2l_ctc_launch_config": (i, [i, i] + [C.POINTER(C.c_int)] * 4),
        "w2l_asg_launch_config": (i, [i, i] + [C.POINTER(C.c_int)] * 6),
        "w2l_logmel_num_frames": (i, [i, i, i]),
        "w2l_logmel_fwd": (i, [vp, vp, vp, vp, i, i, i, i, i, i, i, i, f, f, f, i, vp]),
        "w2l_asg_workspace_bytes": (sz, [i] * 4),
        "w2l_asg_fwd_bwd": (i, [vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, f, vp, sz, vp]),
        "w2l_asg_check_targets_host": (i, [vp, vp, vp, i, i, i, i]),
        "w2l_probe_mfma": (i, [vp, i, i, i, vp]),
        "w2l_sgd_momentum_step": (i, [vp, vp, vp, vp, ll, f, f, f, vp]),
        "w2l_train_step_workspace_bytes": (sz, [C.POINTER(w2l_layer), i, i, i, i, i]),
        "w2l_train_step": (i, [C.POINTER(w2l_layer), i, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                               C.POINTER(vp), vp, vp, vp, vp, vp, vp, i, i, i, i, i, f, vp, sz, vp]),
        "w2l_train_step_asg_workspace_bytes": (sz, [C.POINTER(w2l_layer), i, i, i, i, i]),
        "w2l_train_step_asg": (i, [C.POINTER(w2l_layer), i, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                   C.POINTER(vp), vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, f, vp, sz, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


raw = _load()  # the CDLL itself, for callers that pass raw pointers (error-path tests)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return W2L_F32
    if t.dtype == torch.bfloat16:
        return W2L_BF16
    raise TypeError("unsupported tensor dtype %s" % t.dtype)


def _p(t):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else stream


def _ws(workspace):
    if workspace is None:
        return None, 0
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def _check(rc, where):
    if rc != 0:
        raise W2LError(rc, where)


def workspace(nbytes: int, device="cuda:0") -> torch.Tensor:
    """A device byte buffer of at least ``nbytes`` (256-byte aligned by torch's allocator)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def w2l_version() -> int:
    return raw.w2l_version()


def w2l_status_str(status: int) -> str:
    return raw.w2l_status_str(status).decode()


def w2l_last_hip_error() -> int:
    return raw.w2l_last_hip_error()


def w2l_conv1d_fwd_workspace_bytes(B, T, Cin, Cout, k, stride, dtype) -> int:
    return raw.w2l_conv1d_fwd_workspace_bytes(B, T, Cin, Cout, k, stride, dtype)


def w2l_conv1d_bwd_data_workspace_bytes(B, T, Cin, Cout, k, stride, dtype) -> int:
    return raw.w2l_conv1d_bwd_data_workspace_bytes(B, T, Cin, Cout, k, stride, dtype)


def w2l_conv1d_bwd_weight_workspace_bytes(B, T, Cin, Cout, k, stride, dtype) -> int:
    return raw.w2l_conv1d_bwd_weight_workspace_bytes(B, T, Cin, Cout, k, stride, dtype)


def w2l_conv1d_fwd(x, w, bias, y, stride=1, workspace=None, stream=None):
    """y[B,T',Cout] = conv1d(x[B,T,Cin], w[Cout,k,Cin]) + bias."""
    B, T, Cin = x.shape
    Cout, k, _ = w.shape
    wp, wn = _ws(workspace)
    _check(raw.w2l_conv1d_fwd(_p(x), _p(w), _p(bias), _p(y), B, T, Cin, Cout, k, stride, _dt(x), _dt(y),
                              wp, wn, _stream(stream)), "w2l_conv1d_fwd")
    return y


def w2l_conv1d_bwd_data(dy, w, dx, stride=1, workspace=None, stream=None):
    B, T, Cin = dx.shape
    Cout, k, _ = w.shape
    wp, wn = _ws(workspace)
    _check(raw.w2l_conv1d_bwd_data(_p(dy), _p(w), _p(dx), B, T, Cin, Cout, k, stride, _dt(w), _dt(dy),
                                   wp, wn, _stream(stream)), "w2l_conv1d_bwd_data")
    return dx


def w2l_conv1d_bwd_weight(x, dy, dw, dbias, stride=1, accumulate=False, workspace=None, stream=None):
    B, T, Cin = x.shape
    Cout, k, _ = dw.shape
    wp, wn = _ws(workspace)
    _check(raw.w2l_conv1d_bwd_weight(_p(x), _p(dy), _p(dw), _p(dbias), B, T, Cin, Cout, k, stride, _dt(x),
                                     _dt(dy), int(accumulate), wp, wn, _stream(stream)),
           "w2l_conv1d_bwd_weight")
    return dw, dbias


def w2l_glu_fwd(y, h, stream=None):
    Cout = y.shape[-1]
    _check(raw.w2l_glu_fwd(_p(y), _p(h), y.numel() // Cout, Cout, _dt(y), _stream(stream)), "w2l_glu_fwd")
    return h


def w2l_glu_bwd(y, dh, dy, stream=None):
    Cout = y.shape[-1]
    _check(raw.w2l_glu_bwd(_p(y), _p(dh), _p(dy), y.numel() // Cout, Cout, _dt(y), _stream(stream)),
           "w2l_glu_bwd")
    return dy


def w2l_logsoftmax_fwd(z, lp, stream=None):
    Cc = z.shape[-1]
    _check(raw.w2l_logsoftmax_fwd(_p(z), _p(lp), z.numel() // Cc, Cc, _dt(z), _stream(stream)),
           "w2l_logsoftmax_fwd")
    return lp


def w2l_logsoftmax_bwd(lp, dlp, dz, stream=None):
    Cc = lp.shape[-1]
    _check(raw.w2l_logsoftmax_bwd(_p(lp), _p(dlp), _p(dz), lp.numel() // Cc, Cc, _stream(stream)),
           "w2l_logsoftmax_bwd")
    return dz


def w2l_sgd_momentum_step(w, v, grad, w_lowp, lr, momentum, weight_decay=0.0, stream=None):
    _check(raw.w2l_sgd_momentum_step(_p(w), _p(v), _p(grad), _p(w_lowp) if w_lowp is not None else None,
                                     w.numel(), float(lr), float(momentum), float(weight_decay), _stream(stream)),
           "w2l_sgd_momentum_step")
    return w


def w2l_ctc_workspace_bytes(B, Tp, Cc, Lmax) -> int:
    return raw.w2l_ctc_workspace_bytes(B, Tp, Cc, Lmax)


def w2l_ctc_fwd_bwd(inp, is_logits, targets, in_len, tgt_len, loss, grad, blank=0, grad_scale=1.0,
                    workspace=None, stream=None):
    B, Tp, Cc = inp.shape
    Lmax = targets.shape[1]
    wp, wn = _ws(workspace)
    _check(raw.w2l_ctc_fwd_bwd(_p(inp), int(is_logits), _p(targets), _p(in_len), _p(tgt_len), _p(loss),
                               _p(grad), B, Tp, Cc, Lmax, blank, float(grad_scale), wp, wn, _stream(stream)),
           "w2l_ctc_fwd_bwd")
    return loss, grad


def w2l_ctc_fwd_bwd_noalloc(inp, is_logits, targets, in_len, tgt_len, loss, grad, blank=0, grad_scale=1.0, stream=None):
    """w2l_ctc_fwd_bwd on the library's static scratch array: no workspace, no allocation."""
    B, Tp, Cc = inp.shape
    Lmax = targets.shape[1]
    _check(raw.w2l_ctc_fwd_bwd_noalloc(_p(inp), int(is_logits), _p(targets), _p(in_len), _p(tgt_len), _p(loss),
                                       _p(grad), B, Tp, Cc, Lmax, blank, float(grad_scale), _stream(stream)),
           "w2l_ctc_fwd_bwd_noalloc")
    return loss, grad


def w2l_ctc_check_targets_host(targets, in_len, tgt_len, Tp, Cc, blank=0) -> int:
    """numpy int32 host arrays; returns the status instead of raising."""
    import numpy as np
    t = np.ascontiguousarray(targets, dtype=np.int32)
    il = np.ascontiguousarray(in_len, dtype=np.int32)
    tl = np.ascontiguousarray(tgt_len, dtype=np.int32)
    return raw.w2l_ctc_check_targets_host(t.ctypes.data, il.ctypes.data, tl.ctypes.data, t.shape[0], Tp, Cc,
                                          t.shape[1], blank)


def w2l_ctc_launch_config(Cc, Lmax):
    """(pairs per lane, table values per thread, frames per block, threads) of the alpha/beta kernel; host only."""
    out = [C.c_int() for _ in range(4)]
    _check(raw.w2l_ctc_launch_config(Cc, Lmax, *[C.byref(o) for o in out]), "w2l_ctc_launch_config")
    return tuple(o.value for o in out)


def w2l_asg_launch_config(Cc, Lmax):
    """(positions per lane, class lanes, max threads, frames per block, row values per thread, threads); host only."""
    out = [C.c_int() for _ in range(6)]
    _check(raw.w2l_asg_launch_config(Cc, Lmax, *[C.byref(o) for o in out]), "w2l_asg_launch_config")
    return tuple(o.value for o in out)


def w2l_logmel_num_frames(n_samples, win=400, hop=160) -> int:
    return raw.w2l_logmel_num_frames(int(n_samples), win, hop)


def w2l_logmel_fwd(wav, wav_len, feat, feat_len, sample_rate=16000, win=400, hop=160, nfft=512, fmin=0.0,
                   fmax=None, floor=1e-10, stream=None):
    B, Nmax = wav.shape
    _, Tmax, n_mels = feat.shape
    fmax = sample_rate / 2.0 if fmax is None else fmax
    _check(raw.w2l_logmel_fwd(_p(wav), _p(wav_len), _p(feat), _p(feat_len), B, Nmax, Tmax, n_mels, sample_rate, win, hop,
                              nfft, float(fmin), float(fmax), float(floor), _dt(feat), _stream(stream)),
           "w2l_logmel_fwd")
    return feat, feat_len


def w2l_asg_workspace_bytes(B, Tp, Cc, Lmax) -> int:
    return raw.w2l_asg_workspace_bytes(B, Tp, Cc, Lmax)


def w2l_asg_fwd_bwd(emissions, trans, targets, in_len, tgt_len, loss, grad_emissions, grad_trans=None,
                    grad_scale=1.0, workspace=None, stream=None):
    B, Tp, Cc = emissions.shape
    Lmax = targets.shape[1]
    wp, wn = _ws(workspace)
    _check(raw.w2l_asg_fwd_bwd(_p(emissions), _p(trans), _p(targets), _p(in_len), _p(tgt_len), _p(loss),
                               _p(grad_emissions), _p(grad_trans) if grad_trans is not None else None,
                               B, Tp, Cc, Lmax, float(grad_scale), wp, wn, _stream(stream)),
           "w2l_asg_fwd_bwd")
    return loss, grad_emissions, grad_trans


def w2l_asg_check_targets_host(targets, in_len, tgt_len, Tp, Cc) -> int:
    """numpy int32 host arrays; returns the status instead of raising."""
    import numpy as np
    t = np.ascontiguousarray(targets, dtype=np.int32)
    il = np.ascontiguousarray(in_len, dtype=np.int32)
    tl = np.ascontiguousarray(tgt_len, dtype=np.int32)
    return raw.w2l_asg_check_targets_host(t.ctypes.data, il.ctypes.data, tl.ctypes.data, t.shape[0], Tp, Cc,
                                          t.shape[1])


def w2l_probe_mfma(out, blocks, iters, random_operands=False, stream=None):
    """Measurement aid: blocks*4 wavefronts each issue 8*iters MFMAs (32768 FLOP each); returns the FLOP count."""
    _check(raw.w2l_probe_mfma(_p(out), blocks, iters, int(bool(random_operands)), _stream(stream)), "w2l_probe_mfma")
    return 2.0 * 32 * 32 * 16 * 8 * iters * blocks * 4


def _layer_array(layers):
    arr = (w2l_layer * len(layers))()
    for a, L in zip(arr, layers):
        a.k, a.stride, a.cin, a.cout, a.glu = L["k"], L["stride"], L["cin"], L["cout"], L["glu"]
    return arr


def w2l_train_step_workspace_bytes(layers, B, T, Lmax, dtype) -> int:
    arr = _layer_array(layers)
    return raw.w2l_train_step_workspace_bytes(arr, len(layers), B, T, Lmax, dtype)


def w2l_train_step(layers, weights, biases, dweights, dbiases, x, in_len, targets, tgt_len, loss,
                   logits=None, blank=0, grad_scale=1.0, workspace=None, stream=None):
    n = len(layers)
    arr = _layer_array(layers)
    tab = lambda ts: (C.c_void_p * n)(*[_p(t) for t in ts])
    B, T, _ = x.shape
    wp, wn = _ws(workspace)
    _check(raw.w2l_train_step(arr, n, tab(weights), tab(biases), tab(dweights), tab(dbiases), _p(x),
                              _p(in_len), _p(targets), _p(tgt_len), _p(loss), _p(logits), B, T,
                              targets.shape[1], blank, _dt(x), float(grad_scale), wp, wn, _stream(stream)),
           "w2l_train_step")
    return loss


def w2l_train_step_asg_workspace_bytes(layers, B, T, Lmax, dtype) -> int:
    arr = _layer_array(layers)
    return raw.w2l_train_step_asg_workspace_bytes(arr, len(layers), B, T, Lmax, dtype)


def w2l_train_step_asg(layers, weights, biases, dweights, dbiases, x, in_len, targets, tgt_len, trans, dtrans, loss,
                       logits=None, grad_scale=1.0, workspace=None, stream=None):
    n = len(layers)
    arr = _layer_array(layers)
    tab = lambda ts: (C.c_void_p * n)(*[_p(t) for t in ts])
    B, T, _ = x.shape
    wp, wn = _ws(workspace)
    _check(raw.w2l_train_step_asg(arr, n, tab(weights), tab(biases), tab(dweights), tab(dbiases), _p(x),
                                  _p(in_len), _p(targets), _p(tgt_len), _p(trans), _p(dtrans), _p(loss), _p(logits),
                                  B, T, targets.shape[1], _dt(x), float(grad_scale), wp, wn, _stream(stream)),
           "w2l_train_step_asg")
    return loss
