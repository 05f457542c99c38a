"""Host <-> device plumbing for callers of the library (tests, bench.py, the smoke check): numpy
arrays become torch CUDA tensors and back.  torch serves as the allocator only; nothing here
computes anything of the method."""
import numpy as np
import torch

from . import bf16_bits, bits_to_f32

DEV = "cuda:0"


def to_dev(a, dtype="f32"):
    """numpy -> device tensor.  bf16 inputs must already lie on the bf16 grid."""
    a = np.ascontiguousarray(a)
    if a.dtype in (np.int32, np.int64):
        return torch.from_numpy(a.astype(np.int32)).to(DEV)
    if dtype == "bf16":
        bits = bf16_bits(a.astype(np.float32))
        return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a.astype(np.float32)).to(DEV)


def to_host(t):
    """device tensor -> float64 numpy (bf16 widened exactly)."""
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return bits_to_f32(bits).astype(np.float64).reshape(tuple(t.shape))
    return t.detach().cpu().numpy().astype(np.float64)


def empty(shape, dtype="f32"):
    """An output buffer filled with NaN, so that an element a kernel fails to write is caught."""
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    return torch.full(tuple(shape), float("nan"), dtype=td, device=DEV)


def run_train_step(P, cfg, grad_scale=1.0, want_logits=True):
    """One w2l_train_step call on a model batch from this package's generators; returns host copies
    of loss, logits and every weight/bias gradient (float64).  P: the binding module."""
    dt = cfg["dtype"]
    layers = cfg["layers"]
    B, T = cfg["B"], cfg["T"]
    xd = to_dev(cfg["x"], dt)
    wd = [to_dev(w, dt) for w in cfg["weights"]]
    bd = [to_dev(b) for b in cfg["biases"]]
    dwd = [empty(w.shape) for w in cfg["weights"]]
    dbd = [empty(b.shape) for b in cfg["biases"]]
    tg, il, tl = to_dev(cfg["targets"]), to_dev(cfg["in_len"]), to_dev(cfg["tgt_len"])
    Lmax = cfg["targets"].shape[1]
    code = P.W2L_BF16 if dt == "bf16" else P.W2L_F32
    ws = P.workspace(P.w2l_train_step_workspace_bytes(layers, B, T, Lmax, code))
    loss = empty((B,))
    Tl = T
    for L in layers:
        Tl = (Tl + L["stride"] - 1) // L["stride"]
    logits = empty((B, Tl, layers[-1]["cout"])) if want_logits else None
    P.w2l_train_step(layers, wd, bd, dwd, dbd, xd, il, tg, tl, loss, logits, cfg["blank"], grad_scale, ws)
    torch.cuda.synchronize()
    return dict(loss=to_host(loss), logits=to_host(logits) if want_logits else None,
                dw=[to_host(t) for t in dwd], db=[to_host(t) for t in dbd])
