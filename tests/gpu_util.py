"""Helpers for the GPU parity tests: host<->device plumbing and error norms."""
import numpy as np
import torch

import workloads as W

DEV = "cuda:0"


def to_dev(a, dtype="f32"):
    """numpy -> device tensor.  bf16 inputs must already lie on the bf16 grid."""
    a = np.ascontiguousarray(a)
    if a.dtype in (np.int32, np.int64):
        return torch.from_numpy(a.astype(np.int32)).to(DEV)
    if dtype == "bf16":
        bits = W.bf16_bits(a.astype(np.float32))
        return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a.astype(np.float32)).to(DEV)


def to_host(t):
    """device tensor -> float64 numpy (bf16 widened exactly)."""
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return W.bits_to_f32(bits).astype(np.float64).reshape(tuple(t.shape))
    return t.detach().cpu().numpy().astype(np.float64)


def empty(shape, dtype="f32"):
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    # NaN-fill so that an element the kernel fails to write is caught
    return torch.full(tuple(shape), float("nan"), dtype=td, device=DEV)


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in GPU output"
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((got - ref).ravel())
    return num / den if den > 0 else num


def tdtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32
