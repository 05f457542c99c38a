"""Helpers for the GPU parity tests: error norms and element-wise bounds (the host<->device
plumbing lives in workloads.device)."""
import numpy as np
import torch

from workloads.device import DEV, empty, to_dev, to_host  # noqa: F401  (re-exported for the tests)


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in GPU output"
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((got - ref).ravel())
    return num / den if den > 0 else num


def assert_elementwise(got, ref, rel, abs_rms, what=""):
    """Every element: |got - ref| <= rel * |ref| + abs_rms * rms(ref).  The relative term is the
    rounding of the stored value, the absolute one (in units of the tensor's rms) the error of
    the fp32 accumulation that produced it."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in GPU output (%s)" % what
    rms = np.sqrt(np.mean(ref * ref)) if ref.size else 0.0
    err = np.abs(got - ref)
    bound = rel * np.abs(ref) + abs_rms * rms
    bad = err > bound
    if np.any(bad):
        i = int(np.argmax(err - bound))
        raise AssertionError("%s: %d of %d elements out of bound; worst at flat index %d: got %r ref %r (bound %.3g)"
                             % (what, int(bad.sum()), err.size, i, got.ravel()[i], ref.ravel()[i], bound.ravel()[i]))


# one rounding to bf16 (8 significant bits: at most 2^-9 of the next power of two, i.e. 2^-8 |value|) of a
# value accumulated in fp32
BF16_REL, BF16_ABS = 1.01 * 2.0 ** -8, 2.0 ** -12
# rel-L2 of one bf16 rounding is about 2^-9 / sqrt(3) .. 2^-8 / sqrt(3): 1.1e-3 .. 2.3e-3
BF16_L2 = 3e-3


def tdtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32
