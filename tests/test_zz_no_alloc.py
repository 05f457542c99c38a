"""w2l_ctc_fwd_bwd_noalloc -- the CTC criterion on the library's static scratch array, for callers
that cannot allocate device memory -- against w2l_ctc_fwd_bwd (caller workspace) through the C ABI.

Both entry points launch the same kernels on the same inputs, so the results must be bit-identical
(stricter than the 1e-4 criterion tolerance); the workspace variant is itself held to the oracle
elsewhere, and once more here.  Two calls in a row share the array, the second on a smaller input:
what the first left behind must not leak into the second.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import empty, to_dev

pytestmark = pytest.mark.gpu


def _both(P, cfg, is_logits=1, scale=1.0):
    B, Tp, Cc = cfg["logits"].shape
    Lmax = cfg["targets"].shape[1]
    inp = cfg["logits"] if is_logits else oracle.logsoftmax_fwd(cfg["logits"].astype(np.float64)).astype(np.float32)
    z, tg, il, tl = to_dev(inp), to_dev(cfg["targets"]), to_dev(cfg["in_len"]), to_dev(cfg["tgt_len"])
    need = P.w2l_ctc_workspace_bytes(B, Tp, Cc, Lmax)
    assert need <= 32 << 20
    l0, g0 = P.w2l_ctc_fwd_bwd(z, is_logits, tg, il, tl, empty((B,)), empty((B, Tp, Cc)), 0, scale, P.workspace(need))
    l1, g1 = P.w2l_ctc_fwd_bwd_noalloc(z, is_logits, tg, il, tl, empty((B,)), empty((B, Tp, Cc)), 0, scale)
    torch.cuda.synchronize()
    return (l0.cpu().numpy(), g0.cpu().numpy()), (l1.cpu().numpy(), g1.cpu().numpy()), inp


def test_noalloc_matches_workspace_variant_twice_in_a_row():
    import paper_1812_07625_amd as P
    # first call: the criterion shape of the 100M-parameter model's batch (B=8, 750 frames, targets up to 150)
    big = W.config2(seed=31, B=8, T=750, in_lo=500, in_hi=750, l_lo=60, l_hi=150)
    # second call, smaller in every dimension: fewer utterances, frames, classes and labels
    small = W.config2(seed=32, B=3, T=90, in_lo=40, in_hi=90, l_lo=2, l_hi=20, Cc=11)
    for cfg, is_logits, scale in ((big, 1, 1.0), (small, 0, 0.5)):
        (l0, g0), (l1, g1), inp = _both(P, cfg, is_logits, scale)
        assert np.array_equal(l0, l1) and np.array_equal(g0, g1)
        assert np.all(np.isfinite(l1)) and np.all(np.isfinite(g1))
        x64 = inp.astype(np.float64)
        if is_logits:
            loss_o, _, g_o = oracle.ctc_from_logits(x64, cfg["targets"], cfg["in_len"], cfg["tgt_len"])
        else:
            loss_o, g_o = oracle.ctc(x64, cfg["targets"], cfg["in_len"], cfg["tgt_len"], 0)
        assert np.all(np.abs(l1 - loss_o) <= 1e-4 * np.abs(loss_o))
        for b in range(cfg["B"]):
            assert np.linalg.norm(g1[b] - scale * g_o[b]) <= 1e-4 * np.linalg.norm(scale * g_o[b])
            assert np.all(g1[b, cfg["in_len"][b]:] == 0)


def test_noalloc_refuses_what_does_not_fit():
    import paper_1812_07625_amd as P
    B, Tp, Cc, Lmax = 32, 750, 29, 200   # the criterion benchmark shape needs about 160 MB
    assert P.w2l_ctc_workspace_bytes(B, Tp, Cc, Lmax) > 32 << 20
    z = torch.zeros((B, Tp, Cc), device="cuda:0")
    tg = torch.ones((B, Lmax), dtype=torch.int32, device="cuda:0")
    il = torch.full((B,), Tp, dtype=torch.int32, device="cuda:0")
    tl = torch.full((B,), 5, dtype=torch.int32, device="cuda:0")
    loss, grad = empty((B,)), empty((B, Tp, Cc))
    with pytest.raises(P.W2LError) as e:
        P.w2l_ctc_fwd_bwd_noalloc(z, 1, tg, il, tl, loss, grad)
    assert e.value.status == -5
    torch.cuda.synchronize()
    assert torch.isnan(loss).all() and torch.isnan(grad).all()   # nothing was launched
