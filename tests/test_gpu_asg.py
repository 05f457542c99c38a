"""GPU-vs-oracle parity of the ASG criterion (w2l_asg_fwd_bwd), through the C ABI, on identical
seeded inputs.

Tolerances (fp32 kernels against the fp64 oracle):
  * loss: |error| <= 1e-4 * |loss| + 1e-6 * |FCC|  (the loss is the difference of two log-sums
    of that size, each carried as fp32 states relative to a double offset)
  * gradients (emissions per utterance, transitions): L2 error <= 1e-4 * |gradient| + 1e-6 * sqrt(frames)
    (a gradient is the difference of two occupancy fields whose rows each sum to 1 and carry
    fp32 rounding of that size; where the two cancel -- a single class, a target that leaves no
    choice -- only the absolute term is left)
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import empty, to_dev, to_host
from variant_cases import ASG_CASES, asg_variant

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.fixture(scope="module")
def P():
    import paper_1812_07625_amd as P
    return P


def run_asg(P, em, trans, targets, in_len, tgt_len, grad_scale=1.0, want_trans=True):
    B, Tp, C = em.shape
    Lmax = targets.shape[1]
    ed, td = to_dev(em.astype(np.float32)), to_dev(trans.astype(np.float32))
    tg, il, tl = to_dev(targets.astype(np.int32)), to_dev(np.asarray(in_len, np.int32)), to_dev(np.asarray(tgt_len, np.int32))
    loss, ge = empty((B,)), empty((B, Tp, C))
    gt = empty((C, C)) if want_trans else None
    for t in (loss, ge) + ((gt,) if want_trans else ()):
        t.fill_(float("nan"))        # every output element must be written
    ws = P.workspace(P.w2l_asg_workspace_bytes(B, Tp, C, Lmax))
    P.w2l_asg_fwd_bwd(ed, td, tg, il, tl, loss, ge, gt, grad_scale, ws)
    torch.cuda.synchronize()
    return to_host(loss), to_host(ge), to_host(gt) if want_trans else None


def check_asg(got, em, trans, targets, in_len, tgt_len, grad_scale=1.0):
    loss, ge, gt = got
    lo, geo, gto, fcc, _ = oracle.asg(em.astype(np.float64), trans.astype(np.float64), targets, in_len, tgt_len,
                                      grad_scale, want_terms=True)
    fin = np.isfinite(lo)
    assert np.array_equal(np.isfinite(loss), fin)
    assert np.all(loss[~fin] == lo[~fin])
    assert np.all(np.abs(loss[fin] - lo[fin]) <= TOL * np.abs(lo[fin]) + 1e-6 * np.abs(fcc[fin]))
    assert np.all(np.isfinite(ge))
    for b in range(len(loss)):
        den, err = np.linalg.norm(geo[b]), np.linalg.norm(ge[b] - geo[b])
        assert err <= TOL * den + 1e-6 * abs(grad_scale) * np.sqrt(max(int(in_len[b]), 0)) if fin[b] else err == 0, (b, err, den)
        assert np.all(ge[b, max(int(in_len[b]), 0):] == 0)
    if gt is not None:
        den, err = np.linalg.norm(gto), np.linalg.norm(gt - gto)
        frames = float(np.sum(np.maximum(np.asarray(in_len)[fin], 0)))
        assert err <= TOL * den + 1e-6 * abs(grad_scale) * np.sqrt(frames), (err, den)


@pytest.mark.parametrize("kw", [
    dict(B=4, T=60, in_lo=40, in_hi=60, l_lo=3, l_hi=15),
    dict(B=6, T=200, in_lo=150, in_hi=200, l_lo=30, l_hi=120),           # positions span several wavefronts
    dict(B=3, T=97, in_lo=1, in_hi=97, l_lo=1, l_hi=2, Cc=5),
    dict(B=5, T=130, in_lo=100, in_hi=130, l_lo=20, l_hi=60, Cc=40, allow_repeats=True),  # more than 32 classes
    dict(B=3, T=90, in_lo=70, in_hi=90, l_lo=5, l_hi=30, Cc=64),          # the class limit
    dict(B=2, T=300, in_lo=280, in_hi=300, l_lo=210, l_hi=250, Cc=40, allow_repeats=True),  # > 32 classes, two positions per lane
    dict(B=2, T=50, in_lo=30, in_hi=50, l_lo=1, l_hi=9, Cc=1),            # a single class: loss = log(#alignments)
    dict(),                                                                 # the full benchmark shape
])
def test_asg_matches_oracle(P, kw):
    cfg = W.asg_batch(seed=12, **kw)
    got = run_asg(P, cfg["emissions"], cfg["trans"], cfg["targets"], cfg["in_len"], cfg["tgt_len"])
    check_asg(got, cfg["emissions"], cfg["trans"], cfg["targets"], cfg["in_len"], cfg["tgt_len"])


def _variant_id(case):
    import paper_1812_07625_amd as Pm
    return "C%d-L%d-ppt%d-lanes%d-maxt%d-blk%d-nq%d" % (case + asg_variant(Pm, *case))


@pytest.mark.parametrize("case", ASG_CASES, ids=_variant_id)
def test_asg_every_lattice_variant(P, case):
    """One case per variant of the lattice kernel (positions per lane x class lanes x workgroup
    bound x block length x staged values; the id names the variant the library's own launch query
    reports for the size): targets padded to Lmax, one utterance using all of it, one a third."""
    Cc, Lmax = case
    T = Lmax + 40
    cfg = W.asg_batch(seed=200 + Lmax + Cc, B=2, T=T, Cc=Cc, in_lo=T - 9, in_hi=T, l_lo=Lmax, l_hi=Lmax)
    assert cfg["targets"].shape[1] == Lmax
    cfg["tgt_len"][1] = max(1, Lmax // 3)
    got = run_asg(P, cfg["emissions"], cfg["trans"], cfg["targets"], cfg["in_len"], cfg["tgt_len"])
    check_asg(got, cfg["emissions"], cfg["trans"], cfg["targets"], cfg["in_len"], cfg["tgt_len"])


def test_asg_scale_edges_and_missing_trans_gradient(P):
    rng = np.random.default_rng(19)
    B, Tp, C, Lmax = 8, 50, 6, 8
    em = (rng.standard_normal((B, Tp, C)) * 3.0).astype(np.float32)
    trans = rng.standard_normal((C, C)).astype(np.float32)
    tg = rng.integers(0, 2, size=(B, Lmax)).astype(np.int32)  # classes {0,1}: many equal neighbours
    tg[3] = [3, 4, 5, 3, 4, 5, 3, 4]
    in_len = np.array([50, 31, 0, 8, 50, 7, 1, 0], np.int32)
    tgt_len = np.array([8, 5, 0, 8, 0, 8, 1, 3], np.int32)
    # b=2: no frames, no labels (loss 0); b=3: T = L (one alignment); b=4: frames but no labels,
    # b=5: more labels than frames, b=7: labels but no frames (all three: no alignment)
    got = run_asg(P, em, trans, tg, in_len, tgt_len, 0.25)
    assert np.isposinf(got[0][4]) and np.isposinf(got[0][5]) and np.isposinf(got[0][7]) and got[0][2] == 0
    check_asg(got, em, trans, tg, in_len, tgt_len, 0.25)
    got2 = run_asg(P, em, trans, tg, in_len, tgt_len, 0.25, want_trans=False)
    assert np.array_equal(got2[0], got[0]) and np.array_equal(got2[1], got[1])


def test_asg_wide_score_ranges(P):
    """Transition scores hundreds of nats apart (edges that are all but forbidden, some of which
    the target has to take) and emissions with large margins: every term goes through the log
    domain, so nothing may underflow to "impossible"."""
    rng = np.random.default_rng(23)
    B, Tp, C, Lmax = 4, 80, 7, 20
    em = (rng.standard_normal((B, Tp, C)) * 25.0).astype(np.float32)
    trans = (rng.standard_normal((C, C)) * 2.0).astype(np.float32)
    trans[rng.random((C, C)) < 0.4] -= 300.0
    trans[2, :] -= 150.0                                    # a class that is expensive to enter from anywhere
    tg = rng.integers(0, C, size=(B, Lmax)).astype(np.int32)
    in_len = np.array([80, 64, 33, 80], np.int32)
    tgt_len = np.array([20, 11, 20, 1], np.int32)
    got = run_asg(P, em, trans, tg, in_len, tgt_len)
    check_asg(got, em, trans, tg, in_len, tgt_len)


def test_asg_bad_label_gives_nan_loss_and_zero_grad(P):
    cfg = W.asg_batch(seed=5, B=3, T=40, in_lo=30, in_hi=40, l_lo=3, l_hi=6)
    tg = cfg["targets"].copy()
    tg[1, 0] = cfg["C"]     # outside [0, C)
    loss, ge, gt = run_asg(P, cfg["emissions"], cfg["trans"], tg, cfg["in_len"], cfg["tgt_len"])
    assert np.isnan(loss[1]) and np.all(ge[1] == 0)
    assert np.isfinite(loss[0]) and np.isfinite(loss[2]) and np.all(np.isfinite(ge)) and np.all(np.isfinite(gt))
    # the other utterances are unaffected, and the transition gradient is theirs alone
    keep = [0, 2]
    lo, geo, gto = oracle.asg(cfg["emissions"][keep].astype(np.float64), cfg["trans"].astype(np.float64),
                              cfg["targets"][keep], cfg["in_len"][keep], cfg["tgt_len"][keep])
    assert np.linalg.norm(gt - gto) <= TOL * np.linalg.norm(gto)
    il = cfg["in_len"].copy()
    il[2] = 41              # longer than the padded length
    loss, ge, gt = run_asg(P, cfg["emissions"], cfg["trans"], cfg["targets"], il, cfg["tgt_len"])
    assert np.isnan(loss[2]) and np.all(ge[2] == 0) and np.isfinite(loss[0])
    assert P.w2l_asg_check_targets_host(tg, cfg["in_len"], cfg["tgt_len"], cfg["T"], cfg["C"]) != 0
    assert P.w2l_asg_check_targets_host(cfg["targets"], cfg["in_len"], cfg["tgt_len"], cfg["T"], cfg["C"]) == 0


def test_asg_is_deterministic(P):
    cfg = W.asg_batch(seed=6, B=4, T=120, in_lo=100, in_hi=120, l_lo=10, l_hi=80)
    a = run_asg(P, cfg["emissions"], cfg["trans"], cfg["targets"], cfg["in_len"], cfg["tgt_len"])
    b = run_asg(P, cfg["emissions"], cfg["trans"], cfg["targets"], cfg["in_len"], cfg["tgt_len"])
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_train_step_with_asg_criterion(P):
    """w2l_train_step_asg: the network of the bf16 parity case with its output taken as ASG
    emissions (28 classes) -- loss, every weight / bias gradient and the transition gradient
    against the oracle's train step with the same criterion."""
    from gpu_util import rel_l2
    layers = [dict(k=7, stride=2, cin=40, cout=96, glu=1), dict(k=5, stride=1, cin=48, cout=128, glu=1),
              dict(k=3, stride=1, cin=64, cout=80, glu=1), dict(k=1, stride=1, cin=40, cout=28, glu=0)]
    cfg = W.small_model(31, 5, 90, 171, 40, layers, True, 4, 20)
    rng = np.random.default_rng(32)
    trans = (rng.standard_normal((28, 28)) * 0.5).astype(np.float32)
    targets = (cfg["targets"] % 28).astype(np.int32)            # labels 0..27, no blank
    B, T = cfg["B"], cfg["T"]
    xd = to_dev(cfg["x"], "bf16")
    wd = [to_dev(w, "bf16") for w in cfg["weights"]]
    bd = [to_dev(b) for b in cfg["biases"]]
    dwd = [empty(w.shape) for w in cfg["weights"]]
    dbd = [empty(b.shape) for b in cfg["biases"]]
    tg, il, tl, td = to_dev(targets), to_dev(cfg["in_len"]), to_dev(cfg["tgt_len"]), to_dev(trans)
    dtd, loss = empty((28, 28)), empty((B,))
    Lmax = targets.shape[1]
    ws = P.workspace(P.w2l_train_step_asg_workspace_bytes(layers, B, T, Lmax, P.W2L_BF16))
    Tl = oracle.out_len(T, 2)
    logits = empty((B, Tl, 28))
    P.w2l_train_step_asg(layers, wd, bd, dwd, dbd, xd, il, tg, tl, td, dtd, loss, logits, 0.5, ws)
    torch.cuda.synchronize()
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    ref = oracle.train_step(layers, [f64(w) for w in cfg["weights"]], [f64(b) for b in cfg["biases"]], f64(cfg["x"]),
                            cfg["in_len"], targets, cfg["tgt_len"], 0.5, trans=f64(trans))
    tol = 2e-2                                                   # bf16 activations between the layers
    assert rel_l2(to_host(logits), ref["logits"]) <= tol
    assert np.all(np.abs(to_host(loss) - ref["loss"]) <= tol * np.abs(ref["loss"]))
    for i, (a, b) in enumerate(zip(dwd, ref["dw"])):
        assert rel_l2(to_host(a), b) <= tol, "dw of layer %d" % i
    for i, (a, b) in enumerate(zip(dbd, ref["db"])):
        assert rel_l2(to_host(a), b) <= tol, "db of layer %d" % i
    assert rel_l2(to_host(dtd), ref["dtrans"]) <= tol
    # a class count the criterion does not take is reported, not run
    big = [dict(k=1, stride=1, cin=40, cout=80, glu=0)]
    assert P.w2l_train_step_asg_workspace_bytes(big, 2, 50, 5, P.W2L_F32) == 0
