"""GPU-vs-oracle parity, element by element, on identical seeded inputs, through the C ABI.

Tolerances (written here, derived from the arithmetic):
  * one kernel, bf16 output (conv forward, data gradient, GLU): the fp32 accumulator is rounded
    once, so every element obeys |got - ref| <= 1.01 * 2^-8 |ref| + 2^-12 rms(ref) (half a unit in
    the last of bf16's 8 significant bits, plus the fp32 summation error in units of the tensor's
    rms), and the relative L2 error is <= 3e-3;
  * one kernel, fp32 output (fp32 convolutions, weight and bias gradients of bf16 operands whose
    products are exact, GLU, log-softmax): every element within 1e-5 |ref| + 1e-5 rms(ref), relative
    L2 <= 1e-5 (2e-5 for reductions over more than 10^4 frames);
  * whole train steps in bf16 (roundings compound through the layers): relative L2 <= 2e-2 per
    tensor, the benchmark spec's figure, and every element within 8 x that of (|ref| + rms(ref));
  * CTC: per-utterance relative loss error <= 1e-4, gradient relative L2 <= 1e-4.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import BF16_ABS, BF16_L2, BF16_REL, DEV, assert_elementwise, empty, rel_l2, to_dev, to_host
from variant_cases import CTC_CASES, ctc_variant
from workloads.device import run_train_step

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": BF16_L2}        # one kernel: relative L2
ELEM = {"f32": (1e-5, 1e-5), "bf16": (BF16_REL, BF16_ABS)}  # one kernel: every element (relative, absolute in rms)
TOL_STEP_BF16 = 2e-2                        # a whole bf16 train step: relative L2 per tensor (the benchmark spec)
TOL_CTC = 1e-4


def check_one_kernel(got, ref, dtype, what):
    assert rel_l2(got, ref) <= TOL[dtype], what
    assert_elementwise(got, ref, *ELEM[dtype], what=what)


@pytest.fixture(scope="module")
def P():
    import paper_1812_07625_amd as P
    return P


def _grid(a, dtype):
    a = a.astype(np.float32)
    return W.round_to_bf16(a) if dtype == "bf16" else a


CONV_SHAPES = [
    # B, T, Cin, Cout, k, s
    (2, 100, 40, 128, 5, 1),
    (3, 70, 24, 72, 11, 1),      # ragged against 64-wide tiles
    (2, 131, 40, 64, 13, 2),     # strided, odd T
    (1, 37, 7, 5, 3, 3),         # odd channel counts, stride 3
    (2, 64, 64, 29, 1, 1),       # 1x1 onto the class dimension
    (4, 257, 128, 256, 11, 1),   # several tiles in every dimension, ragged tail in M
    (2, 300, 80, 192, 13, 2),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_three_passes(P, shape, dtype):
    B, T, Cin, Cout, k, s = shape
    rng = np.random.default_rng(hash(shape) % 2**31)
    Tp = oracle.out_len(T, s)
    x = _grid(rng.standard_normal((B, T, Cin)), dtype)
    w = _grid(rng.standard_normal((Cout, k, Cin)) / np.sqrt(k * Cin), dtype)
    bias = rng.standard_normal(Cout).astype(np.float32)
    dy = _grid(rng.standard_normal((B, Tp, Cout)), dtype)

    xd, wd, bd, dyd = to_dev(x, dtype), to_dev(w, dtype), to_dev(bias), to_dev(dy, dtype)
    code = P.W2L_BF16 if dtype == "bf16" else P.W2L_F32
    y_o, y0_o = oracle.conv1d_fwd(x, w, bias, s), oracle.conv1d_fwd(x, w, None, s)
    dx_o = oracle.conv1d_bwd_data(dy, w, T, s)
    # without workspace: loads predicated against the utterance edges; with the workspace the
    # query asks for: operands staged into the zero-haloed layout first
    for use_ws in (False, True):
        wf = P.workspace(P.w2l_conv1d_fwd_workspace_bytes(B, T, Cin, Cout, k, s, code)) if use_ws else None
        y = P.w2l_conv1d_fwd(xd, wd, bd, empty((B, Tp, Cout), dtype), s, wf)
        check_one_kernel(to_host(y), y_o, dtype, "y")
        y0 = P.w2l_conv1d_fwd(xd, wd, None, empty((B, Tp, Cout), dtype), s, wf)
        check_one_kernel(to_host(y0), y0_o, dtype, "y without bias")
        wb = P.workspace(P.w2l_conv1d_bwd_data_workspace_bytes(B, T, Cin, Cout, k, s, code)) if use_ws else None
        dx = P.w2l_conv1d_bwd_data(dyd, wd, empty((B, T, Cin), dtype), s, wb)
        check_one_kernel(to_host(dx), dx_o, dtype, "dx")

    ws = P.workspace(P.w2l_conv1d_bwd_weight_workspace_bytes(B, T, Cin, Cout, k, s, P.W2L_BF16 if dtype == "bf16" else 0))
    dw, db = P.w2l_conv1d_bwd_weight(xd, dyd, empty((Cout, k, Cin)), empty((Cout,)), s, False, ws)
    dw_o, db_o = oracle.conv1d_bwd_weight(x, dy, k, s)
    # fp32 outputs: with bf16 operands the products are exact on both sides, only the fp32 summation differs
    check_one_kernel(to_host(dw), dw_o, "f32", "dw")
    check_one_kernel(to_host(db), db_o, "f32", "db")
    # accumulate = 1 adds onto what is there; run twice -> bit-identical (fixed reduction order)
    dw2 = dw.clone()
    db2 = db.clone()
    P.w2l_conv1d_bwd_weight(xd, dyd, dw2, db2, s, True, ws)
    check_one_kernel(to_host(dw2), 2 * dw_o, "f32", "dw accumulated")
    check_one_kernel(to_host(db2), 2 * db_o, "f32", "db accumulated")
    dw3, db3 = P.w2l_conv1d_bwd_weight(xd, dyd, empty((Cout, k, Cin)), empty((Cout,)), s, False, ws)
    assert torch.equal(dw3, dw) and torch.equal(db3, db)


def test_conv_mixed_output_dtypes(P):
    # bf16 operands with fp32 y (logits) and fp32 dy (gradient of the logits)
    B, T, Cin, Cout, k, s = 2, 90, 64, 29, 1, 1
    rng = np.random.default_rng(77)
    x = _grid(rng.standard_normal((B, T, Cin)), "bf16")
    w = _grid(rng.standard_normal((Cout, k, Cin)) / 8, "bf16")
    dy = rng.standard_normal((B, T, Cout)).astype(np.float32)
    xd, wd, dyd = to_dev(x, "bf16"), to_dev(w, "bf16"), to_dev(dy)
    y = P.w2l_conv1d_fwd(xd, wd, None, empty((B, T, Cout)), s)
    check_one_kernel(to_host(y), oracle.conv1d_fwd(x, w, None, s), "f32", "fp32 y from bf16 operands")
    dx_o = oracle.conv1d_bwd_data(dy, w, T, s)
    dx = P.w2l_conv1d_bwd_data(dyd, wd, empty((B, T, Cin), "bf16"), s)
    check_one_kernel(to_host(dx), dx_o, "bf16", "bf16 dx from fp32 dy")
    # with workspace: dy is cast to bf16 and its 29 channels padded to 64 for the MFMA kernel -- one more rounding
    # (of dy, to 8 significant bits) than the one-kernel bound allows for: relative L2 <= 2 x 3e-3
    wb = P.workspace(P.w2l_conv1d_bwd_data_workspace_bytes(B, T, Cin, Cout, k, s, 1))
    assert wb.numel() > 256
    dx = P.w2l_conv1d_bwd_data(dyd, wd, empty((B, T, Cin), "bf16"), s, wb)
    assert rel_l2(to_host(dx), dx_o) <= 2 * BF16_L2
    assert_elementwise(to_host(dx), dx_o, 4 * BF16_REL, 16 * BF16_REL, what="bf16 dx from fp32 dy, prepared operands")
    ws = P.workspace(P.w2l_conv1d_bwd_weight_workspace_bytes(B, T, Cin, Cout, k, s, 1))
    dw, db = P.w2l_conv1d_bwd_weight(xd, dyd, empty((Cout, k, Cin)), empty((Cout,)), s, False, ws)
    dw_o, db_o = oracle.conv1d_bwd_weight(x, dy, k, s)
    check_one_kernel(to_host(dw), dw_o, "f32", "dw")
    check_one_kernel(to_host(db), db_o, "f32", "db")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,Cout", [(200, 128), (77, 1536), (33, 30), (5, 2), (1000, 2048)])
def test_glu(P, rows, Cout, dtype):
    rng = np.random.default_rng(rows + Cout)
    y = _grid(rng.standard_normal((rows, Cout)) * 2, dtype)
    dh = _grid(rng.standard_normal((rows, Cout // 2)), dtype)
    h = P.w2l_glu_fwd(to_dev(y, dtype), empty((rows, Cout // 2), dtype))
    check_one_kernel(to_host(h), oracle.glu_fwd(y), dtype, "h")
    dy = P.w2l_glu_bwd(to_dev(y, dtype), to_dev(dh, dtype), empty((rows, Cout), dtype))
    check_one_kernel(to_host(dy), oracle.glu_bwd(y, dh), dtype, "dy")


@pytest.mark.parametrize("rows,Cc", [(24000, 29), (100, 1), (37, 100), (9, 4096)])
def test_logsoftmax(P, rows, Cc):
    rng = np.random.default_rng(rows)
    z = (rng.standard_normal((rows, Cc)) * 3).astype(np.float32)
    dlp = rng.standard_normal((rows, Cc)).astype(np.float32)
    lp = P.w2l_logsoftmax_fwd(to_dev(z), empty((rows, Cc)))
    lp_o = oracle.logsoftmax_fwd(z)
    assert rel_l2(to_host(lp), lp_o) <= 1e-5 if Cc > 1 else np.all(to_host(lp) == 0)
    dz = P.w2l_logsoftmax_bwd(lp, to_dev(dlp), empty((rows, Cc)))
    ref = oracle.logsoftmax_bwd(to_host(lp), dlp)
    assert np.linalg.norm(to_host(dz) - ref) <= 1e-5 * max(np.linalg.norm(ref), 1.0)
    zb = W.round_to_bf16(z)
    lpb = P.w2l_logsoftmax_fwd(to_dev(zb, "bf16"), empty((rows, Cc)))
    assert np.linalg.norm(to_host(lpb) - oracle.logsoftmax_fwd(zb)) <= 1e-5 * max(np.linalg.norm(lp_o), 1.0)

@pytest.mark.parametrize("n,steps,wd", [(1 << 20, 3, 0.0), (4099, 5, 1e-3), (3, 2, 0.0), (26_000_001, 1, 0.0),
                                        (6545, 2, 0.0), (2051, 1, 1e-2)])
def test_sgd_momentum(P, n, steps, wd):
    """fp32 update vs the fp64 oracle (tolerance: a few fp32 roundings per step, 1e-6 relative to
    the tensor norm); the bf16 copy must be the round-to-nearest-even of the kernel's own fp32
    weights, bit for bit.  Sizes: several blocks, a ragged tail (n % 4 != 0), fewer values than
    one vector, one weight tensor of the 105M model (k=11, 768 -> 1536 plus one) at full size, and two sizes at
    which only part of the last workgroup's threads have a second group of four values."""
    rng = np.random.default_rng(n)
    w0 = rng.standard_normal(n).astype(np.float32)
    v0 = (rng.standard_normal(n) * 0.1).astype(np.float32)
    lr, mu = 0.05, 0.9
    w, v = to_dev(w0), to_dev(v0)
    lowp = empty((n,), "bf16")
    wo, vo = w0.astype(np.float64), v0.astype(np.float64)
    for s_ in range(steps):
        g = rng.standard_normal(n).astype(np.float32)
        P.w2l_sgd_momentum_step(w, v, to_dev(g), lowp, lr, mu, wd)
        wo, vo = oracle.sgd_momentum(wo, vo, g, lr, mu, wd)
    torch.cuda.synchronize()
    wg = w.cpu().numpy()
    assert rel_l2(wg, wo) <= 1e-6 and rel_l2(v.cpu().numpy(), vo) <= 1e-6
    np.testing.assert_array_equal(to_host(lowp), W.round_to_bf16(wg).astype(np.float64))
    # without the low-precision copy
    w2, v2 = to_dev(w0), to_dev(v0)
    g = rng.standard_normal(n).astype(np.float32)
    P.w2l_sgd_momentum_step(w2, v2, to_dev(g), None, lr, mu, wd)
    w2o, _ = oracle.sgd_momentum(w0.astype(np.float64), v0.astype(np.float64), g, lr, mu, wd)
    assert rel_l2(w2.cpu().numpy(), w2o) <= 1e-6


def _run_ctc(P, inp, is_logits, targets, in_len, tgt_len, blank=0, scale=1.0):
    B, Tp, Cc = inp.shape
    Lmax = targets.shape[1]
    ws = P.workspace(P.w2l_ctc_workspace_bytes(B, Tp, Cc, Lmax))
    loss, grad = P.w2l_ctc_fwd_bwd(to_dev(inp), is_logits, to_dev(targets), to_dev(in_len), to_dev(tgt_len),
                                   empty((B,)), empty((B, Tp, Cc)), blank, scale, ws)
    torch.cuda.synchronize()
    return loss.cpu().numpy().astype(np.float64), grad.cpu().numpy().astype(np.float64)


def _check_ctc(loss, grad, loss_o, grad_o):
    fin = np.isfinite(loss_o)
    assert np.array_equal(np.isfinite(loss), fin)
    assert np.all(np.abs(loss[fin] - loss_o[fin]) <= TOL_CTC * np.abs(loss_o[fin]))
    assert np.all(loss[~fin] == loss_o[~fin])
    assert np.all(np.isfinite(grad))
    for b in range(len(loss)):
        den = np.linalg.norm(grad_o[b])
        err = np.linalg.norm(grad[b] - grad_o[b])
        assert err <= TOL_CTC * den if den > 0 else err == 0, (b, err, den)


@pytest.mark.parametrize("kw", [
    dict(B=4, T=60, in_lo=40, in_hi=60, l_lo=3, l_hi=15),
    dict(B=6, T=200, in_lo=150, in_hi=200, l_lo=30, l_hi=70),     # S spans > 1 wavefront
    dict(B=3, T=97, in_lo=1, in_hi=97, l_lo=0, l_hi=1, Cc=5),
    dict(),                                                         # the full benchmark shape
    dict(B=2, T=2300, in_lo=2250, in_hi=2300, l_lo=1030, l_hi=1100),  # four pairs per lane on six wavefronts
])
def test_ctc_from_logits(P, kw):
    cfg = W.config2(seed=2, **kw)
    loss, grad = _run_ctc(P, cfg["logits"], 1, cfg["targets"], cfg["in_len"], cfg["tgt_len"], 0, 1.0)
    loss_o, _, dz_o = oracle.ctc_from_logits(cfg["logits"].astype(np.float64), cfg["targets"], cfg["in_len"],
                                             cfg["tgt_len"])
    _check_ctc(loss, grad, loss_o, dz_o)
    for b in range(cfg["B"]):
        assert np.all(grad[b, cfg["in_len"][b]:] == 0)


def _variant_id(case):
    import paper_1812_07625_amd as Pm
    return "C%d-L%d-ppt%d-nq%d-blk%d" % (case + ctc_variant(Pm, *case))


@pytest.mark.parametrize("case", CTC_CASES, ids=_variant_id)
def test_ctc_every_lattice_variant(P, case):
    """One case per variant of the alpha/beta kernel (pairs per lane x score-table depth x block
    length; the id names the variant the library's own launch query reports for the size):
    targets padded to Lmax, one utterance using all of it, one a third."""
    Cc, Lmax = case
    T = Lmax + Lmax // 8 + 40
    cfg = W.config2(seed=100 + Lmax + Cc, B=2, T=T, Cc=Cc, in_lo=T - 9, in_hi=T, l_lo=Lmax, l_hi=Lmax)
    assert cfg["targets"].shape[1] == Lmax
    cfg["tgt_len"][1] = max(1, Lmax // 3)
    loss, grad = _run_ctc(P, cfg["logits"], 1, cfg["targets"], cfg["in_len"], cfg["tgt_len"], 0, 1.0)
    loss_o, _, dz_o = oracle.ctc_from_logits(cfg["logits"].astype(np.float64), cfg["targets"], cfg["in_len"],
                                             cfg["tgt_len"])
    assert np.all(np.isfinite(loss_o))
    _check_ctc(loss, grad, loss_o, dz_o)


def test_ctc_from_logprobs_scale_blank_and_edges(P):
    rng = np.random.default_rng(9)
    B, Tp, Cc, Lmax = 7, 50, 6, 8
    z = rng.standard_normal((B, Tp, Cc)) * 1.5
    lp = oracle.logsoftmax_fwd(z).astype(np.float32)
    blank = 2
    tg = rng.integers(0, 2, size=(B, Lmax)).astype(np.int32)  # classes {0,1}: many adjacent repeats
    tg[3] = [3, 4, 5, 3, 4, 5, 3, 4]
    in_len = np.array([50, 31, 0, 8, 50, 9, 1], np.int32)
    tgt_len = np.array([8, 5, 0, 8, 0, 8, 1], np.int32)   # b=2: T=0,L=0 ; b=3: T=L ; b=5: likely infeasible
    loss, grad = _run_ctc(P, lp, 0, tg, in_len, tgt_len, blank, 0.25)
    loss_o, g_o = oracle.ctc(lp.astype(np.float64), tg, in_len, tgt_len, blank)
    assert np.isinf(loss_o[5])
    _check_ctc(loss, grad, loss_o, 0.25 * g_o)


def test_ctc_large_alphabet_gathers_scores_per_lane(P):
    # 600 classes: the class rows of a block of frames do not fit the workgroup's score table
    cfg = W.config2(seed=21, B=3, T=80, in_lo=60, in_hi=80, l_lo=5, l_hi=20, Cc=600)
    loss, grad = _run_ctc(P, cfg["logits"], 1, cfg["targets"], cfg["in_len"], cfg["tgt_len"], 0, 1.0)
    loss_o, _, dz_o = oracle.ctc_from_logits(cfg["logits"].astype(np.float64), cfg["targets"], cfg["in_len"],
                                             cfg["tgt_len"])
    _check_ctc(loss, grad, loss_o, dz_o)


def test_ctc_peaked_and_impossible_scores(P):
    # log-probabilities far outside the range of a linear fp32 recursion (about -1300 per frame), and -inf entries
    rng = np.random.default_rng(22)
    B, Tp, Cc, Lmax = 5, 300, 12, 40
    z = rng.standard_normal((B, Tp, Cc)) * 400.0
    lp = oracle.logsoftmax_fwd(z)
    tg = rng.integers(1, Cc, size=(B, Lmax)).astype(np.int32)
    in_len = np.array([300, 280, 300, 300, 150], np.int32)
    tgt_len = np.array([40, 25, 30, 10, 12], np.int32)
    lp[1, 100, 1:] = -np.inf                     # frame 100 of b=1 must be blank
    lp[2, :, tg[2, 0]] = -np.inf                 # first label of b=2 impossible: no alignment
    lp[3, 7, :] = -np.inf                        # nothing possible at frame 7 of b=3: no alignment
    lp[4, 10:20, 0] = -np.inf                    # no blank for ten frames of b=4
    lp = lp.astype(np.float32)
    loss, grad = _run_ctc(P, lp, 0, tg, in_len, tgt_len, 0, 1.0)
    loss_o, g_o = oracle.ctc(lp.astype(np.float64), tg, in_len, tgt_len, 0)
    assert np.isfinite(loss_o[[0, 1, 4]]).all() and np.isinf(loss_o[[2, 3]]).all()
    assert loss_o[0] > 30000.0                   # log2 P far below fp32's smallest exponent
    _check_ctc(loss, grad, loss_o, g_o)


def test_ctc_longest_utterance_and_lowest_scores(P):
    # 8192 frames (the size limit); utterance 0 has log-probabilities around -45000 per frame (2^-65000, just
    # above the level that counts as probability zero), so the integer exponents of its states run through
    # the whole range they are given; utterance 1 has ordinary scores over the same length
    rng = np.random.default_rng(23)
    B, Tp, Cc, Lmax = 2, 8192, 6, 30
    lp = np.empty((B, Tp, Cc), np.float32)
    lp[0] = (-45000.0 + 3.0 * rng.standard_normal((Tp, Cc))).astype(np.float32)
    lp[1] = oracle.logsoftmax_fwd(rng.standard_normal((1, Tp, Cc)) * 1.5)[0].astype(np.float32)
    tg = rng.integers(1, Cc, size=(B, Lmax)).astype(np.int32)
    in_len = np.array([8192, 8192], np.int32)
    tgt_len = np.array([30, 7], np.int32)
    loss, grad = _run_ctc(P, lp, 0, tg, in_len, tgt_len, 0, 1.0)
    loss_o, g_o = oracle.ctc(lp.astype(np.float64), tg, in_len, tgt_len, 0)
    assert np.isfinite(loss_o).all() and loss_o[0] > 3.6e8
    _check_ctc(loss, grad, loss_o, g_o)


def test_ctc_bad_label_gives_nan_loss_and_zero_grad(P):
    cfg = W.config2(seed=5, B=3, T=40, in_lo=30, in_hi=40, l_lo=3, l_hi=6)
    tg = cfg["targets"].copy()
    tg[1, 0] = 0          # blank inside a target
    loss, grad = _run_ctc(P, cfg["logits"], 1, tg, cfg["in_len"], cfg["tgt_len"])
    assert np.isnan(loss[1]) and np.all(grad[1] == 0)
    assert np.isfinite(loss[0]) and np.isfinite(loss[2]) and np.all(np.isfinite(grad))
    il = cfg["in_len"].copy()
    il[2] = 41            # longer than the padded length
    loss, grad = _run_ctc(P, cfg["logits"], 1, cfg["targets"], il, cfg["tgt_len"])
    assert np.isnan(loss[2]) and np.all(grad[2] == 0) and np.isfinite(loss[0])


def test_ctc_is_deterministic(P):
    cfg = W.config2(seed=6, B=4, T=120, in_lo=100, in_hi=120, l_lo=10, l_hi=40)
    a = _run_ctc(P, cfg["logits"], 1, cfg["targets"], cfg["in_len"], cfg["tgt_len"])
    b = _run_ctc(P, cfg["logits"], 1, cfg["targets"], cfg["in_len"], cfg["tgt_len"])
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


# ----------------------------------------------------------------------------- train step
def oracle_train_step(cfg, grad_scale=1.0):
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    return oracle.train_step(cfg["layers"], [f64(w) for w in cfg["weights"]], [f64(b) for b in cfg["biases"]],
                             f64(cfg["x"]), cfg["in_len"], cfg["targets"], cfg["tgt_len"], grad_scale,
                             cfg["blank"])


def check_step_tensor(got, ref, tol, what):
    assert rel_l2(got, ref) <= tol, what
    assert_elementwise(got, ref, 8 * tol, 8 * tol, what=what)


def check_train_step(got, ref, dtype):
    tol = 1e-4 if dtype == "f32" else TOL_STEP_BF16
    assert np.all(np.abs(got["loss"] - ref["loss"]) <= tol * np.abs(ref["loss"]))
    check_step_tensor(got["logits"], ref["logits"], tol, "logits")
    for i, (a, b) in enumerate(zip(got["dw"], ref["dw"])):
        check_step_tensor(a, b, tol, "dw of layer %d" % i)
    for i, (a, b) in enumerate(zip(got["db"], ref["db"])):
        check_step_tensor(a, b, tol, "db of layer %d" % i)


def test_train_step_tiny_fp32(P):
    cfg = W.config0()
    check_train_step(run_train_step(P, cfg), oracle_train_step(cfg), "f32")
    cfg = W.config0(seed=10, zero_bias=False)
    check_train_step(run_train_step(P, cfg, 0.5), oracle_train_step(cfg, 0.5), "f32")


def test_train_step_small_bf16_ragged(P):
    layers = [dict(k=7, stride=2, cin=40, cout=96, glu=1), dict(k=5, stride=1, cin=48, cout=128, glu=1),
              dict(k=3, stride=1, cin=64, cout=80, glu=1), dict(k=1, stride=1, cin=40, cout=29, glu=0)]
    cfg = W.small_model(21, 5, 90, 171, 40, layers, True, 4, 20)
    check_train_step(run_train_step(P, cfg), oracle_train_step(cfg), "bf16")


def test_train_step_10m_model_reduced_batch(P):
    # the ~10M-parameter bf16 configuration with the batch cut to 4 so the fp64 oracle takes seconds
    cfg = W.config3(B=4)
    check_train_step(run_train_step(P, cfg), oracle_train_step(cfg), "bf16")

def test_train_step_wide_layer_fused_epilogues(P):
    """A model whose second layer has the benchmark's output shape (B*T' = 6000 frames, 1536
    channels) but a short reduction, so that the fp64 oracle stays affordable: the train step then
    takes the kernels the 105M model takes -- forward convolution with the GLU in its epilogue
    (layer 1), data gradient with its reduction split over two workgroups per tile and the GLU
    backward of the layer below in the combining pass (layer 2 writes dy of layer 1), data gradient
    with the GLU backward in its own epilogue (layer 1 writes dy of layer 0), activation slabs,
    256x256 weight-gradient tiles -- and every gradient is compared with the oracle."""
    layers = [dict(k=3, stride=1, cin=16, cout=128, glu=1), dict(k=3, stride=1, cin=64, cout=1536, glu=1),
              dict(k=5, stride=1, cin=768, cout=256, glu=1), dict(k=1, stride=1, cin=128, cout=29, glu=0)]
    cfg = W.small_model(33, 8, 700, 750, 16, layers, True, 20, 60)
    check_train_step(run_train_step(P, cfg), oracle_train_step(cfg), "bf16")


@pytest.mark.parametrize("bf16", [False, True])
def test_train_step_layers_without_glu(P, bf16):
    """Layers without a GLU in the middle of the network -- one between GLU layers, two in a row, a
    strided one first: the output of such a layer feeds the next convolution directly and its dh is
    its dy, so the data gradients must not overwrite a buffer that a weight gradient still reads."""
    layers = [dict(k=5, stride=2, cin=40, cout=64, glu=0), dict(k=3, stride=1, cin=64, cout=96, glu=1),
              dict(k=3, stride=1, cin=48, cout=48, glu=0), dict(k=5, stride=1, cin=48, cout=40, glu=0),
              dict(k=3, stride=1, cin=40, cout=64, glu=1), dict(k=1, stride=1, cin=32, cout=29, glu=0)]
    cfg = W.small_model(41, 4, 150, 233, 40, layers, bf16, 5, 30)
    check_train_step(run_train_step(P, cfg), oracle_train_step(cfg), "bf16" if bf16 else "f32")
    a, b = run_train_step(P, cfg), run_train_step(P, cfg)
    for u, v in zip(a["dw"] + a["db"], b["dw"] + b["db"]):
        assert np.array_equal(u, v)


def test_train_step_two_narrow_layers(P):
    """Both weight gradients take the narrow-output kernel and its scratch: layer 1's on the helper
    stream, layer 0's on the caller's stream at the same time -- each in its own scratch."""
    layers = [dict(k=3, stride=1, cin=40, cout=32, glu=1), dict(k=1, stride=1, cin=16, cout=29, glu=0)]
    cfg = W.small_model(42, 6, 300, 400, 40, layers, True, 5, 40)
    ref = oracle_train_step(cfg)
    for _ in range(3):
        check_train_step(run_train_step(P, cfg), ref, "bf16")


def test_train_step_is_deterministic(P):
    cfg = W.config0(seed=3)
    a, b = run_train_step(P, cfg), run_train_step(P, cfg)
    assert np.array_equal(a["loss"], b["loss"])
    for u, v in zip(a["dw"] + a["db"], b["dw"] + b["db"]):
        assert np.array_equal(u, v)


# ----------------------------------------------------------------------------- full benchmark sizes
FULL_SHAPES = [
    # name, B, T, Cin, Cout, k, s   (launch configurations that bench.py times)
    ("config1", 16, 800, 512, 1024, 11, 1),
    ("config4-body", 8, 750, 768, 1536, 11, 1),
    ("config4-first", 8, 1500, 80, 1536, 13, 2),
    ("config4-1x1", 8, 750, 768, 2048, 1, 1),
    ("config3-body", 16, 800, 256, 512, 11, 1),
]


def _boundary_indices(rng, rows, cols, row_marks, n_random=3000, n_rand_cols=16):
    """Flat indices into a [rows, cols] tensor: every row in `row_marks` and every row next to a
    multiple of 32 (the edge of an MFMA block, of a wavefront's sub-tile and of a workgroup tile of
    any of the kernels' sizes), at the columns next to a multiple of 32, the last 40 columns and a
    few random ones; four complete rows and four complete columns; and a uniform random sample."""
    r = np.arange(rows)
    rsel = np.unique(np.concatenate([r[(r % 32 == 0) | (r % 32 == 31)], np.asarray(row_marks, dtype=np.int64),
                                     r[-70:]]))
    rsel = rsel[(rsel >= 0) & (rsel < rows)]
    c = np.arange(cols)
    csel = np.unique(np.concatenate([c[(c % 32 == 0) | (c % 32 == 31)], c[-40:], rng.integers(0, cols, n_rand_cols)]))
    grid = (rsel[:, None] * cols + csel[None, :]).ravel()
    full_r = rng.integers(0, rows, 4)
    full_c = rng.integers(0, cols, 4)
    lines = np.concatenate([(fr * cols + c) for fr in full_r] + [(r * cols + fc) for fc in full_c])
    return np.unique(np.concatenate([grid, lines, rng.integers(0, rows * cols, n_random)]))


def _frame_marks(B, frames):
    """Rows (b * frames + t) whose position in the zero-haloed layout the kernels tile over
    (LAYOUT_HALO = 8 frames around every utterance) is next to a multiple of 32, plus the first
    and last two frames of every utterance (windows that reach into the padding)."""
    halo = 8
    marks = []
    for b in range(B):
        t = np.arange(frames)
        f = b * (frames + 2 * halo) + t          # layout frame counted from utterance 0's first real frame
        marks.append(b * frames + t[(f % 32 == 0) | (f % 32 == 31)])
        marks.append(b * frames + np.array([0, 1, frames - 2, frames - 1]))
    return np.concatenate(marks)


@pytest.mark.parametrize("shape", FULL_SHAPES, ids=[s[0] for s in FULL_SHAPES])
def test_conv_full_size_sampled(P, shape):
    """bf16 operands at the benchmark shapes, in the launch configuration bench.py times (operands
    staged through the workspace).  A full fp64 pass at these sizes takes minutes, so the oracle
    evaluates outputs one by one: every tile, sub-tile and utterance boundary (rows and columns
    next to multiples of 32 in the dense and in the haloed frame numbering, the ragged last tile),
    whole rows and columns, and a uniform random sample -- each held to the one-kernel bounds."""
    name, B, T, Cin, Cout, k, s = shape
    rng = np.random.default_rng(len(name) * 1000 + B)
    Tp = oracle.out_len(T, s)
    x = W.round_to_bf16(rng.standard_normal((B, T, Cin)).astype(np.float32))
    w = W.round_to_bf16((rng.standard_normal((Cout, k, Cin)) / np.sqrt(k * Cin)).astype(np.float32))
    dy = W.round_to_bf16(rng.standard_normal((B, Tp, Cout)).astype(np.float32))
    bias = rng.standard_normal(Cout).astype(np.float32)
    xd, wd, dyd, bd = to_dev(x, "bf16"), to_dev(w, "bf16"), to_dev(dy, "bf16"), to_dev(bias)

    wf = P.workspace(P.w2l_conv1d_fwd_workspace_bytes(B, T, Cin, Cout, k, s, P.W2L_BF16))
    y = to_host(P.w2l_conv1d_fwd(xd, wd, bd, empty((B, Tp, Cout), "bf16"), s, wf)).reshape(-1)
    idx = _boundary_indices(rng, B * Tp, Cout, _frame_marks(B, Tp))
    ref = oracle.conv1d_fwd_at(x, w, bias, idx, s)
    check_one_kernel(y[idx], ref, "bf16", "y")
    if name == "config4-body":
        # the same kernel family with fp32 output (how a last layer writes logits): no output rounding
        y32 = to_host(P.w2l_conv1d_fwd(xd, wd, bd, empty((B, Tp, Cout)), s, wf)).reshape(-1)
        check_one_kernel(y32[idx], ref, "f32", "fp32 y")

    wb = P.workspace(P.w2l_conv1d_bwd_data_workspace_bytes(B, T, Cin, Cout, k, s, P.W2L_BF16))
    dx = to_host(P.w2l_conv1d_bwd_data(dyd, wd, empty((B, T, Cin), "bf16"), s, wb)).reshape(-1)
    idx = _boundary_indices(rng, B * T, Cin, _frame_marks(B, T))
    ref = oracle.conv1d_bwd_data_at(dy, w, T, idx, s)
    check_one_kernel(dx[idx], ref, "bf16", "dx")

    ws = P.workspace(P.w2l_conv1d_bwd_weight_workspace_bytes(B, T, Cin, Cout, k, s, P.W2L_BF16))
    dw, db = P.w2l_conv1d_bwd_weight(xd, dyd, empty((Cout, k, Cin)), empty((Cout,)), s, False, ws)
    dw = to_host(dw).reshape(-1)
    idx = _boundary_indices(rng, Cout, k * Cin, [0, Cout - 1])
    ref = oracle.conv1d_bwd_weight_at(x, dy, k, idx, s)
    # fp32 sums of exact products over B*T' = 6000..12800 frames
    assert rel_l2(dw[idx], ref) <= 2e-5
    assert_elementwise(dw[idx], ref, 2e-5, 2e-5, what="dw")
    db_o = dy.astype(np.float64).sum((0, 1))
    assert rel_l2(to_host(db), db_o) <= 2e-5
    assert_elementwise(to_host(db), db_o, 2e-5, 2e-5, what="db")


def _replicated(cfg, picks, times):
    """A batch made of the utterances `picks` of cfg, the group repeated `times` times."""
    sel = list(picks) * times
    out = dict(cfg)
    for key in ("x", "in_len", "targets", "tgt_len"):
        out[key] = np.ascontiguousarray(cfg[key][sel])
    out["B"] = len(sel)
    return out


def _check_replicated_step(P, cfg, picks, times):
    """The GPU step on the replicated batch (the benchmark's launch shapes) against the oracle's
    step on the distinct utterances alone: losses and logits repeat, every dw/db is `times` x the
    oracle's sum over the distinct utterances."""
    rep = _replicated(cfg, picks, times)
    got = run_train_step(P, rep)
    ref = oracle_train_step(_replicated(cfg, picks, 1))
    n = len(picks)
    tol = TOL_STEP_BF16
    for r in range(times):
        sl = slice(r * n, (r + 1) * n)
        assert np.all(np.abs(got["loss"][sl] - ref["loss"]) <= tol * np.abs(ref["loss"]))
        check_step_tensor(got["logits"][sl], ref["logits"], tol, "logits of copy %d" % r)
    for i, (a, b) in enumerate(zip(got["dw"], ref["dw"])):
        check_step_tensor(a, times * b, tol, "dw of layer %d" % i)
    for i, (a, b) in enumerate(zip(got["db"], ref["db"])):
        check_step_tensor(a, times * b, tol, "db of layer %d" % i)
    return got, ref


def test_train_step_105m_all_gradients(P):
    """The benchmark configuration itself (B=8, T=1500, 11 layers, 107M parameters): forward,
    criterion and every weight and bias gradient against the fp64 oracle.  The batch is two of the
    configuration's utterances (the longest and the shortest), four times over, so that the GPU runs
    the benchmark's launch shapes (M = 6000 frames per layer) while the oracle needs only the two
    distinct utterances (about a minute on 16 cores; the whole batch would take four)."""
    cfg = W.config4()
    order = np.argsort(cfg["in_len"])
    _check_replicated_step(P, cfg, [int(order[-1]), int(order[0])], 4)


def test_train_step_10m_full_batch(P):
    """The ~10M-parameter configuration at its full batch of 16 (four utterances, four times over)."""
    cfg = W.config3()
    order = np.argsort(cfg["in_len"])
    _check_replicated_step(P, cfg, [int(order[-1]), int(order[5]), int(order[10]), int(order[0])], 4)
