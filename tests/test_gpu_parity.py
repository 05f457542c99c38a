"""GPU-vs-oracle parity, element by element, on identical seeded inputs, through the C ABI.

Tolerances (written here, derived from the arithmetic):
  * bf16 tensors (conv outputs and gradients): relative L2 error <= 2e-2
  * fp32 conv / GLU / log-softmax: relative L2 error <= 1e-5
  * CTC: per-utterance relative loss error <= 1e-4, gradient relative L2 <= 1e-4
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from gpu_util import DEV, empty, rel_l2, to_dev, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
TOL_CTC = 1e-4


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
        assert rel_l2(to_host(y), y_o) <= TOL[dtype]
        y0 = P.w2l_conv1d_fwd(xd, wd, None, empty((B, Tp, Cout), dtype), s, wf)
        assert rel_l2(to_host(y0), y0_o) <= TOL[dtype]
        wb = P.workspace(P.w2l_conv1d_bwd_data_workspace_bytes(B, T, Cin, Cout, k, s, code)) if use_ws else None
        dx = P.w2l_conv1d_bwd_data(dyd, wd, empty((B, T, Cin), dtype), s, wb)
        assert rel_l2(to_host(dx), dx_o) <= TOL[dtype]

    ws = P.workspace(P.w2l_conv1d_bwd_weight_workspace_bytes(B, T, Cin, Cout, k, s, P.W2L_BF16 if dtype == "bf16" else 0))
    dw, db = P.w2l_conv1d_bwd_weight(xd, dyd, empty((Cout, k, Cin)), empty((Cout,)), s, False, ws)
    dw_o, db_o = oracle.conv1d_bwd_weight(x, dy, k, s)
    tol_w = 1e-5 if dtype == "f32" else 1e-4  # operands are exact on both sides; only the fp32 summation differs
    assert rel_l2(to_host(dw), dw_o) <= tol_w
    assert rel_l2(to_host(db), db_o) <= tol_w
    # accumulate = 1 adds onto what is there; run twice -> bit-identical (fixed reduction order)
    dw2 = dw.clone()
    db2 = db.clone()
    P.w2l_conv1d_bwd_weight(xd, dyd, dw2, db2, s, True, ws)
    assert rel_l2(to_host(dw2), 2 * dw_o) <= tol_w
    assert rel_l2(to_host(db2), 2 * db_o) <= tol_w
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
    assert rel_l2(to_host(y), oracle.conv1d_fwd(x, w, None, s)) <= 1e-5
    dx = P.w2l_conv1d_bwd_data(dyd, wd, empty((B, T, Cin), "bf16"), s)
    assert rel_l2(to_host(dx), oracle.conv1d_bwd_data(dy, w, T, s)) <= TOL["bf16"]
    ws = P.workspace(P.w2l_conv1d_bwd_weight_workspace_bytes(B, T, Cin, Cout, k, s, 1))
    dw, db = P.w2l_conv1d_bwd_weight(xd, dyd, empty((Cout, k, Cin)), empty((Cout,)), s, False, ws)
    dw_o, db_o = oracle.conv1d_bwd_weight(x, dy, k, s)
    assert rel_l2(to_host(dw), dw_o) <= 1e-5 and rel_l2(to_host(db), db_o) <= 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,Cout", [(200, 128), (77, 1536), (33, 30), (5, 2), (1000, 2048)])
def test_glu(P, rows, Cout, dtype):
    rng = np.random.default_rng(rows + Cout)
    y = _grid(rng.standard_normal((rows, Cout)) * 2, dtype)
    dh = _grid(rng.standard_normal((rows, Cout // 2)), dtype)
    h = P.w2l_glu_fwd(to_dev(y, dtype), empty((rows, Cout // 2), dtype))
    tol = 1e-5 if dtype == "f32" else 4e-3   # one bf16 rounding of the result: <= 2^-9 per element
    assert rel_l2(to_host(h), oracle.glu_fwd(y)) <= tol
    dy = P.w2l_glu_bwd(to_dev(y, dtype), to_dev(dh, dtype), empty((rows, Cout), dtype))
    assert rel_l2(to_host(dy), oracle.glu_bwd(y, dh)) <= tol


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

@pytest.mark.parametrize("n,steps,wd", [(1 << 20, 3, 0.0), (4099, 5, 1e-3), (3, 2, 0.0), (26_000_001, 1, 0.0)])
def test_sgd_momentum(P, n, steps, wd):
    """fp32 update vs the fp64 oracle (tolerance: a few fp32 roundings per step, 1e-6 relative to
    the tensor norm); the bf16 copy must be the round-to-nearest-even of the kernel's own fp32
    weights, bit for bit.  Sizes: several blocks, a ragged tail (n % 4 != 0), fewer values than
    one vector, and one weight tensor of the 105M model (k=11, 768 -> 1536 plus one) at full size."""
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
    dict(B=2, T=700, in_lo=650, in_hi=700, l_lo=250, l_hi=300),       # two pairs per lane, blocks of 16 frames
    dict(B=2, T=900, in_lo=860, in_hi=900, l_lo=390, l_hi=440),       # two pairs per lane, blocks of 8 frames
    dict(B=2, T=1300, in_lo=1250, in_hi=1300, l_lo=550, l_hi=600),    # four pairs per lane, blocks of 16
    dict(B=2, T=1800, in_lo=1750, in_hi=1800, l_lo=800, l_hi=850),    # four pairs per lane, blocks of 8
])
def test_ctc_from_logits(P, kw):
    cfg = W.config2(seed=2, **kw)
    loss, grad = _run_ctc(P, cfg["logits"], 1, cfg["targets"], cfg["in_len"], cfg["tgt_len"], 0, 1.0)
    loss_o, _, dz_o = oracle.ctc_from_logits(cfg["logits"].astype(np.float64), cfg["targets"], cfg["in_len"],
                                             cfg["tgt_len"])
    _check_ctc(loss, grad, loss_o, dz_o)
    for b in range(cfg["B"]):
        assert np.all(grad[b, cfg["in_len"][b]:] == 0)


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
def run_train_step(P, cfg, grad_scale=1.0, want_logits=True):
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
        Tl = oracle.out_len(Tl, L["stride"])
    logits = empty((B, Tl, layers[-1]["cout"])) if want_logits else None
    P.w2l_train_step(layers, wd, bd, dwd, dbd, xd, il, tg, tl, loss, logits, cfg["blank"], grad_scale, ws)
    torch.cuda.synchronize()
    return dict(loss=to_host(loss), logits=to_host(logits) if want_logits else None,
                dw=[to_host(t) for t in dwd], db=[to_host(t) for t in dbd])


def oracle_train_step(cfg, grad_scale=1.0):
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    return oracle.train_step(cfg["layers"], [f64(w) for w in cfg["weights"]], [f64(b) for b in cfg["biases"]],
                             f64(cfg["x"]), cfg["in_len"], cfg["targets"], cfg["tgt_len"], grad_scale,
                             cfg["blank"])


def check_train_step(got, ref, dtype):
    tol = 1e-4 if dtype == "f32" else 2e-2
    assert np.all(np.abs(got["loss"] - ref["loss"]) <= (1e-4 if dtype == "f32" else 2e-2) * np.abs(ref["loss"]))
    assert rel_l2(got["logits"], ref["logits"]) <= tol
    for i, (a, b) in enumerate(zip(got["dw"], ref["dw"])):
        assert rel_l2(a, b) <= tol, "dw of layer %d" % i
    for i, (a, b) in enumerate(zip(got["db"], ref["db"])):
        assert rel_l2(a, b) <= tol, "db of layer %d" % i


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


@pytest.mark.parametrize("shape", FULL_SHAPES, ids=[s[0] for s in FULL_SHAPES])
def test_conv_full_size_sampled(P, shape):
    """bf16 operands at the benchmark shapes; the oracle evaluates a random sample of outputs
    one by one (a full fp64 pass at these sizes takes minutes)."""
    name, B, T, Cin, Cout, k, s = shape
    rng = np.random.default_rng(abs(hash(name)) % 2**31 if False else len(name) * 1000 + B)
    Tp = oracle.out_len(T, s)
    x = W.round_to_bf16(rng.standard_normal((B, T, Cin)).astype(np.float32))
    w = W.round_to_bf16((rng.standard_normal((Cout, k, Cin)) / np.sqrt(k * Cin)).astype(np.float32))
    dy = W.round_to_bf16(rng.standard_normal((B, Tp, Cout)).astype(np.float32))
    bias = rng.standard_normal(Cout).astype(np.float32)
    xd, wd, dyd, bd = to_dev(x, "bf16"), to_dev(w, "bf16"), to_dev(dy, "bf16"), to_dev(bias)
    nsamp = 3000

    def sample(n_total, edge_rows=None):
        idx = rng.integers(0, n_total, size=nsamp)
        return np.unique(idx)

    wf = P.workspace(P.w2l_conv1d_fwd_workspace_bytes(B, T, Cin, Cout, k, s, P.W2L_BF16))
    y = to_host(P.w2l_conv1d_fwd(xd, wd, bd, empty((B, Tp, Cout), "bf16"), s, wf)).reshape(-1)
    idx = sample(y.size)
    # always include the corners of every utterance (zero-padded windows) and the last tile
    corners = []
    for b in range(B):
        for tp in (0, 1, Tp - 2, Tp - 1):
            for co in (0, Cout - 1):
                corners.append((b * Tp + tp) * Cout + co)
    idx = np.unique(np.concatenate([idx, np.array(corners)]))
    ref = oracle.conv1d_fwd_at(x, w, bias, idx, s)
    assert rel_l2(y[idx], ref) <= TOL["bf16"]
    if name == "config4-body":
        # the same kernel family with fp32 output (how a last layer writes logits): no output rounding
        y32 = to_host(P.w2l_conv1d_fwd(xd, wd, bd, empty((B, Tp, Cout)), s, wf)).reshape(-1)
        assert rel_l2(y32[idx], ref) <= 2e-5  # fp32 accumulation over k*Cin = 8448 products

    if s == 1:
        wb = P.workspace(P.w2l_conv1d_bwd_data_workspace_bytes(B, T, Cin, Cout, k, s, P.W2L_BF16))
        dx = to_host(P.w2l_conv1d_bwd_data(dyd, wd, empty((B, T, Cin), "bf16"), s, wb)).reshape(-1)
        idx = sample(dx.size)
        corners = [(b * T + t) * Cin + c for b in range(B) for t in (0, 1, T - 2, T - 1) for c in (0, Cin - 1)]
        idx = np.unique(np.concatenate([idx, np.array(corners)]))
        ref = oracle.conv1d_bwd_data_at(dy, w, T, idx, s)
        assert rel_l2(dx[idx], ref) <= TOL["bf16"]

    ws = P.workspace(P.w2l_conv1d_bwd_weight_workspace_bytes(B, T, Cin, Cout, k, s, P.W2L_BF16))
    dw, db = P.w2l_conv1d_bwd_weight(xd, dyd, empty((Cout, k, Cin)), empty((Cout,)), s, False, ws)
    dw = to_host(dw).reshape(-1)
    idx = sample(dw.size)
    corners = [(co * k + j) * Cin + c for co in (0, Cout - 1) for j in range(k) for c in (0, Cin - 1)]
    idx = np.unique(np.concatenate([idx, np.array(corners)]))
    ref = oracle.conv1d_bwd_weight_at(x, dy, k, idx, s)
    assert rel_l2(dw[idx], ref) <= 1e-4
    assert rel_l2(to_host(db), dy.astype(np.float64).sum((0, 1))) <= 1e-5


def test_train_step_105m_forward_and_sampled_gradients(P):
    """The benchmark configuration itself (B=8, 11 layers, 107M parameters).  The fp64 oracle
    runs the whole network for one utterance only (the batch couples utterances only through
    the sums in dw/db): its loss and logits must match the full-batch GPU step."""
    cfg = W.config4()
    got = run_train_step(P, cfg)
    assert np.all(np.isfinite(got["loss"]))
    b = 3
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    ref = oracle.train_step(cfg["layers"], [f64(w) for w in cfg["weights"]], [f64(v) for v in cfg["biases"]],
                            f64(cfg["x"][b:b + 1]), cfg["in_len"][b:b + 1], cfg["targets"][b:b + 1],
                            cfg["tgt_len"][b:b + 1])
    assert abs(got["loss"][b] - ref["loss"][0]) <= 2e-2 * abs(ref["loss"][0])
    assert rel_l2(got["logits"][b], ref["logits"][0]) <= 2e-2
    for t in got["dw"] + got["db"]:
        assert np.all(np.isfinite(t))
