"""Pins of the oracle's GLU, log-softmax and composed train step (paper Sec. 2.3: network
then criterion; Sec. 4.1: the gated all-convolutional network).  Closed forms, invariants,
finite differences, and torch's CPU ops as an independent third opinion."""
import numpy as np
import pytest

import oracle
import workloads as W


def test_glu_special_values_and_split():
    a = np.array([[1.5, -2.0, 0.25]])
    y = np.concatenate([a, np.zeros_like(a)], -1)
    np.testing.assert_allclose(oracle.glu_fwd(y), a / 2, atol=0)          # sigmoid(0) = 1/2
    y = np.concatenate([a, np.full_like(a, 800.0)], -1)
    np.testing.assert_allclose(oracle.glu_fwd(y), a, atol=0)              # gate -> 1
    y = np.concatenate([a, np.full_like(a, -800.0)], -1)
    np.testing.assert_allclose(oracle.glu_fwd(y), 0 * a, atol=0)          # gate -> 0
    # first half is the value, second half the gate
    y = np.array([[3.0, 0.0]])
    assert oracle.glu_fwd(y)[0, 0] == 1.5
    y = np.array([[0.0, 3.0]])
    assert oracle.glu_fwd(y)[0, 0] == 0.0


def test_glu_bwd_finite_differences_and_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    y, dh = rng.standard_normal((4, 5, 10)), rng.standard_normal((4, 5, 5))
    dy = oracle.glu_bwd(y, dh)
    h = 1e-6
    for _ in range(30):
        idx = tuple(rng.integers(n) for n in y.shape)
        d = np.zeros_like(y)
        d[idx] = h
        fd = (np.vdot(oracle.glu_fwd(y + d), dh) - np.vdot(oracle.glu_fwd(y - d), dh)) / (2 * h)
        assert abs(fd - dy[idx]) < 1e-8 * max(1.0, abs(fd))
    yt = torch.tensor(y, requires_grad=True)
    ht = torch.nn.functional.glu(yt, dim=-1)
    np.testing.assert_allclose(oracle.glu_fwd(y), ht.detach().numpy(), atol=1e-14)
    ht.backward(torch.tensor(dh))
    np.testing.assert_allclose(dy, yt.grad.numpy(), atol=1e-14)


def test_logsoftmax_invariants():
    rng = np.random.default_rng(1)
    z = rng.standard_normal((3, 7, 29)) * 4
    lp = oracle.logsoftmax_fwd(z)
    np.testing.assert_allclose(np.exp(lp).sum(-1), 1.0, atol=1e-14)
    np.testing.assert_allclose(oracle.logsoftmax_fwd(z + 123.0), lp, atol=1e-12)
    np.testing.assert_allclose(lp - lp[..., :1], z - z[..., :1], atol=1e-12)
    big = np.array([[1000.0, 0.0, -1000.0]])
    out = oracle.logsoftmax_fwd(big)
    assert np.all(np.isfinite(out)) and abs(out[0, 0]) < 1e-300 + 1e-12 and out[0, 2] == -2000.0
    np.testing.assert_allclose(oracle.logsoftmax_fwd(np.zeros((1, 8))), -np.log(8.0), atol=1e-15)


def test_logsoftmax_bwd_finite_differences_and_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    z, dlp = rng.standard_normal((5, 11)), rng.standard_normal((5, 11))
    lp = oracle.logsoftmax_fwd(z)
    dz = oracle.logsoftmax_bwd(lp, dlp)
    h = 1e-6
    for _ in range(30):
        idx = tuple(rng.integers(n) for n in z.shape)
        d = np.zeros_like(z)
        d[idx] = h
        fd = (np.vdot(oracle.logsoftmax_fwd(z + d), dlp) - np.vdot(oracle.logsoftmax_fwd(z - d), dlp)) / (2 * h)
        assert abs(fd - dz[idx]) < 1e-8 * max(1.0, abs(fd))
    zt = torch.tensor(z, requires_grad=True)
    lt = torch.log_softmax(zt, -1)
    lt.backward(torch.tensor(dlp))
    np.testing.assert_allclose(lp, lt.detach().numpy(), atol=1e-14)
    np.testing.assert_allclose(dz, zt.grad.numpy(), atol=1e-14)


def test_ctc_against_torch_cpu():
    torch = pytest.importorskip("torch")
    cfg = W.config2(seed=11, B=4, T=60, in_lo=40, in_hi=60, l_lo=3, l_hi=15)
    z = cfg["logits"].astype(np.float64)
    loss, lp, dz = oracle.ctc_from_logits(z, cfg["targets"], cfg["in_len"], cfg["tgt_len"])
    zt = torch.tensor(z, requires_grad=True)
    lpt = torch.log_softmax(zt, -1).transpose(0, 1)
    lt = torch.nn.functional.ctc_loss(lpt, torch.tensor(cfg["targets"], dtype=torch.long),
                                      torch.tensor(cfg["in_len"], dtype=torch.long),
                                      torch.tensor(cfg["tgt_len"], dtype=torch.long),
                                      blank=0, reduction="none")
    lt.sum().backward()
    np.testing.assert_allclose(loss, lt.detach().numpy(), rtol=1e-12)
    np.testing.assert_allclose(dz, zt.grad.numpy(), atol=1e-11)


def _tiny(seed=0):
    cfg = W.config0(seed=seed, zero_bias=False)
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    return cfg, f64(cfg["x"]), [f64(w) for w in cfg["weights"]], [f64(b) for b in cfg["biases"]]


def test_train_step_finite_differences_on_tiny_config():
    cfg, x, ws, bs = _tiny()
    out = oracle.train_step(cfg["layers"], ws, bs, x, cfg["in_len"], cfg["targets"], cfg["tgt_len"])
    assert np.all(np.isfinite(out["loss"]))
    rng = np.random.default_rng(5)
    h = 1e-6

    def total(ws_, bs_):
        return oracle.train_step(cfg["layers"], ws_, bs_, x, cfg["in_len"], cfg["targets"],
                                 cfg["tgt_len"])["loss"].sum()

    for li in range(len(ws)):
        for _ in range(6):
            idx = tuple(rng.integers(n) for n in ws[li].shape)
            wp = [w.copy() for w in ws]
            wm = [w.copy() for w in ws]
            wp[li][idx] += h
            wm[li][idx] -= h
            fd = (total(wp, bs) - total(wm, bs)) / (2 * h)
            assert abs(fd - out["dw"][li][idx]) < 2e-6 * max(1.0, abs(fd))
        c = rng.integers(bs[li].size)
        bp = [b.copy() for b in bs]
        bm = [b.copy() for b in bs]
        bp[li][c] += h
        bm[li][c] -= h
        fd = (total(ws, bp) - total(ws, bm)) / (2 * h)
        assert abs(fd - out["db"][li][c]) < 2e-6 * max(1.0, abs(fd))


def test_train_step_descent_and_batch_permutation():
    cfg, x, ws, bs = _tiny(seed=1)
    args = (cfg["in_len"], cfg["targets"], cfg["tgt_len"])
    out = oracle.train_step(cfg["layers"], ws, bs, x, *args)
    lr = 1e-3
    ws2 = [w - lr * g for w, g in zip(ws, out["dw"])]
    bs2 = [b - lr * g for b, g in zip(bs, out["db"])]
    out2 = oracle.train_step(cfg["layers"], ws2, bs2, x, *args)
    assert out2["loss"].sum() < out["loss"].sum()
    perm = [1, 0]
    outp = oracle.train_step(cfg["layers"], ws, bs, x[perm], cfg["in_len"][perm],
                             cfg["targets"][perm], cfg["tgt_len"][perm])
    np.testing.assert_allclose(outp["loss"], out["loss"][perm], rtol=1e-13)
    for a, b in zip(outp["dw"], out["dw"]):
        np.testing.assert_allclose(a, b, atol=1e-11)


def test_train_step_length_mask():
    # frames beyond in_len are zero input; the criterion ignores them and their logits
    # receive no gradient.  Stride-2 first layer: criterion length = ceil(in_len / 2).
    layers = [dict(k=5, stride=2, cin=6, cout=8, glu=1), dict(k=3, stride=1, cin=4, cout=5, glu=0)]
    cfg = W.small_model(3, 3, 11, 20, 6, layers, False, 1, 3)
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    out = oracle.train_step(layers, [f64(w) for w in cfg["weights"]], [f64(b) for b in cfg["biases"]],
                            f64(cfg["x"]), cfg["in_len"], cfg["targets"] % 5 + (cfg["targets"] % 5 == 0),
                            cfg["tgt_len"])
    for b in range(3):
        n = (cfg["in_len"][b] + 1) // 2
        assert out["crit_len"][b] == n
        assert np.all(out["dlogits"][b, n:] == 0)
        assert np.any(out["dlogits"][b, :n] != 0)


def test_workload_recipes():
    c2 = W.config2()
    assert c2["logits"].shape == (32, 750, 29) and c2["logits"].dtype == np.float32
    assert 600 <= c2["in_len"].min() and c2["in_len"].max() <= 750
    assert 50 <= c2["tgt_len"].min() and c2["tgt_len"].max() <= 200
    for b in range(32):
        lab = c2["targets"][b, :c2["tgt_len"][b]]
        assert lab.min() >= 1 and lab.max() <= 28
        assert c2["in_len"][b] >= len(lab) + np.sum(lab[1:] == lab[:-1])
    assert abs(float(c2["logits"].var()) - 2.0) < 0.02
    assert W.num_params(W.layers_105m()) == 107024925
    assert W.num_params(W.layers_10m()) == 9198621
    assert W.num_params(W.layers_tiny()) == 68701
    assert abs(W.step_flops(W.layers_105m(), 8, 1500) / 1e9 - 3833.2) < 0.1
    c0 = W.config0()
    assert c0["x"].shape == (2, 100, 40) and list(c0["tgt_len"]) == [10, 7]
    assert all(np.all(b == 0) for b in c0["biases"])
    # same seed -> same bits
    np.testing.assert_array_equal(W.config0()["x"], c0["x"])
    # bf16 rounding: representable, nearest, ties to even
    v = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -9, -3.1415926], np.float32)
    r = W.round_to_bf16(v)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2 ** -6 and r[3] == 1.0
    assert abs(r[4] - v[4]) <= abs(v[4]) * 2 ** -8
    np.testing.assert_array_equal(W.bits_to_f32(W.bf16_bits(r)), r)


def test_sgd_momentum_pins():
    """Pins of the SGD-with-momentum oracle (paper Sec. 4.1 names the optimiser; the update is the
    classical heavy-ball form): closed forms that a dropped term or a wrong sign would break."""
    rng = np.random.default_rng(7)
    w0 = rng.standard_normal(257)
    g = rng.standard_normal(257)
    v0 = np.zeros(257)
    # momentum 0, no decay: plain gradient descent
    w1, v1 = oracle.sgd_momentum(w0, v0, g, 0.1, 0.0)
    np.testing.assert_allclose(w1, w0 - 0.1 * g, rtol=0, atol=1e-15)
    np.testing.assert_allclose(v1, g, rtol=0, atol=0)
    # constant gradient, n steps: v_n = g (1 - mu^n) / (1 - mu),  w_n = w_0 - lr * sum_i v_i
    mu, lr, n = 0.9, 0.05, 25
    w, v = w0.copy(), v0.copy()
    for _ in range(n):
        w, v = oracle.sgd_momentum(w, v, g, lr, mu)
    vn = g * (1 - mu ** n) / (1 - mu)
    sum_v = g * (n - mu * (1 - mu ** n) / (1 - mu)) / (1 - mu)
    np.testing.assert_allclose(v, vn, rtol=1e-12)
    np.testing.assert_allclose(w, w0 - lr * sum_v, rtol=1e-12, atol=1e-12)
    # quadratic bowl f = a w^2 / 2 (g = a w): the iterates follow the 2x2 linear recurrence
    #   [w'; v'] = [[1 - lr a, -lr mu], [a, mu]] [w; v];  its powers give the iterate in closed form
    a_, lr, mu = 2.0, 0.1, 0.5
    M = np.array([[1 - lr * a_, -lr * mu], [a_, mu]])
    w, v = np.array([1.5]), np.array([0.25])
    for _ in range(7):
        w, v = oracle.sgd_momentum(w, v, a_ * w, lr, mu)
    ref = np.linalg.matrix_power(M, 7) @ np.array([1.5, 0.25])
    np.testing.assert_allclose([w[0], v[0]], ref, rtol=1e-12)
    # weight decay is the gradient of wd |w|^2 / 2 added to g; inputs are not modified
    w2, v2 = oracle.sgd_momentum(w0, v0, g, 0.1, 0.9, weight_decay=0.01)
    w3, v3 = oracle.sgd_momentum(w0, v0, g + 0.01 * w0, 0.1, 0.9)
    np.testing.assert_allclose(w2, w3, rtol=1e-15)
    np.testing.assert_allclose(v2, v3, rtol=1e-15)
    assert np.all(v0 == 0)
