"""Pins of the oracle's temporal convolution and its two gradients (paper Sec. 2.3 names
1-D convolutions; the paper gives no formula, the definitions are stated in
oracle/w2l_oracle.c).  Pins: reduction to a matrix product for k=1, pure time shift for a
one-hot kernel, linearity, stride-2 = subsampled stride-1, batch independence, adjoint
identities, finite differences, and torch's CPU conv1d as an independent third opinion."""
import numpy as np
import pytest

import oracle


def rnd(rng, *shape):
    return rng.standard_normal(shape)


def test_k1_is_matrix_product():
    rng = np.random.default_rng(0)
    x, w, b = rnd(rng, 3, 17, 5), rnd(rng, 7, 1, 5), rnd(rng, 7)
    y = oracle.conv1d_fwd(x, w, b)
    np.testing.assert_allclose(y, x @ w[:, 0, :].T + b, atol=1e-12)


@pytest.mark.parametrize("k,j", [(5, 0), (5, 2), (5, 4), (3, 2), (7, 1)])
def test_one_hot_kernel_is_time_shift(k, j):
    rng = np.random.default_rng(1)
    T, Cc = 12, 4
    x = rnd(rng, 2, T, Cc)
    w = np.zeros((Cc, k, Cc))
    w[np.arange(Cc), j, np.arange(Cc)] = 1.0
    y = oracle.conv1d_fwd(x, w, None)
    p = (k - 1) // 2
    expect = np.zeros_like(x)
    for t in range(T):
        src = t + j - p
        if 0 <= src < T:
            expect[:, t] = x[:, src]
    np.testing.assert_allclose(y, expect, atol=0)


def test_linearity_and_batch_independence():
    rng = np.random.default_rng(2)
    x1, x2 = rnd(rng, 2, 20, 6), rnd(rng, 2, 20, 6)
    w1, w2 = rnd(rng, 8, 5, 6), rnd(rng, 8, 5, 6)
    f = lambda x, w: oracle.conv1d_fwd(x, w, None, 1)
    np.testing.assert_allclose(f(2 * x1 - 3 * x2, w1), 2 * f(x1, w1) - 3 * f(x2, w1), atol=1e-12)
    np.testing.assert_allclose(f(x1, w1 + 0.5 * w2), f(x1, w1) + 0.5 * f(x1, w2), atol=1e-12)
    np.testing.assert_allclose(f(x1, w1)[1], f(x1[1:], w1)[0], atol=0)


@pytest.mark.parametrize("T", [20, 21])
def test_stride2_is_subsampled_stride1(T):
    rng = np.random.default_rng(3)
    x, w, b = rnd(rng, 2, T, 3), rnd(rng, 4, 7, 3), rnd(rng, 4)
    y1 = oracle.conv1d_fwd(x, w, b, 1)
    y2 = oracle.conv1d_fwd(x, w, b, 2)
    assert y2.shape[1] == (T + 1) // 2
    np.testing.assert_allclose(y2, y1[:, ::2], atol=0)


@pytest.mark.parametrize("k,s,T", [(1, 1, 9), (5, 1, 16), (11, 1, 13), (13, 2, 21), (3, 2, 10), (5, 3, 17)])
def test_adjoint_identities(k, s, T):
    rng = np.random.default_rng(10 + k + s)
    B, Cin, Cout = 3, 5, 4
    x, w = rnd(rng, B, T, Cin), rnd(rng, Cout, k, Cin)
    y = oracle.conv1d_fwd(x, w, None, s)
    dy = rnd(rng, *y.shape)
    dx = oracle.conv1d_bwd_data(dy, w, T, s)
    dw, db = oracle.conv1d_bwd_weight(x, dy, k, s)
    ref = np.vdot(y, dy)
    assert abs(np.vdot(x, dx) - ref) < 1e-12 * abs(ref) + 1e-12
    assert abs(np.vdot(w, dw) - ref) < 1e-12 * abs(ref) + 1e-12
    bias = rnd(rng, Cout)
    yb = oracle.conv1d_fwd(np.zeros_like(x), w, bias, s)
    assert abs(np.vdot(yb, dy) - np.vdot(bias, db)) < 1e-12 * abs(np.vdot(bias, db)) + 1e-12


def test_gradients_by_finite_differences():
    rng = np.random.default_rng(20)
    B, T, Cin, Cout, k, s = 2, 11, 3, 4, 5, 2
    x, w, b = rnd(rng, B, T, Cin), rnd(rng, Cout, k, Cin), rnd(rng, Cout)
    r = rnd(rng, B, (T + s - 1) // s, Cout)
    f = lambda x, w, b: np.vdot(oracle.conv1d_fwd(x, w, b, s), r)
    dx = oracle.conv1d_bwd_data(r, w, T, s)
    dw, db = oracle.conv1d_bwd_weight(x, r, k, s)
    h = 1e-6
    for arr, g, which in ((x, dx, 0), (w, dw, 1), (b, db, 2)):
        for _ in range(15):
            idx = tuple(rng.integers(n) for n in arr.shape)
            d = np.zeros_like(arr)
            d[idx] = h
            args_p = [x, w, b]
            args_m = [x, w, b]
            args_p[which] = arr + d
            args_m[which] = arr - d
            fd = (f(*args_p) - f(*args_m)) / (2 * h)
            assert abs(fd - g[idx]) < 1e-7 * max(1.0, abs(fd))


@pytest.mark.parametrize("k,s", [(11, 1), (13, 2), (1, 1)])
def test_against_torch_cpu(k, s):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(30 + k)
    B, T, Cin, Cout = 2, 23, 6, 5
    x, w, b = rnd(rng, B, T, Cin), rnd(rng, Cout, k, Cin), rnd(rng, Cout)
    xt = torch.tensor(x.transpose(0, 2, 1), dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w.transpose(0, 2, 1).copy(), dtype=torch.float64, requires_grad=True)
    bt = torch.tensor(b, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.conv1d(xt, wt, bt, stride=s, padding=(k - 1) // 2)
    y = oracle.conv1d_fwd(x, w, b, s)
    np.testing.assert_allclose(y, yt.detach().numpy().transpose(0, 2, 1), atol=1e-12)
    dy = rnd(rng, *y.shape)
    yt.backward(torch.tensor(dy.transpose(0, 2, 1).copy()))
    np.testing.assert_allclose(oracle.conv1d_bwd_data(dy, w, T, s),
                               xt.grad.numpy().transpose(0, 2, 1), atol=1e-12)
    dw, db = oracle.conv1d_bwd_weight(x, dy, k, s)
    np.testing.assert_allclose(dw, wt.grad.numpy().transpose(0, 2, 1), atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), atol=1e-12)


def test_sampled_variants_equal_full():
    rng = np.random.default_rng(40)
    B, T, Cin, Cout, k, s = 2, 15, 4, 6, 5, 2
    x, w, b = rnd(rng, B, T, Cin), rnd(rng, Cout, k, Cin), rnd(rng, Cout)
    y = oracle.conv1d_fwd(x, w, b, s)
    dy = rnd(rng, *y.shape)
    dx = oracle.conv1d_bwd_data(dy, w, T, s)
    dw, _ = oracle.conv1d_bwd_weight(x, dy, k, s)
    for full, fn in ((y, lambda i: oracle.conv1d_fwd_at(x, w, b, i, s)),
                     (dx, lambda i: oracle.conv1d_bwd_data_at(dy, w, T, i, s)),
                     (dw, lambda i: oracle.conv1d_bwd_weight_at(x, dy, k, i, s))):
        idx = rng.integers(0, full.size, size=50)
        np.testing.assert_array_equal(fn(idx), full.reshape(-1)[idx])
