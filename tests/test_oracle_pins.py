"""Pins for the CPU oracle: each test fixes the oracle to something other than itself.

Sources of truth used here: the defining sums written out as brute-force Python loops on tiny shapes,
hand-countable cases, the adjoint identity <conv(x), y> = <x, convT(y)>, linearity in the weights,
central finite differences in double precision, BatchNorm moment invariants, closed forms of the
logistic loss (Eqs. 3-4 with D = sigmoid(s)) and of Adam's first steps, and an independent library's
CPU operators used strictly as black boxes.
"""
import math

import numpy as np
import pytest

import oracle as O
from paper_2102_10485_amd import synth

rng0 = np.random.default_rng(1234)


def brute_conv(X, W, b, k, s, p):
    N, Ci, H, Wd = X.shape
    Co = W.shape[0]
    Ho, Wo = (H + 2 * p - k) // s + 1, (Wd + 2 * p - k) // s + 1
    Y = np.zeros((N, Co, Ho, Wo))
    for n in range(N):
        for co in range(Co):
            for oy in range(Ho):
                for ox in range(Wo):
                    acc = b[co]
                    for ci in range(Ci):
                        for ky in range(k):
                            for kx in range(k):
                                iy, ix = oy * s - p + ky, ox * s - p + kx
                                if 0 <= iy < H and 0 <= ix < Wd:
                                    acc += X[n, ci, iy, ix] * W[co, ci, ky, kx]
                    Y[n, co, oy, ox] = acc
    return Y


def brute_convT(X, W, b, k, s, p):
    """Gather form: Y[oy] takes X[(oy+p-ky)/s] when divisible and in range."""
    N, Ci, H, Wd = X.shape
    Co = W.shape[1]
    Ho, Wo = (H - 1) * s - 2 * p + k, (Wd - 1) * s - 2 * p + k
    Y = np.zeros((N, Co, Ho, Wo))
    for n in range(N):
        for co in range(Co):
            for oy in range(Ho):
                for ox in range(Wo):
                    acc = b[co]
                    for ci in range(Ci):
                        for ky in range(k):
                            for kx in range(k):
                                ty, tx = oy + p - ky, ox + p - kx
                                if ty % s or tx % s:
                                    continue
                                iy, ix = ty // s, tx // s
                                if 0 <= iy < H and 0 <= ix < Wd:
                                    acc += X[n, ci, iy, ix] * W[ci, co, ky, kx]
                    Y[n, co, oy, ox] = acc
    return Y


@pytest.mark.parametrize("k,s,p,H", [(4, 2, 1, 6), (3, 1, 1, 5), (3, 2, 1, 5), (4, 1, 0, 4)])
def test_conv2d_brute_force(k, s, p, H):
    X = rng0.normal(size=(2, 3, H, H + 1))
    W = rng0.normal(size=(4, 3, k, k))
    b = rng0.normal(size=4)
    np.testing.assert_allclose(O.conv2d(X, W, b, k, s, p), brute_conv(X, W, b, k, s, p), rtol=1e-13, atol=1e-13)


def test_conv2d_tap_count():
    # all-ones input and filter: the output counts the valid taps times Cin: 9 at corners, 12 on edges, 16 inside
    Cin = 5
    Y = O.conv2d(np.ones((1, Cin, 8, 8)), np.ones((1, Cin, 4, 4)), None)
    assert Y.shape == (1, 1, 4, 4)
    exp = np.full((4, 4), 16.0 * Cin)
    exp[0, :] = exp[-1, :] = exp[:, 0] = exp[:, -1] = 12.0 * Cin
    exp[0, 0] = exp[0, -1] = exp[-1, 0] = exp[-1, -1] = 9.0 * Cin
    np.testing.assert_array_equal(Y[0, 0], exp)


@pytest.mark.parametrize("k,s,p,H", [(4, 2, 1, 3), (3, 2, 1, 4), (4, 1, 0, 1)])
def test_conv_transpose_brute_force(k, s, p, H):
    X = rng0.normal(size=(2, 3, H, H))
    W = rng0.normal(size=(3, 2, k, k))
    b = rng0.normal(size=2)
    Y = O.conv_transpose2d(X, W, b, k, s, p)
    assert Y.shape[-1] == (H - 1) * s - 2 * p + k
    np.testing.assert_allclose(Y, brute_convT(X, W, b, k, s, p), rtol=1e-13, atol=1e-13)


def test_conv_transpose_is_adjoint_of_conv():
    x = rng0.normal(size=(3, 5, 8, 8))
    W = rng0.normal(size=(7, 5, 4, 4))        # conv: 5 -> 7 ; read as convT weight: 7 -> 5
    y = rng0.normal(size=(3, 7, 4, 4))
    lhs = np.sum(O.conv2d(x, W, None) * y)
    rhs = np.sum(x * O.conv_transpose2d(y, W, None))
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


def test_conv_transpose_1x1_input_is_outer_product():
    # k4 s1 p0 on a 1x1 map: Y[n,co,ky,kx] = sum_ci X[n,ci] W[ci,co,ky,kx]  (a linear layer)
    x = rng0.normal(size=(4, 6, 1, 1))
    W = rng0.normal(size=(6, 3, 4, 4))
    Y = O.conv_transpose2d(x, W, None, 4, 1, 0)
    np.testing.assert_allclose(Y, np.einsum("nc,cokl->nokl", x[:, :, 0, 0], W), rtol=1e-13, atol=1e-13)


def test_conv_backward_is_adjoint_and_linear():
    x = rng0.normal(size=(2, 3, 6, 6))
    W = rng0.normal(size=(4, 3, 4, 4))
    dY = rng0.normal(size=(2, 4, 3, 3))
    V = rng0.normal(size=W.shape)
    dX, dW, db = O.conv2d_bwd(x, W, dY)
    np.testing.assert_allclose(dX, O.conv_transpose2d(dY, W, None), rtol=1e-12, atol=1e-12)
    # the output is linear in W: <dW, V> = <conv(x; V), dY>
    assert abs(np.sum(dW * V) - np.sum(O.conv2d(x, V, None) * dY)) < 1e-11
    np.testing.assert_allclose(db, dY.sum(axis=(0, 2, 3)), rtol=1e-13)
    # each entry of dW is the derivative w.r.t. that single weight
    E = np.zeros_like(W)
    E[2, 1, 3, 0] = 1.0
    assert abs(dW[2, 1, 3, 0] - np.sum(O.conv2d(x, E, None) * dY)) < 1e-12


def test_conv_transpose_backward_is_adjoint_and_linear():
    x = rng0.normal(size=(2, 4, 3, 3))
    W = rng0.normal(size=(4, 3, 4, 4))
    dY = rng0.normal(size=(2, 3, 6, 6))
    V = rng0.normal(size=W.shape)
    dX, dW, db = O.conv_transpose2d_bwd(x, W, dY)
    np.testing.assert_allclose(dX, O.conv2d(dY, W, None), rtol=1e-12, atol=1e-12)
    assert abs(np.sum(dW * V) - np.sum(O.conv_transpose2d(x, V, None) * dY)) < 1e-11
    np.testing.assert_allclose(db, dY.sum(axis=(0, 2, 3)), rtol=1e-13)
    E = np.zeros_like(W)
    E[3, 0, 1, 2] = 1.0
    assert abs(dW[3, 0, 1, 2] - np.sum(O.conv_transpose2d(x, E, None) * dY)) < 1e-12


def test_linear_matches_matmul():
    X, W, b = rng0.normal(size=(5, 7)), rng0.normal(size=(3, 7)), rng0.normal(size=3)
    dY = rng0.normal(size=(5, 3))
    np.testing.assert_allclose(O.linear(X, W, b), X @ W.T + b, rtol=1e-13)
    dX, dW, db = O.linear_bwd(X, W, dY)
    np.testing.assert_allclose(dX, dY @ W, rtol=1e-13)
    np.testing.assert_allclose(dW, dY.T @ X, rtol=1e-13)
    np.testing.assert_allclose(db, dY.sum(0), rtol=1e-13)


def test_bn_forward_invariants():
    X = rng0.normal(2.0, 3.0, size=(6, 4, 5, 5))
    g, b = np.ones(4), np.zeros(4)
    eps = 1e-5
    Y, mean, var = O.bn_train(X, g, b, eps)
    np.testing.assert_allclose(mean, X.mean(axis=(0, 2, 3)), rtol=1e-13)
    np.testing.assert_allclose(var, X.var(axis=(0, 2, 3)), rtol=1e-12)            # biased
    np.testing.assert_allclose(Y.mean(axis=(0, 2, 3)), 0.0, atol=1e-13)
    np.testing.assert_allclose(Y.var(axis=(0, 2, 3)), var / (var + eps), rtol=1e-12)
    # eps = 0: invariant under positive rescaling of the input
    Y0, _, _ = O.bn_train(X, g, b, 0.0)
    Y1, _, _ = O.bn_train(7.5 * X, g, b, 0.0)
    np.testing.assert_allclose(Y0, Y1, rtol=1e-11, atol=1e-12)
    # affine part
    g2, b2 = rng0.normal(size=4), rng0.normal(size=4)
    Y2, _, _ = O.bn_train(X, g2, b2, eps)
    np.testing.assert_allclose(Y2, Y * g2[None, :, None, None] + b2[None, :, None, None], rtol=1e-12, atol=1e-12)
    # the paper's tables list eps = 0.8 on most layers: the variance is then var/(var+0.8)
    Y8, _, _ = O.bn_train(X, g, b, 0.8)
    np.testing.assert_allclose(Y8.var(axis=(0, 2, 3)), var / (var + 0.8), rtol=1e-12)
    # evaluation mode with the same statistics reproduces the training output
    np.testing.assert_allclose(O.bn_eval(X, g2, b2, eps, mean, var), Y2, rtol=1e-13, atol=1e-13)


def test_bn_running_update():
    rm, rv = np.array([1.0, -2.0]), np.array([1.0, 4.0])
    mean, var = np.array([0.5, 0.25]), np.array([2.0, 3.0])
    m2, v2 = O.bn_running_update(rm, rv, mean, var, 0.1, 10)
    np.testing.assert_allclose(m2, 0.9 * rm + 0.1 * mean, rtol=1e-15)
    np.testing.assert_allclose(v2, 0.9 * rv + 0.1 * var * 10.0 / 9.0, rtol=1e-15)
    m3, v3 = O.bn_running_update(rm, rv, mean, var, 0.1, 1)       # single element: variance untouched
    np.testing.assert_allclose(v3, rv)
    np.testing.assert_allclose(m3, m2)


def test_bn_backward_invariants_and_finite_differences():
    X = rng0.normal(size=(4, 3, 2, 3))
    g, b = rng0.normal(size=3), rng0.normal(size=3)
    dY = rng0.normal(size=X.shape)
    eps = 1e-3
    Y, mean, var = O.bn_train(X, g, b, eps)
    dX, dg, db = O.bn_bwd(X, g, mean, var, eps, dY)
    xh = (X - mean[None, :, None, None]) / np.sqrt(var + eps)[None, :, None, None]
    np.testing.assert_allclose(dX.sum(axis=(0, 2, 3)), 0.0, atol=1e-12)
    # sum dx*xhat = gamma*rstd*dgamma*(1 - var/(var+eps)): vanishes only as eps -> 0
    dX0, dg0, _ = O.bn_bwd(X, g, mean, var, 0.0, dY)
    xh0 = (X - mean[None, :, None, None]) / np.sqrt(var)[None, :, None, None]
    np.testing.assert_allclose((dX0 * xh0).sum(axis=(0, 2, 3)), 0.0, atol=1e-11)
    np.testing.assert_allclose(db, dY.sum(axis=(0, 2, 3)), rtol=1e-13)
    np.testing.assert_allclose(dg, (dY * xh).sum(axis=(0, 2, 3)), rtol=1e-12)

    def f(Xp):
        return np.sum(O.bn_train(Xp, g, b, eps)[0] * dY)

    h = 1e-6
    for idx in [(0, 0, 0, 0), (3, 2, 1, 2), (1, 1, 0, 1)]:
        Xp, Xm = X.copy(), X.copy()
        Xp[idx] += h
        Xm[idx] -= h
        fd = (f(Xp) - f(Xm)) / (2 * h)
        assert abs(fd - dX[idx]) < 1e-7 * max(1.0, abs(fd))


def test_activations():
    x = np.array([-2.0, -0.0, 0.0, 1.5])
    np.testing.assert_array_equal(O.leaky_relu(x, 0.2), [-0.4, -0.0, 0.0, 1.5])
    np.testing.assert_array_equal(O.leaky_relu(x, 0.0), [0.0, 0.0, 0.0, 1.5])
    dy = np.array([1.0, 2.0, 3.0, 4.0])
    np.testing.assert_allclose(O.leaky_relu_bwd(x, dy, 0.2), [0.2, 0.4, 0.6, 4.0], rtol=1e-15)   # slope branch at 0
    np.testing.assert_array_equal(O.leaky_relu_bwd(x, dy, 0.0), [0.0, 0.0, 0.0, 4.0])
    t = O.tanh(np.array([-50.0, -1.0, 0.0, 0.3, 50.0]))
    assert np.all(np.abs(t) <= 1.0) and t[2] == 0.0
    np.testing.assert_allclose(t[1], -math.tanh(1.0), rtol=1e-15)
    h = 1e-6
    fd = (math.tanh(0.3 + h) - math.tanh(0.3 - h)) / (2 * h)
    np.testing.assert_allclose(O.tanh_bwd(t, np.ones(5))[3], fd, rtol=1e-9)


def test_logistic_loss_closed_forms():
    # s = 0 => D = 1/2: -log D = log 2 for every sample
    v, ds = O.logistic_loss(np.zeros(8), -1, 0.5)
    assert abs(v - 0.5 * math.log(2.0)) < 1e-15
    np.testing.assert_allclose(ds, -0.5 * 0.5 / 8)
    v, ds = O.logistic_loss(np.zeros(8), +1, 0.5)
    assert abs(v - 0.5 * math.log(2.0)) < 1e-15
    np.testing.assert_allclose(ds, +0.5 * 0.5 / 8)
    s = np.array([-3.0, 0.7, 2.0])
    Dv = 1.0 / (1.0 + np.exp(-s))
    v, ds = O.logistic_loss(s, -1, 0.5)                           # -1/2 E log D
    np.testing.assert_allclose(v, -0.5 * np.mean(np.log(Dv)), rtol=1e-13)
    np.testing.assert_allclose(ds, 0.5 * (Dv - 1.0) / 3, rtol=1e-13)
    v, ds = O.logistic_loss(s, +1, 0.5)                           # -1/2 E log(1 - D)
    np.testing.assert_allclose(v, -0.5 * np.mean(np.log(1.0 - Dv)), rtol=1e-13)
    np.testing.assert_allclose(ds, 0.5 * Dv / 3, rtol=1e-13)
    for big in (100.0, -100.0, 800.0, -800.0):
        v, ds = O.logistic_loss(np.array([big]), -1, 1.0)
        assert np.isfinite(v) and np.all(np.isfinite(ds))
        np.testing.assert_allclose(v, max(-big, 0.0), atol=1e-12)


def test_adam_closed_forms():
    g = np.array([3.0, -0.02, 1e-3, 0.0])
    th0 = np.array([1.0, 1.0, 1.0, 1.0])
    th, m, v = O.adam(th0, np.zeros(4), np.zeros(4), g, 1)
    # first step: m_hat = g, v_hat = g^2 => step = lr * g / (|g| + eps)
    np.testing.assert_allclose(th, th0 - 2e-4 * g / (np.abs(g) + 1e-8), rtol=1e-14)
    assert th[3] == 1.0
    np.testing.assert_allclose(m, 0.5 * g)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-12)
    # constant gradient: bias correction is exact, every step moves by lr*sign(g)
    th, m, v = th0.copy(), np.zeros(4), np.zeros(4)
    for t in range(1, 8):
        th, m, v = O.adam(th, m, v, g, t)
    np.testing.assert_allclose(th[:3], th0[:3] - 7 * 2e-4 * np.sign(g[:3]), rtol=0, atol=7 * 2e-4 * 2e-5)
    assert th[3] == 1.0


def test_routing_brute_force():
    lab = np.array([3, 1, 3, 0, 2, 1, 3, 0, 9, -1], np.int32)
    perm, offs, bad = O.route(lab, 4, 4)
    assert bad == 2
    exp = [[i for i, y in enumerate(lab) if y == l] for l in range(4)]
    assert list(offs) == [0, 2, 4, 5, 8]
    assert list(perm[:8]) == sum(exp, [])
    perm, offs, bad = O.route(np.array([3, 1, 2], np.int32), 1, 4)   # a single model takes every label
    assert list(perm) == [0, 1, 2] and list(offs) == [0, 3] and bad == 0


def test_library_cross_check_ops():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    T = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    x = rng0.normal(size=(3, 5, 10, 10))
    W = rng0.normal(size=(6, 5, 4, 4))
    b = rng0.normal(size=6)
    np.testing.assert_allclose(O.conv2d(x, W, b), F.conv2d(T(x), T(W), T(b), stride=2, padding=1).numpy(),
                               rtol=1e-12, atol=1e-12)
    y = rng0.normal(size=(3, 6, 5, 5))
    b5 = rng0.normal(size=5)
    np.testing.assert_allclose(O.conv_transpose2d(y, W, b5),
                               F.conv_transpose2d(T(y), T(W), T(b5), stride=2, padding=1).numpy(),
                               rtol=1e-12, atol=1e-12)
    g, be = rng0.normal(size=5), rng0.normal(size=5)
    rm, rv = torch.zeros(5, dtype=torch.float64), torch.ones(5, dtype=torch.float64)
    yt = F.batch_norm(T(x), rm, rv, T(g), T(be), training=True, momentum=0.1, eps=1e-5)
    Y, mean, var = O.bn_train(x, g, be, 1e-5)
    np.testing.assert_allclose(Y, yt.numpy(), rtol=1e-11, atol=1e-11)
    m2, v2 = O.bn_running_update(np.zeros(5), np.ones(5), mean, var, 0.1, 3 * 100)
    np.testing.assert_allclose(m2, rm.numpy(), rtol=1e-12)
    np.testing.assert_allclose(v2, rv.numpy(), rtol=1e-12)
    s = rng0.normal(size=9) * 4
    v, _ = O.logistic_loss(s, -1, 1.0)
    np.testing.assert_allclose(v, F.binary_cross_entropy_with_logits(T(s), torch.ones(9, dtype=torch.float64)).item(),
                               rtol=1e-13)
    v, _ = O.logistic_loss(s, +1, 1.0)
    np.testing.assert_allclose(v, F.binary_cross_entropy_with_logits(T(s), torch.zeros(9, dtype=torch.float64)).item(),
                               rtol=1e-13)


def test_label_map_shortcut_identity():
    """A constant one-hot input plane contributes, per output position, the sum of the weights of the taps
    that fall inside the image; its weight gradient is the sum of dY over the positions where the tap is valid."""
    C, cond, y = 3, 5, 2
    H = 8
    x = rng0.normal(size=(2, C, H, H))
    maps = np.zeros((2, cond, H, H))
    maps[:, y] = 1.0
    W = rng0.normal(size=(4, C + cond, 4, 4))
    dense = O.conv2d(np.concatenate([x, maps], 1), W, None)
    Ho = H // 2
    valid = np.ones((Ho, 4), bool)           # valid[o, k]: tap k is inside the image at output row/col o
    valid[0, 0] = False
    valid[Ho - 1, 3] = False
    table = np.einsum("ak,bl,ckl->cab", valid, valid, W[:, C + y])     # [co, oy, ox]
    np.testing.assert_allclose(dense, O.conv2d(x, W[:, :C], None) + table[None], rtol=1e-12, atol=1e-12)
    dY = rng0.normal(size=dense.shape)
    _, dW, _ = O.conv2d_bwd(np.concatenate([x, maps], 1), W, dY, need_dx=False)
    exp = np.einsum("ncab,ak,bl->ckl", dY, valid, valid)
    np.testing.assert_allclose(dW[:, C + y], exp, rtol=1e-12, atol=1e-12)
    assert np.all(dW[:, C + np.array([0, 1, 3, 4])] == 0.0)
