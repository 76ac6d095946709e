"""Pins for oracle/layers.py and the C direct convolution: brute force, adjoints, float64
library routines as special cases, closed forms, finite differences."""
import itertools
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import layers as L

CONV_CASES = [  # N C H W K R stride pad
    (2, 3, 5, 5, 4, 3, 1, 1), (1, 2, 6, 7, 3, 3, 2, 1), (2, 4, 4, 4, 5, 1, 1, 0),
    (2, 4, 6, 6, 3, 1, 2, 0), (1, 3, 9, 9, 2, 7, 2, 3), (1, 1, 3, 3, 1, 3, 1, 1),
]


def _brute_conv(x, w, stride, pad):
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    y = np.zeros((N, K, P, Q))
    for n, k, p, q, c, r, s in itertools.product(range(N), range(K), range(P), range(Q),
                                                 range(C), range(R), range(S)):
        ih, iw = p * stride + r - pad, q * stride + s - pad
        if 0 <= ih < H and 0 <= iw < W:
            y[n, k, p, q] += x[n, c, ih, iw] * w[k, c, r, s]
    return y


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd_bruteforce(case):
    N, C, H, W, K, R, st, pad = case
    rng = np.random.default_rng(1)
    x, w = rng.standard_normal((N, C, H, W)), rng.standard_normal((K, C, R, R))
    np.testing.assert_allclose(L.conv2d_fwd(x, w, st, pad), _brute_conv(x, w, st, pad),
                               rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("case", CONV_CASES + [(3, 8, 12, 12, 16, 3, 2, 1), (2, 8, 8, 8, 8, 3, 1, 1)])
def test_conv_adjoint_and_library(case):
    """<conv(x,w), dy> = <x, dgrad(dy,w)> = <w, wgrad(dy,x)>, and all three equal the float64
    library convolution and its autograd."""
    N, C, H, W, K, R, st, pad = case
    rng = np.random.default_rng(2)
    x, w = rng.standard_normal((N, C, H, W)), rng.standard_normal((K, C, R, R))
    y = L.conv2d_fwd(x, w, st, pad)
    dy = rng.standard_normal(y.shape)
    dx = L.conv2d_dgrad(dy, w, x.shape, st, pad)
    dw = L.conv2d_wgrad(dy, x, w.shape, st, pad)
    ip = float((y * dy).sum())
    assert math.isclose(ip, float((x * dx).sum()), rel_tol=1e-10, abs_tol=1e-10)
    assert math.isclose(ip, float((w * dw).sum()), rel_tol=1e-10, abs_tol=1e-10)
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    yt = F.conv2d(xt, wt, stride=st, padding=pad)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_conv_dgrad_unit_impulse():
    """dgrad of a one-hot dy scatters the filter (a mistake in the index map shows here)."""
    w = np.arange(2 * 3 * 3 * 3, dtype=np.float64).reshape(2, 3, 3, 3)
    dy = np.zeros((1, 2, 3, 3))
    dy[0, 1, 1, 2] = 1.0
    dx = L.conv2d_dgrad(dy, w, (1, 3, 6, 6), 2, 1)        # stride 2: window rows 1..3, cols 3..5
    want = np.zeros((1, 3, 6, 6))
    want[0, :, 1:4, 3:6] = w[1]
    np.testing.assert_array_equal(dx, want)


def test_bn_forward_closed_forms():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((4, 5, 3, 3)) * 3 + 2
    eps = 1e-5
    y, (xhat, invstd, mean, var) = L.bn_fwd(x, np.ones(5), np.zeros(5), eps)
    np.testing.assert_allclose(y.mean(axis=(0, 2, 3)), 0, atol=1e-12)
    np.testing.assert_allclose(y.var(axis=(0, 2, 3)), var / (var + eps), rtol=1e-12)
    g, b = rng.standard_normal(5), rng.standard_normal(5)
    y2, _ = L.bn_fwd(x, g, b, eps)
    ref = F.batch_norm(torch.tensor(x), None, None, torch.tensor(g), torch.tensor(b), True, 0.1, eps)
    np.testing.assert_allclose(y2, ref.numpy(), rtol=1e-11, atol=1e-11)


def test_bn_running_stats_library():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((3, 4, 2, 2)) + 1
    rm0, rv0 = rng.standard_normal(4), rng.random(4) + 0.5
    _, (_, _, mean, var) = L.bn_fwd(x, np.ones(4), np.zeros(4), 1e-5)
    rm, rv = L.bn_running_update(rm0, rv0, mean, var, 12, 0.1)
    trm, trv = torch.tensor(rm0.copy()), torch.tensor(rv0.copy())
    F.batch_norm(torch.tensor(x), trm, trv, None, None, True, 0.1, 1e-5)
    np.testing.assert_allclose(rm, trm.numpy(), rtol=1e-12)
    np.testing.assert_allclose(rv, trv.numpy(), rtol=1e-12)


def test_bn_backward_invariants_and_fd():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 4, 3, 2))
    g, b = rng.standard_normal(4) + 1, rng.standard_normal(4)
    dy = rng.standard_normal(x.shape)
    y, cache = L.bn_fwd(x, g, b, 1e-5)
    dx, dg, db = L.bn_bwd(dy, cache, g)
    np.testing.assert_allclose(dx.sum(axis=(0, 2, 3)), 0, atol=1e-12)
    # sum dx*xhat = gamma*invstd*dgamma*(1 - sum(xhat^2)/m), and sum(xhat^2)/m = var/(var+eps)
    xhat, invstd, _, var = cache
    np.testing.assert_allclose((dx * xhat).sum(axis=(0, 2, 3)),
                               g * invstd * dg * (1e-5 / (var + 1e-5)), rtol=1e-9, atol=1e-13)
    f = lambda xx, gg, bb: float((L.bn_fwd(xx, gg, bb, 1e-5)[0] * dy).sum())
    h = 1e-6
    for idx in [(0, 0, 0, 0), (2, 3, 1, 1), (1, 2, 2, 0)]:
        e = np.zeros_like(x)
        e[idx] = h
        assert math.isclose((f(x + e, g, b) - f(x - e, g, b)) / (2 * h), dx[idx], rel_tol=1e-6, abs_tol=1e-8)
    for c in range(4):
        e = np.zeros(4)
        e[c] = h
        assert math.isclose((f(x, g + e, b) - f(x, g - e, b)) / (2 * h), dg[c], rel_tol=1e-6, abs_tol=1e-8)
        assert math.isclose((f(x, g, b + e) - f(x, g, b - e)) / (2 * h), db[c], rel_tol=1e-6, abs_tol=1e-8)


def test_maxpool_library_and_ties():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((2, 3, 8, 9))
    y, cache = L.maxpool_fwd(x)
    xt = torch.tensor(x, requires_grad=True)
    yt = F.max_pool2d(xt, 3, 2, 1)
    np.testing.assert_array_equal(y, yt.detach().numpy())
    dy = rng.standard_normal(y.shape)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(L.maxpool_bwd(dy, cache), xt.grad.numpy(), atol=1e-14)
    # ties: a constant image routes each window's gradient to its first in-range element
    xc = np.zeros((1, 1, 4, 4))
    yc, cache = L.maxpool_fwd(xc)
    dx = L.maxpool_bwd(np.ones_like(yc), cache)
    want = np.zeros((4, 4))
    want[0, 0] = want[0, 1] = want[1, 0] = want[1, 1] = 1.0   # windows start at (-1,-1),(-1,1),(1,-1),(1,1)
    np.testing.assert_array_equal(dx[0, 0], want)


def test_avgpool_fc_adjoint():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((3, 4, 2, 5))
    p = L.avgpool_fwd(x)
    np.testing.assert_allclose(p[1, 2], x[1, 2].sum() / 10)
    dp = rng.standard_normal(p.shape)
    assert math.isclose(float((p * dp).sum()), float((x * L.avgpool_bwd(dp, x.shape)).sum()), rel_tol=1e-12)
    w, b = rng.standard_normal((6, 4)), rng.standard_normal(6)
    z = L.fc_fwd(p, w, b)
    assert math.isclose(z[2, 5], sum(p[2, c] * w[5, c] for c in range(4)) + b[5], rel_tol=1e-12)
    dz = rng.standard_normal(z.shape)
    dx, dw, db = L.fc_bwd(dz, p, w)
    ip = float((dz * (z - b)).sum())
    assert math.isclose(ip, float((dx * p).sum()), rel_tol=1e-12)
    assert math.isclose(ip, float((dw * w).sum()), rel_tol=1e-12)
    np.testing.assert_allclose(db, dz.sum(0))


@pytest.mark.parametrize("classes", [10, 100, 1000])
def test_ce_closed_forms(classes):
    N = 6
    labels = np.arange(N) % classes
    loss, dz = L.softmax_ce(np.zeros((N, classes)), labels)
    assert math.isclose(loss, math.log(classes), rel_tol=1e-14)
    rng = np.random.default_rng(8)
    z = rng.standard_normal((N, classes)) * 5
    loss, dz = L.softmax_ce(z, labels)
    np.testing.assert_allclose(dz.sum(axis=1), 0, atol=1e-15)
    ref = F.cross_entropy(torch.tensor(z), torch.tensor(labels, dtype=torch.long))
    assert math.isclose(loss, float(ref), rel_tol=1e-13)
    # shift invariance and large logits (stable log-sum-exp)
    loss2, _ = L.softmax_ce(z + 1000.0, labels)
    assert math.isclose(loss, loss2, rel_tol=1e-10)


def test_single_output_functions_match_full_convolutions():
    """The one-output-at-a-time functions (used on full-size tensors) against the full-tensor oracle."""
    rng = np.random.default_rng(7)
    for (N, H, W, C, K, RS, st, pad) in [(2, 7, 6, 5, 4, 3, 1, 1), (2, 8, 8, 3, 6, 3, 2, 1), (3, 6, 6, 4, 5, 1, 2, 0),
                                         (1, 9, 9, 2, 3, 7, 2, 3)]:
        x = rng.standard_normal((N, C, H, W))
        w = rng.standard_normal((K, C, RS, RS))
        y = L.conv2d_fwd(x, w, st, pad)
        dy = rng.standard_normal(y.shape)
        dx = L.conv2d_dgrad(dy, w, x.shape, st, pad)
        dw = L.conv2d_wgrad(dy, x, w.shape, st, pad)
        xl, wl, dyl = x.transpose(0, 2, 3, 1), w.transpose(0, 2, 3, 1), dy.transpose(0, 2, 3, 1)
        P, Q = y.shape[2], y.shape[3]
        pts = [(rng.integers(N), rng.integers(P), rng.integers(Q), rng.integers(K)) for _ in range(20)] + [(0, 0, 0, 0), (N - 1, P - 1, Q - 1, K - 1)]
        np.testing.assert_allclose(L.conv2d_fwd_points(xl, wl, st, pad, pts), [y[n, k, p, q] for n, p, q, k in pts], rtol=1e-12, atol=1e-12)
        pts = [(rng.integers(N), rng.integers(H), rng.integers(W), rng.integers(C)) for _ in range(20)] + [(0, 0, 0, 0), (N - 1, H - 1, W - 1, C - 1)]
        np.testing.assert_allclose(L.conv2d_dgrad_points(dyl, wl, st, pad, pts), [dx[n, c, h, v] for n, h, v, c in pts], rtol=1e-12, atol=1e-12)
        pts = [(rng.integers(K), rng.integers(RS), rng.integers(RS), rng.integers(C)) for _ in range(20)] + [(0, 0, 0, 0), (K - 1, RS - 1, RS - 1, C - 1)]
        np.testing.assert_allclose(L.conv2d_wgrad_points(dyl, xl, st, pad, RS, RS, pts), [dw[k, c, r, s] for k, r, s, c in pts], rtol=1e-12, atol=1e-12)
