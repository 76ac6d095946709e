"""Oracle layer functions in float64 (numpy + the C direct convolution) -- TEST INFRASTRUCTURE ONLY.

Each function is the textbook definition of the layer a ResNet training step uses
(the paper's local update, Algorithm 1 inner loop, is ordinary SGD on such a network).
Logical layouts: activations [N,C,H,W], conv weights [K,C,R,S], FC weights [classes,C].
Pins (tests/test_oracle_layers.py): pure-Python brute-force loops on tiny shapes, adjoint
identities, float64 library routines as special cases, finite differences, closed forms.
"""
import ctypes

import numpy as np

from . import build as _build

_lib = None


def _conv_lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build.build())
        dp = ctypes.POINTER(ctypes.c_double)
        for name in ("oracle_conv2d_fwd", "oracle_conv2d_dgrad", "oracle_conv2d_wgrad"):
            f = getattr(_lib, name)
            f.argtypes = [dp, dp, dp] + [ctypes.c_int] * 9
            f.restype = None
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads():
    """Threads the C convolution loops actually run on (OpenMP's team size on this machine)."""
    return int(_conv_lib().oracle_num_threads())


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def conv_out(h, k, stride, pad):
    return (h + 2 * pad - k) // stride + 1


def conv2d_fwd(x, w, stride, pad):
    x, w = _f64(x), _f64(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    y = np.empty((N, K, conv_out(H, R, stride, pad), conv_out(W, S, stride, pad)), np.float64)
    _conv_lib().oracle_conv2d_fwd(_p(x), _p(w), _p(y), N, C, H, W, K, R, S, stride, pad)
    return y


def conv2d_dgrad(dy, w, x_shape, stride, pad):
    dy, w = _f64(dy), _f64(w)
    N, C, H, W = x_shape
    K, _, R, S = w.shape
    dx = np.empty((N, C, H, W), np.float64)
    _conv_lib().oracle_conv2d_dgrad(_p(dy), _p(w), _p(dx), N, C, H, W, K, R, S, stride, pad)
    return dx


def conv2d_wgrad(dy, x, w_shape, stride, pad):
    dy, x = _f64(dy), _f64(x)
    N, C, H, W = x.shape
    K, _, R, S = w_shape
    dw = np.empty((K, C, R, S), np.float64)
    _conv_lib().oracle_conv2d_wgrad(_p(dy), _p(x), _p(dw), N, C, H, W, K, R, S, stride, pad)
    return dw


# ---- single outputs of a convolution, straight from the definition ------------------------
# For tensors too large to run the whole oracle on: one output element at a time, float64, on
# channels-last arrays (x [N,H,W,C], w [K,R,S,C], y / dy [N,P,Q,K]) so that a test can hand over the
# tensors as the library lays them out.  Pinned against the full-tensor functions above.

def conv2d_fwd_points(x, w, stride, pad, points):
    """y[n,p,q,k] = sum_{r,s,c} x[n, p*stride+r-pad, q*stride+s-pad, c] * w[k,r,s,c] for each (n,p,q,k)."""
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    out = []
    for n, p, q, k in points:
        acc = 0.0
        for r in range(R):
            ih = p * stride + r - pad
            if ih < 0 or ih >= H:
                continue
            for s in range(S):
                iw = q * stride + s - pad
                if iw < 0 or iw >= W:
                    continue
                acc += float(np.dot(x[n, ih, iw, :].astype(np.float64), w[k, r, s, :].astype(np.float64)))
        out.append(acc)
    return np.array(out)


def conv2d_dgrad_points(dy, w, stride, pad, points):
    """dx[n,h,w_,c] = sum over (k,r,s) and the (p,q) with h = p*stride+r-pad, w_ = q*stride+s-pad of
    dy[n,p,q,k] * w[k,r,s,c], for each (n,h,w_,c)."""
    N, P, Q, K = dy.shape
    _, R, S, _ = w.shape
    out = []
    for n, h, ww, c in points:
        acc = 0.0
        for r in range(R):
            t = h + pad - r
            if t % stride or t < 0 or t // stride >= P:
                continue
            for s in range(S):
                u = ww + pad - s
                if u % stride or u < 0 or u // stride >= Q:
                    continue
                acc += float(np.dot(dy[n, t // stride, u // stride, :].astype(np.float64),
                                    w[:, r, s, c].astype(np.float64)))
        out.append(acc)
    return np.array(out)


def conv2d_wgrad_points(dy, x, stride, pad, R, S, points):
    """dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n, p*stride+r-pad, q*stride+s-pad, c] for each (k,r,s,c)."""
    N, P, Q, K = dy.shape
    _, H, W, C = x.shape
    out = []
    for k, r, s, c in points:
        ps = [p for p in range(P) if 0 <= p * stride + r - pad < H]
        qs = [q for q in range(Q) if 0 <= q * stride + s - pad < W]
        if not ps or not qs:
            out.append(0.0)
            continue
        ih = np.array(ps) * stride + r - pad
        iw = np.array(qs) * stride + s - pad
        a = dy[:, ps[0]:ps[-1] + 1, qs[0]:qs[-1] + 1, k].astype(np.float64)
        b = x[:, ih[0]:ih[-1] + 1:stride, iw[0]:iw[-1] + 1:stride, c].astype(np.float64)
        out.append(float((a * b).sum()))
    return np.array(out)


# ---- batch normalisation, training mode -------------------------------------------------

def bn_fwd(x, gamma, beta, eps):
    """y = gamma * (x - mean_c) / sqrt(var_c + eps) + beta with batch statistics over (N,H,W);
    var is the biased (divide-by-m) variance.  Returns y and the cache for the backward."""
    mean = x.mean(axis=(0, 2, 3))
    var = ((x - mean[None, :, None, None]) ** 2).mean(axis=(0, 2, 3))
    invstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mean[None, :, None, None]) * invstd[None, :, None, None]
    y = gamma[None, :, None, None] * xhat + beta[None, :, None, None]
    return y, (xhat, invstd, mean, var)


def bn_running_update(rm, rv, mean, var, m, momentum):
    """running <- (1 - momentum) * running + momentum * stat; the variance fed to the running
    estimate is the unbiased one (m / (m - 1) times the biased batch variance)."""
    unbiased = var * (m / (m - 1.0)) if m > 1 else var
    return (1 - momentum) * rm + momentum * mean, (1 - momentum) * rv + momentum * unbiased


def bn_bwd(dy, cache, gamma):
    """dbeta = sum dy, dgamma = sum dy*xhat, dx = gamma*invstd*(dy - dbeta/m - xhat*dgamma/m)."""
    xhat, invstd, _, _ = cache
    m = dy.shape[0] * dy.shape[2] * dy.shape[3]
    dbeta = dy.sum(axis=(0, 2, 3))
    dgamma = (dy * xhat).sum(axis=(0, 2, 3))
    dx = (gamma * invstd)[None, :, None, None] * (
        dy - dbeta[None, :, None, None] / m - xhat * dgamma[None, :, None, None] / m)
    return dx, dgamma, dbeta


# ---- pooling ----------------------------------------------------------------------------

def maxpool_fwd(x, k=3, stride=2, pad=1):
    """Max over k x k windows, -inf padding; ties resolved to the first maximum in row-major
    window order.  Returns y and the flat argmax (index into H*W) for the backward."""
    N, C, H, W = x.shape
    P, Q = conv_out(H, k, stride, pad), conv_out(W, k, stride, pad)
    xp = np.full((N, C, H + 2 * pad, W + 2 * pad), -np.inf)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    wins = np.empty((k * k, N, C, P, Q))
    for r in range(k):
        for s in range(k):
            wins[r * k + s] = xp[:, :, r:r + stride * P:stride, s:s + stride * Q:stride]
    idx = wins.argmax(axis=0)                      # first maximum
    y = np.take_along_axis(wins, idx[None], axis=0)[0]
    r, s = idx // k, idx % k
    ih = np.arange(P)[None, None, :, None] * stride + r - pad
    iw = np.arange(Q)[None, None, None, :] * stride + s - pad
    return y, (ih * W + iw, (N, C, H, W))


def maxpool_bwd(dy, cache):
    flat, shape = cache
    N, C, H, W = shape
    dx = np.zeros((N, C, H * W))
    n = np.arange(N)[:, None, None, None]
    c = np.arange(C)[None, :, None, None]
    np.add.at(dx, (n, c, flat), dy)
    return dx.reshape(shape)


def avgpool_fwd(x):
    return x.mean(axis=(2, 3))


def avgpool_bwd(dy, x_shape):
    N, C, H, W = x_shape
    return np.broadcast_to(dy[:, :, None, None] / (H * W), x_shape).copy()


# ---- head -------------------------------------------------------------------------------

def fc_fwd(x, w, b):
    return x @ w.T + b[None, :]


def fc_bwd(dz, x, w):
    return dz @ w, dz.T @ x, dz.sum(axis=0)      # dx, dw, db


def softmax_ce(z, labels):
    """L = (1/N) sum_n [logsumexp(z_n) - z_n[label_n]];  dz = (softmax(z) - onehot) / N."""
    N = z.shape[0]
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    se = e.sum(axis=1, keepdims=True)
    lse = np.log(se) + zmax
    loss = float((lse[:, 0] - z[np.arange(N), labels]).sum() / N)
    dz = e / se
    dz[np.arange(N), labels] -= 1.0
    return loss, dz / N
