"""Operator definitions in fp64 numpy (test oracle; not used by the product path).

Each function is the plain mathematical definition of one operator type of the
model DAG (paper Sec. 3.1: a vertex is a DNN operator such as Conv or MaxPool).
The paper does not define the operators' arithmetic (it uses vendor libraries,
Sec. 5.1), so the standard definitions are used; readings where a config is silent
are stated per function.  Inputs and outputs are fp64 arrays; rounding to the
storage type happens in the executor, between operators.
"""
import numpy as np
from scipy.special import erf


def conv2d(x, w, b, stride, pad, relu):
    """Cross-correlation with zero padding, dilation 1, groups 1, floor output size.
    x [Cin,H,W], w [Cout,Cin,kh,kw], b [Cout];
    y[co,oh,ow] = b[co] + sum_{ci,i,j} x[ci, oh*sh+i-ph, ow*sw+j-pw] * w[co,ci,i,j]."""
    cin, h, wd = x.shape
    cout, cin2, kh, kw = w.shape
    assert cin == cin2
    sh, sw = stride
    ph, pw = pad
    ho = (h + 2 * ph - kh) // sh + 1
    wo = (wd + 2 * pw - kw) // sw + 1
    xp = np.zeros((cin, h + 2 * ph, wd + 2 * pw), dtype=np.float64)
    xp[:, ph:ph + h, pw:pw + wd] = x
    y = np.zeros((cout, ho, wo), dtype=np.float64)
    for i in range(kh):
        for j in range(kw):
            patch = xp[:, i:i + sh * (ho - 1) + 1:sh, j:j + sw * (wo - 1) + 1:sw]
            y += np.tensordot(w[:, :, i, j], patch, axes=([1], [0]))
    y += b[:, None, None]
    return np.maximum(y, 0.0) if relu else y


def gemm(x, w, b, extras=(), relu=False):
    """Y = X.W + b (+ sum of extra [M,N] inputs); X [M,K], W [K,N], b [N]."""
    y = x @ w + b[None, :]
    for e in extras:
        y = y + e
    return np.maximum(y, 0.0) if relu else y


def bgemm_qk(q, k, heads, alpha):
    """Per-head scaled scores S_h = alpha * Q_h . K_h^T; q,k [S, heads*d] -> [heads,S,S].
    No mask, no dropout."""
    s, hd = q.shape
    d = hd // heads
    out = np.empty((heads, s, s), dtype=np.float64)
    for h in range(heads):
        out[h] = alpha * (q[:, h * d:(h + 1) * d] @ k[:, h * d:(h + 1) * d].T)
    return out


def bgemm_pv(p, v, heads, alpha=1.0):
    """Per-head context C_h = alpha * P_h . V_h, heads written back side by side:
    p [heads,S,S], v [S, heads*d] -> [S, heads*d]."""
    s, hd = v.shape
    d = hd // heads
    out = np.empty((s, hd), dtype=np.float64)
    for h in range(heads):
        out[:, h * d:(h + 1) * d] = alpha * (p[h] @ v[:, h * d:(h + 1) * d])
    return out


def _windows(x, k, stride, pad, fill):
    c, h, w = x.shape
    kh, kw = k
    sh, sw = stride
    ph, pw = pad
    ho = (h + 2 * ph - kh) // sh + 1
    wo = (w + 2 * pw - kw) // sw + 1
    xp = np.full((c, h + 2 * ph, w + 2 * pw), fill, dtype=np.float64)
    xp[:, ph:ph + h, pw:pw + w] = x
    for i in range(kh):
        for j in range(kw):
            yield xp[:, i:i + sh * (ho - 1) + 1:sh, j:j + sw * (wo - 1) + 1:sw]


def maxpool(x, k, stride, pad):
    """Window maximum, padding acts as -inf, floor output size."""
    y = None
    for win in _windows(x, k, stride, pad, -np.inf):
        y = win.copy() if y is None else np.maximum(y, win)
    return y


def avgpool(x, k, stride, pad):
    """Window mean with zero padding, divisor always kh*kw (padding counted)."""
    y = None
    for win in _windows(x, k, stride, pad, 0.0):
        y = win.copy() if y is None else y + win
    return y / float(k[0] * k[1])


def gavgpool(x):
    """Mean over H x W; [C,H,W] -> [C,1,1]."""
    return x.mean(axis=(1, 2), keepdims=True)


def concat(xs, axis):
    """Join along the channel axis ([C,H,W], axis 0) or the columns ([R,C], axis 1)."""
    return np.concatenate(xs, axis=axis)


def _sum(xs):
    y = xs[0]
    for e in xs[1:]:
        y = y + e
    return y


def layernorm(xs, eps):
    """Row-wise (x-mean)/sqrt(var+eps) with biased variance, gamma=1, beta=0,
    applied to the sum of the inputs."""
    x = _sum(xs)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def softmax(xs):
    """Row-wise softmax over the last axis (max-subtracted) of the sum of the inputs."""
    x = _sum(xs)
    e = np.exp(x - x.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def gelu(xs):
    """Exact (erf) GELU 0.5*x*(1+erf(x/sqrt(2))) of the sum of the inputs."""
    x = _sum(xs)
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def relu(xs):
    return np.maximum(_sum(xs), 0.0)


def add(xs):
    return _sum(xs)
