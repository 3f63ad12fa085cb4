"""Layer definitions (forward and hand-derived backward) in float64.

Every function works on one virtual node's rows only: statistics of BatchNorm
are over exactly the rows passed in (Section 4.1: such state is computed by each
pass on its own and never synchronised; Section 3.2: every node is a separate
forward and backward pass).
"""
import numpy as np
from scipy.special import erf


# ---- Linear: y = x W + b --------------------------------------------------------

def linear_fwd(x, W, b=None):
    y = x @ W
    if b is not None:
        y = y + b
    return y


def linear_bwd(x, W, dy, has_bias):
    dW = x.T @ dy
    db = dy.sum(axis=0) if has_bias else None
    dx = dy @ W.T
    return dx, dW, db


# ---- BatchNorm over the rows given (biased variance) -------------------------------

def batchnorm_fwd(z, gamma, beta, eps):
    n = z.shape[0]
    mu = z.sum(axis=0) / n
    var = ((z - mu) ** 2).sum(axis=0) / n
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (z - mu) * rstd
    return gamma * xhat + beta, (xhat, rstd, mu, var)


def batchnorm_bwd(dout, gamma, cache):
    xhat, rstd = cache[:2]
    n = dout.shape[0]
    dgamma = (dout * xhat).sum(axis=0)
    dbeta = dout.sum(axis=0)
    dxhat = dout * gamma
    s1 = dxhat.sum(axis=0)
    s2 = (dxhat * xhat).sum(axis=0)
    dz = (dxhat - s1 / n - xhat * (s2 / n)) * rstd
    return dz, dgamma, dbeta


# ---- LayerNorm over the last axis (biased variance) ----------------------------------

def layernorm_fwd(x, gamma, beta, eps):
    d = x.shape[-1]
    mu = x.sum(axis=-1, keepdims=True) / d
    var = ((x - mu) ** 2).sum(axis=-1, keepdims=True) / d
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return gamma * xhat + beta, (xhat, rstd)


def layernorm_bwd(dout, gamma, cache):
    xhat, rstd = cache
    d = dout.shape[-1]
    lead = tuple(range(dout.ndim - 1))
    dgamma = (dout * xhat).sum(axis=lead)
    dbeta = dout.sum(axis=lead)
    dxhat = dout * gamma
    s1 = dxhat.sum(axis=-1, keepdims=True)
    s2 = (dxhat * xhat).sum(axis=-1, keepdims=True)
    dx = (dxhat - s1 / d - xhat * (s2 / d)) * rstd
    return dx, dgamma, dbeta


# ---- activations --------------------------------------------------------------------

def relu_fwd(x):
    return np.maximum(x, 0.0)


def relu_bwd(dout, x):
    return dout * (x > 0.0)


def gelu_fwd(x):
    """Exact GELU: x * Phi(x) with Phi the standard normal CDF."""
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def gelu_bwd(dout, x):
    cdf = 0.5 * (1.0 + erf(x / np.sqrt(2.0)))
    pdf = np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)
    return dout * (cdf + x * pdf)


# ---- softmax cross-entropy, mean over the rows given ------------------------------------

def softmax_xent_fwd_bwd(logits, labels):
    """Returns (mean loss, dlogits of the mean loss)."""
    n = logits.shape[0]
    zmax = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - zmax)
    denom = e.sum(axis=1, keepdims=True)
    lse = np.log(denom) + zmax
    rows = np.arange(n)
    loss = (lse[:, 0] - logits[rows, labels]).sum() / n
    dlogits = e / denom
    dlogits[rows, labels] -= 1.0
    return loss, dlogits / n


# ---- multi-head self-attention (no mask, no dropout) --------------------------------------

def _identity(a):
    return a


def attention_fwd(q, k, v, operand=_identity):
    """q, k, v: [n_seq, n_heads, T, d_head].  softmax(q k^T / sqrt(d_head)) v.
    `operand` is applied to the probabilities before they enter the product with v
    (identity, or bf16 rounding for bf16 workloads); the returned p is that operand."""
    dh = q.shape[-1]
    s = (q @ np.swapaxes(k, -1, -2)) / np.sqrt(dh)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = operand(p / p.sum(axis=-1, keepdims=True))
    return p @ v, p


def attention_bwd(do, q, k, v, p, operand=_identity):
    """`operand` is applied to the score gradient before its products with k and q."""
    dh = q.shape[-1]
    dv = np.swapaxes(p, -1, -2) @ do
    dp = do @ np.swapaxes(v, -1, -2)
    ds = operand(p * (dp - (dp * p).sum(axis=-1, keepdims=True)))
    dq = (ds @ k) / np.sqrt(dh)
    dk = (np.swapaxes(ds, -1, -2) @ q) / np.sqrt(dh)
    return dq, dk, dv


# ---- 3x3 convolution, stride 1, zero padding 1, NHWC ---------------------------------------
# y[n,h,w,o] = sum_{kh,kw,c} xpad[n, h+kh, w+kw, c] * W[o, kh, kw, c]   (cross-correlation, as
# deep-learning frameworks define "convolution"), xpad = x with one ring of zeros.

def conv3x3_fwd(x, W):
    n, H, Wd, _ = x.shape
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    y = np.zeros((n, H, Wd, W.shape[0]))
    for kh in range(3):
        for kw in range(3):
            y += xp[:, kh:kh + H, kw:kw + Wd, :] @ W[:, kh, kw, :].T
    return y


def conv3x3_bwd(x, W, dy, need_dx=True):
    """(dx, dW) of conv3x3_fwd; dx is None when not needed (first layer)."""
    n, H, Wd, _ = x.shape
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    dW = np.zeros_like(W, dtype=np.float64)
    dxp = np.zeros_like(xp, dtype=np.float64) if need_dx else None
    for kh in range(3):
        for kw in range(3):
            dW[:, kh, kw, :] = np.tensordot(dy, xp[:, kh:kh + H, kw:kw + Wd, :], axes=([0, 1, 2], [0, 1, 2]))
            if need_dx:
                dxp[:, kh:kh + H, kw:kw + Wd, :] += dy @ W[:, kh, kw, :]
    return (dxp[:, 1:-1, 1:-1, :] if need_dx else None), dW
