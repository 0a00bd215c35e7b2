"""CPU fp64 oracle: layer forward / backward definitions.  TEST INFRASTRUCTURE ONLY.

Plain numpy float64, one function per layer, written as the textbook definition
of each operation (the paper delegates stage execution to an autograd framework,
Sec. 4 "Implementation"; what a stage computes is FP and BP of its layers,
Sec. 3.2).  A numpy matmul serves as a step where the definition is a sum of
products; there is no tiling, fusion or reordering.  Nothing here is shared with,
or imported by, the HIP library.

Conventions: activations are logical NCHW (or (N,S,D) for token tensors);
x = input, y = output, g = dL/dy.  Every backward returns (dx, [param grads...]).
"""
import math

import numpy as np
from scipy.special import erf as _erf     # library erf (vectorised libm erf)

F = np.float64


# --------------------------------------------------------------------------- conv
def _taps(x, k, stride, pad, ho, wo):
    """Yield (u, v, window) where window[n,c,i,j] = xpad[n,c,i*stride+u, j*stride+v]."""
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    for u in range(k):
        for v in range(k):
            yield u, v, xp[:, :, u:u + stride * (ho - 1) + 1:stride, v:v + stride * (wo - 1) + 1:stride]


def conv2d_fwd(x, w, b, stride, pad, groups):
    """Cross-correlation with zero padding:
    y[n,o,i,j] = b[o] + sum_{c,u,v} w[o,c,u,v] * x[n, grp(o)*cg + c, i*s-p+u, j*s-p+v]."""
    n, cin, h, wd = x.shape
    cout, cg, k, _ = w.shape
    og = cout // groups
    ho = (h + 2 * pad - k) // stride + 1
    wo = (wd + 2 * pad - k) // stride + 1
    y = np.zeros((n, groups, og, ho * wo), F)
    wg = w.reshape(groups, og, cg, k, k)
    for u, v, win in _taps(x, k, stride, pad, ho, wo):
        xs = np.ascontiguousarray(win).reshape(n, groups, cg, ho * wo)
        wt = np.ascontiguousarray(wg[:, :, :, u, v])   # contiguous: lets matmul use the BLAS gemm
        y += np.matmul(wt, xs)                         # (G,og,cg) @ (n,G,cg,P)
    y = y.reshape(n, cout, ho, wo)
    if b is not None:
        y = y + b.reshape(1, cout, 1, 1)
    return y


def conv2d_bwd(x, w, g, stride, pad, groups, has_bias):
    """Adjoints of conv2d_fwd: dx scatters w*g back through each tap;
    dw[o,c,u,v] = sum_{n,i,j} g[n,o,i,j] * x[n, ., i*s-p+u, j*s-p+v]; db[o] = sum g."""
    n, cin, h, wd = x.shape
    cout, cg, k, _ = w.shape
    og = cout // groups
    ho, wo = g.shape[2], g.shape[3]
    wg = w.reshape(groups, og, cg, k, k)
    gg = np.ascontiguousarray(g).reshape(n, groups, og, ho * wo)
    dxp = np.zeros((n, cin, h + 2 * pad, wd + 2 * pad), F)
    dw = np.zeros((groups, og, cg, k, k), F)
    for u, v, win in _taps(x, k, stride, pad, ho, wo):
        xs = np.ascontiguousarray(win).reshape(n, groups, cg, ho * wo)
        dw[:, :, :, u, v] = np.matmul(gg, xs.transpose(0, 1, 3, 2)).sum(axis=0)
        wt = np.ascontiguousarray(wg[:, :, :, u, v])
        dxs = np.matmul(wt.transpose(0, 2, 1), gg)                     # (n,G,cg,P)
        dxp[:, :, u:u + stride * (ho - 1) + 1:stride, v:v + stride * (wo - 1) + 1:stride] += \
            dxs.reshape(n, cin, ho, wo)
    dx = dxp[:, :, pad:pad + h, pad:pad + wd]
    grads = [dw.reshape(w.shape)]
    if has_bias:
        grads.append(g.sum(axis=(0, 2, 3)))
    return np.ascontiguousarray(dx), grads


# --------------------------------------------------------------------------- norms
def batchnorm2d_fwd(x, gamma, beta, eps):
    """Training-mode batch normalisation over (n,h,w) of this micro-batch, biased variance."""
    mu = x.mean(axis=(0, 2, 3), keepdims=True)
    var = ((x - mu) ** 2).mean(axis=(0, 2, 3), keepdims=True)
    istd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * istd
    y = gamma.reshape(1, -1, 1, 1) * xhat + beta.reshape(1, -1, 1, 1)
    return y, (xhat, istd, mu.ravel(), var.ravel())


def batchnorm2d_bwd(g, gamma, xhat, istd):
    """dbeta = sum g; dgamma = sum g*xhat;
    dx = gamma*istd * (g - mean(g) - xhat*mean(g*xhat)), means over (n,h,w)."""
    dbeta = g.sum(axis=(0, 2, 3))
    dgamma = (g * xhat).sum(axis=(0, 2, 3))
    mg = g.mean(axis=(0, 2, 3), keepdims=True)
    mgx = (g * xhat).mean(axis=(0, 2, 3), keepdims=True)
    dx = gamma.reshape(1, -1, 1, 1) * istd * (g - mg - xhat * mgx)
    return dx, [dgamma, dbeta]


def layernorm_fwd(x, gamma, beta, eps):
    """Per-token normalisation over the last dimension, biased variance."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    istd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * istd
    return gamma * xhat + beta, (xhat, istd)


def layernorm_bwd(g, gamma, xhat, istd):
    red = tuple(range(g.ndim - 1))
    dbeta = g.sum(axis=red)
    dgamma = (g * xhat).sum(axis=red)
    gh = g * gamma
    dx = istd * (gh - gh.mean(axis=-1, keepdims=True) - xhat * (gh * xhat).mean(axis=-1, keepdims=True))
    return dx, [dgamma, dbeta]


# --------------------------------------------------------------------------- pointwise
def relu_fwd(x):
    return np.maximum(x, 0.0)


def relu_bwd(g, x):
    return g * (x > 0)


def relu6_fwd(x):
    return np.minimum(np.maximum(x, 0.0), 6.0)


def relu6_bwd(g, x):
    return g * ((x > 0) & (x < 6))


def gelu_fwd(x):
    """x * Phi(x), Phi = standard normal CDF via erf."""
    return x * 0.5 * (1.0 + _erf(x / math.sqrt(2.0)))


def gelu_bwd(g, x):
    """d/dx [x Phi(x)] = Phi(x) + x phi(x)."""
    cdf = 0.5 * (1.0 + _erf(x / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)
    return g * (cdf + x * pdf)


def sigmoid_fwd(x):
    """1 / (1 + exp(-x))."""
    return 1.0 / (1.0 + np.exp(-x))


def sigmoid_bwd(g, x):
    s = sigmoid_fwd(x)
    return g * s * (1.0 - s)


def swish_fwd(x):
    """x * sigmoid(x): the activation of the EfficientNet workload (Sec. 5.1, Table 4)."""
    return x * sigmoid_fwd(x)


def swish_bwd(g, x):
    """d/dx [x s(x)] = s + x s (1 - s)."""
    s = sigmoid_fwd(x)
    return g * (s + x * s * (1.0 - s))


# --------------------------------------------------------------------------- pooling
def global_avgpool_fwd(x):
    return x.mean(axis=(2, 3))


def global_avgpool_bwd(g, h, w):
    return np.broadcast_to(g[:, :, None, None] / (h * w), g.shape + (h, w)).copy()


def maxpool2x2_fwd(x):
    """2x2 window, stride 2; ties resolved to the first maximum in row-major (u,v) order."""
    n, c, h, w = x.shape
    ho, wo = h // 2, w // 2
    win = np.stack([x[:, :, u:2 * ho:2, v:2 * wo:2] for u in range(2) for v in range(2)], axis=-1)
    idx = win.argmax(axis=-1)           # numpy argmax returns the first maximum
    y = np.take_along_axis(win, idx[..., None], axis=-1)[..., 0]
    return y, idx


def maxpool2x2_bwd(g, idx, h, w):
    n, c, ho, wo = g.shape
    dx = np.zeros((n, c, h, w), F)
    for t in range(4):
        u, v = divmod(t, 2)
        dx[:, :, u:2 * ho:2, v:2 * wo:2] += g * (idx == t)
    return dx


def maxpool3x3s2_fwd(x):
    """3x3 window, stride 2, padding 1 (the pooling behind ResNet's stem; padding never wins: it
    counts as minus infinity); ties resolved to the first maximum in row-major (u,v) order."""
    n, c, h, w = x.shape
    ho, wo = (h - 1) // 2 + 1, (w - 1) // 2 + 1
    xp = np.full((n, c, 2 * ho + 1, 2 * wo + 1), -np.inf, F)
    xp[:, :, 1:h + 1, 1:w + 1] = x
    win = np.stack([xp[:, :, u:u + 2 * ho:2, v:v + 2 * wo:2] for u in range(3) for v in range(3)], axis=-1)
    idx = win.argmax(axis=-1)
    y = np.take_along_axis(win, idx[..., None], axis=-1)[..., 0]
    return y, idx


def maxpool3x3s2_bwd(g, idx, h, w):
    n, c, ho, wo = g.shape
    dp = np.zeros((n, c, 2 * ho + 1, 2 * wo + 1), F)
    for t in range(9):
        u, v = divmod(t, 3)
        dp[:, :, u:u + 2 * ho:2, v:v + 2 * wo:2] += g * (idx == t)
    return dp[:, :, 1:h + 1, 1:w + 1]


# --------------------------------------------------------------------------- linear / loss
def linear_fwd(x, w, b):
    y = np.matmul(x, w.T)
    return y + b if b is not None else y


def linear_bwd(x, w, g, has_bias):
    x2 = x.reshape(-1, x.shape[-1])
    g2 = g.reshape(-1, g.shape[-1])
    grads = [np.matmul(g2.T, x2)]
    if has_bias:
        grads.append(g2.sum(axis=0))
    return np.matmul(g, w), grads


def softmax_ce_fwd(z, labels, denom):
    """p = softmax(z) row-wise; loss = (1/denom) * sum_n -log p[n, label_n]."""
    zs = z - z.max(axis=1, keepdims=True)
    e = np.exp(zs)
    p = e / e.sum(axis=1, keepdims=True)
    logp = zs - np.log(e.sum(axis=1, keepdims=True))
    loss = -logp[np.arange(z.shape[0]), labels].sum() / denom
    return loss, p


def softmax_ce_bwd(p, labels, denom):
    dz = p.copy()
    dz[np.arange(p.shape[0]), labels] -= 1.0
    return dz / denom


# --------------------------------------------------------------------------- attention
def mha_fwd(x, w_qkv, b_qkv, w_o, b_o, heads):
    """Multi-head self-attention, no mask, no dropout.
    [Q;K;V] = x W_qkv^T + b_qkv; per head S = Q K^T / sqrt(d); P = softmax_rows(S);
    O = P V; y = concat_heads(O) W_o^T + b_o."""
    n, s, dm = x.shape
    d = dm // heads
    qkv = np.matmul(x, w_qkv.T) + b_qkv
    q, k, v = [qkv[..., i * dm:(i + 1) * dm].reshape(n, s, heads, d).transpose(0, 2, 1, 3)
               for i in range(3)]
    sc = np.matmul(q, k.transpose(0, 1, 3, 2)) / math.sqrt(d)
    sc = sc - sc.max(axis=-1, keepdims=True)
    e = np.exp(sc)
    p = e / e.sum(axis=-1, keepdims=True)
    o = np.matmul(p, v)
    oc = o.transpose(0, 2, 1, 3).reshape(n, s, dm)
    y = np.matmul(oc, w_o.T) + b_o
    return y, (q, k, v, p, oc)


def mha_bwd(x, w_qkv, w_o, g, saved, heads):
    """dV = P^T dO; dP = dO V^T; dS = P*(dP - rowsum(dP*P)); dQ = dS K/sqrt(d);
    dK = dS^T Q/sqrt(d); then linear backward through both projections."""
    q, k, v, p, oc = saved
    n, s, dm = x.shape
    d = dm // heads
    g2 = g.reshape(-1, dm)
    dw_o = np.matmul(g2.T, oc.reshape(-1, dm))
    db_o = g2.sum(axis=0)
    doc = np.matmul(g, w_o)
    do = doc.reshape(n, s, heads, d).transpose(0, 2, 1, 3)
    dv = np.matmul(p.transpose(0, 1, 3, 2), do)
    dp = np.matmul(do, v.transpose(0, 1, 3, 2))
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    dq = np.matmul(ds, k) / math.sqrt(d)
    dk = np.matmul(ds.transpose(0, 1, 3, 2), q) / math.sqrt(d)
    dqkv = np.concatenate([t.transpose(0, 2, 1, 3).reshape(n, s, dm) for t in (dq, dk, dv)], axis=-1)
    d2 = dqkv.reshape(-1, 3 * dm)
    dw_qkv = np.matmul(d2.T, x.reshape(-1, dm))
    db_qkv = d2.sum(axis=0)
    dx = np.matmul(dqkv, w_qkv)
    return dx, [dw_qkv, db_qkv, dw_o, db_o]
