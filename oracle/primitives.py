"""Plain definitions of the UNet building blocks, fp64, NCHW / [batch, tokens, channels].

Each function is the textbook definition written out; a matmul is the only library step.
The paper uses the denoiser as a black box (Section 4.1), so these follow the standard
definitions of the layers a Stable-Diffusion-shaped UNet is made of.
"""
import math

import numpy as np
from scipy.special import erf

F = np.float64


def conv2d(x, w, b=None, stride=1, pad=None):
    """Direct-summation 2-D cross-correlation with zero padding.

    y[n,o,i,j] = b[o] + sum_{c,u,v} w[o,c,u,v] * x[n,c,i*stride+u-pad,j*stride+v-pad]
    x: [N,C,H,W]; w: [O,C,k,k]; pad defaults to k//2.
    """
    x = np.asarray(x, F)
    w = np.asarray(w, F)
    n, c, h, wd = x.shape
    o, c2, k, k2 = w.shape
    assert c == c2 and k == k2
    p = k // 2 if pad is None else pad
    ho = (h + 2 * p - k) // stride + 1
    wo = (wd + 2 * p - k) // stride + 1
    xp = np.zeros((n, c, h + 2 * p, wd + 2 * p), F)
    xp[:, :, p:p + h, p:p + wd] = x
    y = np.zeros((o, n * ho * wo), F)
    for u in range(k):
        for v in range(k):
            xs = xp[:, :, u:u + (ho - 1) * stride + 1:stride, v:v + (wo - 1) * stride + 1:stride]
            # sum over input channels for this tap: [O,C] @ [C, N*Ho*Wo]
            y += np.matmul(np.ascontiguousarray(w[:, :, u, v]), xs.transpose(1, 0, 2, 3).reshape(c, n * ho * wo))
    y = y.reshape(o, n, ho, wo).transpose(1, 0, 2, 3).copy()
    if b is not None:
        y += np.asarray(b, F)[None, :, None, None]
    return y


def linear(x, w, b=None):
    """y[..., o] = b[o] + sum_i w[o,i] * x[..., i]."""
    y = np.matmul(np.asarray(x, F), np.asarray(w, F).T)
    if b is not None:
        y = y + np.asarray(b, F)
    return y


def group_norm(x, groups, gamma, beta, eps):
    """Per (sample, group) mean and biased variance over (C/G, H, W); affine per channel."""
    x = np.asarray(x, F)
    n, c = x.shape[:2]
    assert c % groups == 0
    xg = x.reshape(n, groups, -1)
    mu = xg.mean(axis=2, keepdims=True)
    var = ((xg - mu) ** 2).mean(axis=2, keepdims=True)
    y = ((xg - mu) / np.sqrt(var + eps)).reshape(x.shape)
    shape = (1, c) + (1,) * (x.ndim - 2)
    return y * np.asarray(gamma, F).reshape(shape) + np.asarray(beta, F).reshape(shape)


def layer_norm(x, gamma, beta, eps):
    """Mean / biased variance over the last axis; affine per feature."""
    x = np.asarray(x, F)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(gamma, F) + np.asarray(beta, F)


def silu(x):
    x = np.asarray(x, F)
    return x / (1.0 + np.exp(-x))


def gelu(x):
    """Exact (erf) GELU: x * Phi(x), Phi the standard normal CDF."""
    x = np.asarray(x, F)
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def softmax_rows(s):
    s = np.asarray(s, F)
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attention(q, k, v, heads):
    """Multi-head scaled dot-product attention without mask.

    q: [B,L,C], k,v: [B,Lk,C]; channel c belongs to head c // (C/heads).
    out[b,l,h*d:(h+1)*d] = softmax_row(q_h k_h^T / sqrt(d)) v_h
    """
    q, k, v = (np.asarray(a, F) for a in (q, k, v))
    bsz, l, c = q.shape
    d = c // heads
    assert d * heads == c
    out = np.zeros((bsz, l, c), F)
    for b in range(bsz):
        for h in range(heads):
            sl = slice(h * d, (h + 1) * d)
            p = softmax_rows(np.matmul(q[b, :, sl], k[b, :, sl].T) / math.sqrt(d))
            out[b, :, sl] = np.matmul(p, v[b, :, sl])
    return out


def geglu_ff(x, w1, b1, w2, b2):
    """GEGLU feed-forward: proj C->8C, halves (value, gate), value*GELU(gate), proj 4C->C."""
    h = linear(x, w1, b1)
    half = h.shape[-1] // 2
    return linear(h[..., :half] * gelu(h[..., half:]), w2, b2)


def upsample_nearest2x(x):
    """out[..., i, j] = in[..., i // 2, j // 2]."""
    x = np.asarray(x, F)
    return x.repeat(2, axis=-2).repeat(2, axis=-1)


def timestep_embedding(tau, dim):
    """Sinusoidal embedding [cos(tau f_k) | sin(tau f_k)], f_k = exp(-ln(1e4) k / (dim/2))."""
    half = dim // 2
    k = np.arange(half, dtype=F)
    f = np.exp(-math.log(10000.0) * k / half)
    a = F(tau) * f
    return np.concatenate([np.cos(a), np.sin(a)])
