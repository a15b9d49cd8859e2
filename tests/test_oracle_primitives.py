"""Pins for oracle/primitives.py: brute force, library routines, invariants, special cases."""
import itertools
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import primitives as P

rng = np.random.default_rng(7)


def brute_conv(x, w, b, stride, pad):
    n, c, h, wd = x.shape
    o, _, k, _ = w.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (wd + 2 * pad - k) // stride + 1
    y = np.zeros((n, o, ho, wo))
    for nn, oo, i, j in itertools.product(range(n), range(o), range(ho), range(wo)):
        acc = b[oo]
        for cc, u, v in itertools.product(range(c), range(k), range(k)):
            ii, jj = i * stride + u - pad, j * stride + v - pad
            if 0 <= ii < h and 0 <= jj < wd:
                acc += w[oo, cc, u, v] * x[nn, cc, ii, jj]
        y[nn, oo, i, j] = acc
    return y


@pytest.mark.parametrize("k,stride,h,w", [(3, 1, 5, 6), (3, 2, 6, 8), (1, 1, 4, 3), (3, 2, 7, 5)])
def test_conv_brute_force_and_library(k, stride, h, w):
    x = rng.standard_normal((2, 3, h, w))
    wt = rng.standard_normal((4, 3, k, k))
    b = rng.standard_normal(4)
    y = P.conv2d(x, wt, b, stride=stride)
    np.testing.assert_allclose(y, brute_conv(x, wt, b, stride, k // 2), rtol=1e-12, atol=1e-12)
    yt = TF.conv2d(torch.from_numpy(x), torch.from_numpy(wt), torch.from_numpy(b), stride=stride, padding=k // 2)
    np.testing.assert_allclose(y, yt.numpy(), rtol=1e-12, atol=1e-12)


def test_conv_delta_kernel_shifts():
    x = rng.standard_normal((1, 2, 6, 6))
    for u, v in itertools.product(range(3), range(3)):
        w = np.zeros((2, 2, 3, 3))
        w[0, 0, u, v] = w[1, 1, u, v] = 1.0
        y = P.conv2d(x, w)
        ref = np.zeros_like(x)
        for i, j in itertools.product(range(6), range(6)):
            ii, jj = i + u - 1, j + v - 1
            if 0 <= ii < 6 and 0 <= jj < 6:
                ref[:, :, i, j] = x[:, :, ii, jj]
        np.testing.assert_array_equal(y, ref)


def test_conv_1x1_is_matmul_and_linear():
    x = rng.standard_normal((2, 5, 4, 4))
    w = rng.standard_normal((3, 5, 1, 1))
    y = P.conv2d(x, w)
    ref = np.einsum("oc,nchw->nohw", w[:, :, 0, 0], x)
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)
    x2 = rng.standard_normal(x.shape)
    w3 = rng.standard_normal((3, 5, 3, 3))
    np.testing.assert_allclose(P.conv2d(2 * x - 3 * x2, w3), 2 * P.conv2d(x, w3) - 3 * P.conv2d(x2, w3), atol=1e-12)


def test_linear_matches_loops():
    x = rng.standard_normal((3, 4))
    w = rng.standard_normal((5, 4))
    b = rng.standard_normal(5)
    ref = np.array([[b[o] + sum(w[o, i] * x[r, i] for i in range(4)) for o in range(5)] for r in range(3)])
    np.testing.assert_allclose(P.linear(x, w, b), ref, rtol=1e-13)


def test_group_norm_invariants_and_library():
    x = rng.standard_normal((2, 8, 5, 5)) * 3 + 1.5
    g, b = np.ones(8), np.zeros(8)
    y = P.group_norm(x, 4, g, b, 1e-5)
    yg = y.reshape(2, 4, -1)
    np.testing.assert_allclose(yg.mean(axis=2), 0, atol=1e-12)
    np.testing.assert_allclose(yg.var(axis=2), 1, atol=1e-4)
    # invariant to a positive affine map of the input (up to eps)
    np.testing.assert_allclose(P.group_norm(2.5 * x + 7, 4, g, b, 1e-12), P.group_norm(x, 4, g, b, 1e-12), atol=1e-9)
    gam, bet = rng.standard_normal(8), rng.standard_normal(8)
    ref = TF.group_norm(torch.from_numpy(x), 4, torch.from_numpy(gam), torch.from_numpy(bet), 1e-5).numpy()
    np.testing.assert_allclose(P.group_norm(x, 4, gam, bet, 1e-5), ref, rtol=1e-11, atol=1e-11)
    # G = C is instance norm
    ref = TF.instance_norm(torch.from_numpy(x), eps=1e-5).numpy()
    np.testing.assert_allclose(P.group_norm(x, 8, g, b, 1e-5), ref, rtol=1e-11, atol=1e-11)
    # G = 1 on a 1x1 map is LayerNorm over channels
    v = rng.standard_normal((3, 8, 1, 1))
    np.testing.assert_allclose(P.group_norm(v, 1, gam, bet, 1e-5)[:, :, 0, 0],
                               P.layer_norm(v[:, :, 0, 0], gam, bet, 1e-5), atol=1e-13)


def test_layer_norm_library():
    x = rng.standard_normal((2, 7, 12))
    g, b = rng.standard_normal(12), rng.standard_normal(12)
    ref = TF.layer_norm(torch.from_numpy(x), (12,), torch.from_numpy(g), torch.from_numpy(b), 1e-5).numpy()
    np.testing.assert_allclose(P.layer_norm(x, g, b, 1e-5), ref, rtol=1e-11, atol=1e-11)


def test_activations():
    x = np.linspace(-6, 6, 41)
    np.testing.assert_allclose(P.silu(x), TF.silu(torch.from_numpy(x)).numpy(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(P.gelu(x), TF.gelu(torch.from_numpy(x)).numpy(), rtol=1e-12, atol=1e-15)
    assert P.silu(np.array([0.0]))[0] == 0.0
    assert abs(P.gelu(np.array([1.0]))[0] - 0.5 * (1 + math.erf(1 / math.sqrt(2)))) < 1e-15
    # GELU(x) - GELU(-x) = x (Phi(x) + Phi(-x) = 1)
    np.testing.assert_allclose(P.gelu(x) - P.gelu(-x), x, atol=1e-14)


def naive_attention(q, k, v, heads):
    bsz, l, c = q.shape
    d = c // heads
    out = np.zeros_like(q)
    for b, h, i in itertools.product(range(bsz), range(heads), range(l)):
        s = [sum(q[b, i, h * d + t] * k[b, j, h * d + t] for t in range(d)) / math.sqrt(d) for j in range(k.shape[1])]
        m = max(s)
        e = [math.exp(a - m) for a in s]
        z = sum(e)
        for t in range(d):
            out[b, i, h * d + t] = sum(e[j] / z * v[b, j, h * d + t] for j in range(len(s)))
    return out


def test_attention_naive_library_and_invariants():
    q = rng.standard_normal((2, 6, 8))
    k = rng.standard_normal((2, 5, 8))
    v = rng.standard_normal((2, 5, 8))
    o = P.attention(q, k, v, heads=2)
    np.testing.assert_allclose(o, naive_attention(q, k, v, 2), rtol=1e-12, atol=1e-13)
    sp = lambda a: torch.from_numpy(a).reshape(2, -1, 2, 4).permute(0, 2, 1, 3)
    ref = TF.scaled_dot_product_attention(sp(q), sp(k), sp(v)).permute(0, 2, 1, 3).reshape(2, 6, 8).numpy()
    np.testing.assert_allclose(o, ref, rtol=1e-11, atol=1e-12)
    # rows of the softmax sum to one
    p = P.softmax_rows(rng.standard_normal((4, 9)) * 30)
    np.testing.assert_allclose(p.sum(axis=-1), 1.0, atol=1e-12)
    # constant V is returned unchanged; a single key returns its value
    vc = np.broadcast_to(rng.standard_normal((1, 1, 8)), (2, 5, 8))
    np.testing.assert_allclose(P.attention(q, k, vc, 2), np.broadcast_to(vc[:, :1], (2, 6, 8)), atol=1e-13)
    np.testing.assert_allclose(P.attention(q, k[:, :1], v[:, :1], 2), np.broadcast_to(v[:, :1], (2, 6, 8)), atol=1e-13)
    # peaky scores: one key dominates
    qq = np.zeros((1, 1, 4)); qq[0, 0, 0] = 100.0
    kk = np.zeros((1, 3, 4)); kk[0, 1, 0] = 1.0
    vv = rng.standard_normal((1, 3, 4))
    np.testing.assert_allclose(P.attention(qq, kk, vv, 1)[0, 0], vv[0, 1], atol=1e-12)


def test_geglu_and_upsample_and_temb():
    x = rng.standard_normal((2, 3, 4))
    w1, b1 = rng.standard_normal((32, 4)), rng.standard_normal(32)
    w2, b2 = rng.standard_normal((4, 16)), rng.standard_normal(4)
    h = x @ w1.T + b1
    ref = (h[..., :16] * TF.gelu(torch.from_numpy(h[..., 16:])).numpy()) @ w2.T + b2
    np.testing.assert_allclose(P.geglu_ff(x, w1, b1, w2, b2), ref, rtol=1e-12)
    a = rng.standard_normal((1, 2, 3, 3))
    up = P.upsample_nearest2x(a)
    assert up.shape == (1, 2, 6, 6)
    for i, j in itertools.product(range(6), range(6)):
        np.testing.assert_array_equal(up[:, :, i, j], a[:, :, i // 2, j // 2])
    np.testing.assert_array_equal(up, TF.interpolate(torch.from_numpy(a), scale_factor=2, mode="nearest").numpy())
    e = P.timestep_embedding(0, 8)
    np.testing.assert_array_equal(e, [1, 1, 1, 1, 0, 0, 0, 0])
    e = P.timestep_embedding(500, 8)
    f = [math.exp(-math.log(10000) * k / 4) for k in range(4)]
    np.testing.assert_allclose(e, [math.cos(500 * a) for a in f] + [math.sin(500 * a) for a in f], rtol=1e-13)
    np.testing.assert_allclose(e[:4] ** 2 + e[4:] ** 2, 1.0, atol=1e-13)
