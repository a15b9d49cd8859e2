"""Pins for the video model of the oracle: the temporal attention layer (frames are the tokens at every spatial
position, placed after each spatial transformer) and the per-frame latent handling of the pipeline.

What fixes it: softmax attention written out with explicit loops on a tiny case, the structural facts of the layer
(it mixes frames but never positions; without a positional term it commutes with a permutation of the frames; on
identical frames the softmax average is the value itself), and the reduction to the image model when the temporal
output projection is zero.
"""
import math

import numpy as np
import pytest

import synthetic_inputs as SI
from configs import CONFIGS
from oracle import primitives as P
from oracle.asyncdiff import Pipeline
from oracle.partition import unit_flops
from oracle.unet import UNetConfig, _temporal, build_units, unet_forward, weight_manifest


@pytest.fixture(scope="module")
def vid():
    cfg = UNetConfig(**CONFIGS["video_tiny"])
    wts = {k: v.astype(np.float64) for k, v in SI.make_weights(weight_manifest(cfg), std=0.2).items()}
    x = SI.make_video_latent(cfg.frames, 4, cfg.height, cfg.width).astype(np.float64)
    ctx = SI.make_text(1, cfg.ctx_len, cfg.ctx_dim).astype(np.float64)
    return cfg, wts, x, ctx


def tfm_unit(cfg, name):
    return next(u for u in build_units(cfg) if u.name == name)


def test_manifest_has_one_temporal_layer_per_spatial_transformer(vid):
    cfg = vid[0]
    names = [n for n, _ in weight_manifest(cfg)]
    tfms = [u.name for u in build_units(cfg) if u.kind == "tfm"]
    assert tfms == ["d0.0.tfm", "mid.tfm", "u0.0.tfm", "u0.1.tfm"]
    for t in tfms:
        assert [n for n in names if n.startswith(t + ".temp.")] == [
            f"{t}.temp.ln.g", f"{t}.temp.ln.b", f"{t}.temp.q.w", f"{t}.temp.k.w", f"{t}.temp.v.w", f"{t}.temp.o.w", f"{t}.temp.o.b"]
    image = dict(CONFIGS["video_tiny"], frames=0, temporal_heads=0, batch=1)
    assert not [n for n, _ in weight_manifest(UNetConfig(**image)) if ".temp." in n]


def test_temporal_layer_brute_force(vid):
    cfg, wts, _, _ = vid
    u = tfm_unit(cfg, "mid.tfm")
    f, c, hh, ww = cfg.frames, 64, 2, 3
    z = np.random.default_rng(5).standard_normal((f, c, hh, ww))
    got = _temporal(cfg, u, wts, z)
    g, b = wts["mid.tfm.temp.ln.g"], wts["mid.tfm.temp.ln.b"]
    wq, wk, wv, wo, bo = (wts[f"mid.tfm.temp.{k}"] for k in ("q.w", "k.w", "v.w", "o.w", "o.b"))
    heads, d = cfg.temporal_heads, c // cfg.temporal_heads
    ref = np.zeros_like(z)
    for y in range(hh):
        for x in range(ww):
            tok = [z[i, :, y, x] for i in range(f)]
            nrm = [(t - t.mean()) / math.sqrt(((t - t.mean()) ** 2).mean() + cfg.ln_eps) * g + b for t in tok]
            q, k, v = ([w @ t for t in nrm] for w in (wq, wk, wv))
            for i in range(f):
                att = np.zeros(c)
                for h in range(heads):
                    sl = slice(h * d, (h + 1) * d)
                    s = [float(q[i][sl] @ k[j][sl]) / math.sqrt(d) for j in range(f)]
                    e = [math.exp(v_ - max(s)) for v_ in s]
                    for j in range(f):
                        att[sl] += e[j] / sum(e) * v[j][sl]
                ref[i, :, y, x] = tok[i] + wo @ att + bo
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)


def test_temporal_layer_mixes_frames_but_not_positions(vid):
    cfg, wts, _, _ = vid
    u = tfm_unit(cfg, "mid.tfm")
    z = np.random.default_rng(6).standard_normal((cfg.frames, 64, 4, 4))
    base = _temporal(cfg, u, wts, z)
    z2 = z.copy()
    z2[1, :, 2, 3] += np.random.default_rng(9).standard_normal(64)      # one frame, one position
    diff = np.abs(_temporal(cfg, u, wts, z2) - base).max(axis=1)        # [frames, H, W]
    mask = np.zeros_like(diff, bool)
    mask[:, 2, 3] = True
    assert (diff[~mask] == 0).all()             # no other position moves
    assert (diff[mask] > 1e-6).all()            # every frame at that position does


def test_temporal_layer_commutes_with_frame_permutation(vid):
    cfg, wts, _, _ = vid
    u = tfm_unit(cfg, "mid.tfm")
    z = np.random.default_rng(7).standard_normal((cfg.frames, 64, 3, 3))
    perm = [2, 0, 1]
    np.testing.assert_allclose(_temporal(cfg, u, wts, z[perm]), _temporal(cfg, u, wts, z)[perm], rtol=1e-12, atol=1e-13)


def test_identical_frames_reduce_to_the_value_path(vid):
    cfg, wts, _, _ = vid
    u = tfm_unit(cfg, "mid.tfm")
    one = np.random.default_rng(8).standard_normal((1, 64, 3, 3))
    z = np.repeat(one, cfg.frames, axis=0)
    t = one.reshape(1, 64, 9).transpose(0, 2, 1)
    y = P.layer_norm(t, wts["mid.tfm.temp.ln.g"], wts["mid.tfm.temp.ln.b"], cfg.ln_eps)
    ref = t + P.linear(P.linear(y, wts["mid.tfm.temp.v.w"]), wts["mid.tfm.temp.o.w"], wts["mid.tfm.temp.o.b"])
    ref = ref.transpose(0, 2, 1).reshape(1, 64, 3, 3)
    got = _temporal(cfg, u, wts, z)
    for i in range(cfg.frames):
        np.testing.assert_allclose(got[i], ref[0], rtol=1e-12, atol=1e-13)


def image_twin(cfg, wts):
    """The image model with the same spatial weights, batch 1."""
    d = dict(CONFIGS["video_tiny"], frames=0, temporal_heads=0, batch=1)
    icfg = UNetConfig(**d)
    return icfg, {k: v for k, v in wts.items() if ".temp." not in k}


def test_zero_temporal_output_gives_the_image_model_per_frame(vid):
    cfg, wts, x, ctx = vid
    z = dict(wts)
    for k in wts:
        if k.endswith(".temp.o.w") or k.endswith(".temp.o.b"):
            z[k] = np.zeros_like(wts[k])
    icfg, iw = image_twin(cfg, wts)
    got = unet_forward(cfg, z, x, 400, ctx)
    assert got.shape == x.shape
    for i in range(cfg.frames):
        np.testing.assert_allclose(got[i], unet_forward(icfg, iw, x[i:i + 1], 400, ctx)[0], rtol=1e-10, atol=1e-12)
    # and with the projection in place the frames do talk to each other
    full = unet_forward(cfg, wts, x, 400, ctx)
    x2 = x.copy()
    x2[0] += 0.5
    assert np.abs(unet_forward(cfg, wts, x2, 400, ctx)[2] - full[2]).max() > 1e-8


def test_video_unet_commutes_with_frame_permutation(vid):
    cfg, wts, x, ctx = vid
    perm = [1, 2, 0]
    np.testing.assert_allclose(unet_forward(cfg, wts, x[perm], 300, ctx), unet_forward(cfg, wts, x, 300, ctx)[perm],
                               rtol=1e-10, atol=1e-12)


def test_video_pipeline_keeps_one_latent_per_frame(vid):
    cfg, wts, x, ctx = vid
    z = dict(wts)
    for k in wts:
        if k.endswith(".temp.o.w") or k.endswith(".temp.o.b"):
            z[k] = np.zeros_like(wts[k])
    icfg, iw = image_twin(cfg, wts)
    pv = Pipeline(cfg, z, N=2, w=1, S=1, T=4, cfg_scale=1.0)
    xs = pv.run(x, ctx)
    assert xs[-1].shape == x.shape
    # same cuts for the image twin (its FLOP balance may differ: the temporal layers carry cost)
    cuts = [r[0] for r in pv.ranges[1:]]
    for i in range(cfg.frames):
        pi = Pipeline(icfg, iw, N=2, w=1, S=1, T=4, cfg_scale=1.0, cuts=cuts)
        np.testing.assert_allclose(xs[-1][i], pi.run(x[i], ctx)[-1], rtol=1e-9, atol=1e-11)
    # the three evaluators agree on the video model too, and N=1 is plain sequential denoising
    full = Pipeline(cfg, wts, N=2, w=1, S=1, T=4, cfg_scale=1.0)
    a, b = full.run(x, ctx, mode="table"), full.run(x, ctx, mode="recursive")
    for u_, v_ in zip(a, b):
        np.testing.assert_array_equal(u_, v_)
    one = Pipeline(cfg, wts, N=1, w=0, S=1, T=4, cfg_scale=1.0)
    for u_, v_ in zip(one.run(x, ctx, mode="table"), one.run(x, ctx, mode="sequential")):
        np.testing.assert_array_equal(u_, v_)


def test_video_flops_by_hand():
    # mid.tfm of the tiny video model: C = 64, L = 4x4 = 16 positions, 3 frames, 8 text tokens of width 32
    cfg = UNetConfig(**CONFIGS["video_tiny"])
    u = next(x for x in build_units(cfg) if x.name == "mid.tfm")
    B, L, C, F, Lk, D = 3, 16, 64, 3, 8, 32
    lin = 2 * B * L * C * C
    spatial = 2 * lin + 4 * lin + 4 * B * L * L * C + 2 * lin + 2 * (2 * 1 * Lk * C * D) + 4 * B * L * Lk * C + 24 * B * L * C * C
    temporal = 4 * lin + 4 * L * F * F * C
    assert spatial == 7_864_320 + 360_448 and temporal == 1_572_864 + 36_864
    assert unit_flops(cfg, u) == spatial + temporal
