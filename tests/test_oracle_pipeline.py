"""Pins for the glued oracle (oracle/asyncdiff.py) on the tiny configuration."""
import numpy as np
import pytest

import synthetic_inputs as SI
from configs import CONFIGS, RUNS
from oracle.asyncdiff import Pipeline
from oracle.unet import UNetConfig, unet_forward, weight_manifest
from oracle import sampler as SM


@pytest.fixture(scope="module")
def setup():
    cfg = UNetConfig(**CONFIGS["tiny"])
    wts = SI.make_weights(weight_manifest(cfg), std=0.1)
    return cfg, wts, SI.make_latent(4, 16, 16), SI.make_text(1, 8, 32)


def test_three_evaluators_agree(setup):
    cfg, wts, noise, ctx = setup
    for (N, w, S) in [(2, 1, 1), (3, 2, 1), (3, 1, 2)]:
        p = Pipeline(cfg, wts, N=N, w=w, S=S, T=7, cfg_scale=1.0)
        a = p.run(noise, ctx, mode="table")
        b = p.run(noise, ctx, mode="recursive")
        for xa, xb in zip(a, b):
            np.testing.assert_array_equal(xa, xb)


def test_n1_and_full_warmup_reproduce_sequential_denoising(setup):
    cfg, wts, noise, ctx = setup
    T = 6
    taus, acp = SM.timesteps(T), SM.alphas_cumprod()
    x = noise.astype(np.float64)
    w64 = {k: v.astype(np.float64) for k, v in wts.items()}
    ref = [x]
    for i in range(T):                                   # the plain loop of Section 3.2, written out
        eps = unet_forward(cfg, w64, x[None], taus[i], ctx.astype(np.float64))[0]
        x = SM.ddim_step(x, eps, i, taus, acp)
        ref.append(x)
    for (N, w) in [(1, 0), (1, 1), (2, T), (3, T)]:
        got = Pipeline(cfg, wts, N=N, w=w, S=1, T=T, cfg_scale=1.0).run(noise, ctx)
        for a, b in zip(got, ref):
            np.testing.assert_array_equal(a, b)


def test_async_is_an_approximation_that_improves_with_warmup(setup):
    """Section 4.3 / Table 2: more warm-up steps bring the result closer to the original output."""
    cfg, wts, noise, ctx = setup
    T = 10
    seq = Pipeline(cfg, wts, N=1, w=0, S=1, T=T, cfg_scale=1.0).run(noise, ctx)[-1]
    errs = []
    for w in (1, 4, 8):
        x = Pipeline(cfg, wts, N=2, w=w, S=1, T=T, cfg_scale=1.0).run(noise, ctx)[-1]
        errs.append(np.linalg.norm(x - seq) / np.linalg.norm(seq))
    assert errs[0] > errs[1] > errs[2] > 0


def test_euler_and_ddim_pipelines_agree_for_same_schedule(setup):
    cfg, wts, noise, ctx = setup
    a = Pipeline(cfg, wts, N=2, w=1, S=2, T=7, sampler="euler", cfg_scale=1.0).run(noise, ctx)[-1]
    b = Pipeline(cfg, wts, N=2, w=1, S=2, T=7, sampler="ddim", cfg_scale=1.0).run(noise, ctx)[-1]
    np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-10)


def test_wrapped_segmentation_pipeline(setup):
    """Wrapped segmentation on the real (tiny) UNet: table and recursion agree, a warm-up that covers every step is
    sequential denoising bit for bit, and because the tail sees this step's skip features the result differs from
    the sequential segmentation's."""
    cfg, wts, noise, text = setup
    N, T = 2, 6
    p = Pipeline(cfg, wts, N=N, w=1, S=1, T=T, cfg_scale=1.0, wrap=True)
    assert len(p.ranges) == N + 1 and p.ranges[0][0] == 0 and p.ranges[-1][1] == len(p.units) - 1
    a = p.run(noise, text, mode="table")
    b = p.run(noise, text, mode="recursive")
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    seq = Pipeline(cfg, wts, N=1, w=0, S=1, T=T, cfg_scale=1.0).run(noise, text, mode="sequential")
    full = Pipeline(cfg, wts, N=N, w=T, S=1, T=T, cfg_scale=1.0, wrap=True).run(noise, text)
    assert all(np.array_equal(x, y) for x, y in zip(full, seq))
    plain = Pipeline(cfg, wts, N=N, w=1, S=1, T=T, cfg_scale=1.0).run(noise, text)
    assert not np.array_equal(a[-1], plain[-1])
    rel = lambda x, y: np.linalg.norm(x - y) / np.linalg.norm(y)
    assert rel(a[-1], seq[-1]) < 0.5
