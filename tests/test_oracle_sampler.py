"""Pins for oracle/sampler.py: closed forms and defining properties of deterministic DDIM."""
import math

import numpy as np

from oracle import sampler as SM

rng = np.random.default_rng(11)


def test_timesteps_and_alphas():
    assert SM.timesteps(10) == [900, 800, 700, 600, 500, 400, 300, 200, 100, 0]
    assert SM.timesteps(50)[:3] == [980, 960, 940] and SM.timesteps(50)[-1] == 0
    a = SM.alphas_cumprod()
    assert len(a) == 1000 and abs(a[0] - (1 - 0.00085)) < 1e-15 and np.all(np.diff(a) < 0)
    # cumulative product of (1 - beta) (Section 3.1), written as a sum of logs
    betas = [0.00085 + (0.012 - 0.00085) * k / 999 for k in range(1000)]
    assert abs(math.log(a[999]) - sum(math.log(1 - b) for b in betas)) < 1e-12
    s = SM.alphas_cumprod(kind="scaled_linear")
    assert abs(s[0] - (1 - 0.00085)) < 1e-15 and s[999] > a[999]


def test_ddim_maps_the_forward_marginal_to_itself():
    """If x = sqrt(a) x0 + sqrt(1-a) e and the model returns e, the step lands on the same form at a'."""
    taus, acp = SM.timesteps(50), SM.alphas_cumprod()
    x0, e = rng.standard_normal((4, 5, 5)), rng.standard_normal((4, 5, 5))
    for i in (0, 7, 48):
        a, a2 = acp[taus[i]], acp[taus[i + 1]]
        x = math.sqrt(a) * x0 + math.sqrt(1 - a) * e
        np.testing.assert_allclose(SM.ddim_step(x, e, i, taus, acp), math.sqrt(a2) * x0 + math.sqrt(1 - a2) * e, atol=1e-13)
    a = acp[taus[49]]
    np.testing.assert_allclose(SM.ddim_step(math.sqrt(a) * x0 + math.sqrt(1 - a) * e, e, 49, taus, acp), x0, atol=1e-13)


def test_ddim_closed_form_for_constant_eps():
    """u = x/sqrt(a) moves by (sigma' - sigma) c each step, so the end point telescopes."""
    T = 50
    taus, acp = SM.timesteps(T), SM.alphas_cumprod()
    x = x_init = rng.standard_normal((4, 6, 6))
    c = rng.standard_normal((4, 6, 6))
    sig = lambda i: math.sqrt((1 - acp[taus[i]]) / acp[taus[i]])
    for i in range(T):
        x = SM.ddim_step(x, c, i, taus, acp)
        if i + 1 < T:
            u = x_init / math.sqrt(acp[taus[0]]) + (sig(i + 1) - sig(0)) * c
            np.testing.assert_allclose(x / math.sqrt(acp[taus[i + 1]]), u, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(x, x_init / math.sqrt(acp[taus[0]]) - sig(0) * c, rtol=1e-11, atol=1e-11)


def test_euler_is_ddim_in_rescaled_coordinates():
    T = 20
    taus, acp = SM.timesteps(T), SM.alphas_cumprod(kind="scaled_linear")
    noise = rng.standard_normal((4, 4, 4))
    xe = noise * SM.euler_init_scale(taus, acp)
    xd = noise.copy()
    for i in range(T):
        e = rng.standard_normal((4, 4, 4))
        # the model sees the same input in both parametrisations
        np.testing.assert_allclose(xe * SM.euler_input_scale(i, taus, acp), xd, rtol=1e-11, atol=1e-12)
        xe = SM.euler_step(xe, e, i, taus, acp)
        xd = SM.ddim_step(xd, e, i, taus, acp)
    np.testing.assert_allclose(xe, xd, rtol=1e-11, atol=1e-12)      # final sigma = 0: same clean sample
    c = rng.standard_normal((4, 4, 4))
    x = x_init = rng.standard_normal((4, 4, 4))
    for i in range(T):
        x = SM.euler_step(x, c, i, taus, acp)
    np.testing.assert_allclose(x, x_init - SM.sigma(0, taus, acp) * c, atol=1e-12)


def test_cfg_combine():
    e = rng.standard_normal((2, 4, 3, 3))
    np.testing.assert_allclose(SM.cfg_combine(e, 1.0), e[0], atol=1e-15)    # scale 1 = conditional branch
    np.testing.assert_allclose(SM.cfg_combine(e, 0.0), e[1], atol=1e-15)    # scale 0 = unconditional branch
    np.testing.assert_allclose(SM.cfg_combine(e, 7.5), 7.5 * e[0] - 6.5 * e[1], atol=1e-13)
    np.testing.assert_array_equal(SM.cfg_combine(e[:1], 7.5), e[0])
