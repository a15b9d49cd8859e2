"""Sampler S(x_t, eps_t, t) (Section 3.2, first paragraph) and classifier-free guidance.

The printed Eq. 3 is not a consistent DDIM update (its epsilon coefficient mixes alpha_t and
alpha_{t-1} under one square root); the deterministic DDIM step it stands for is
    x' = sqrt(a') * (x - sqrt(1-a) eps) / sqrt(a) + sqrt(1-a') eps,
with a = cumulative product of (1 - beta) (Section 3.1) at the current timestep and a' at the
next one, a' = 1 after the last step.  Euler (discrete) is the same trajectory in the
variable x / sqrt(a):  sigma = sqrt((1-a)/a),  x' = x + (sigma' - sigma) eps.
"""
import numpy as np

F = np.float64


def timesteps(T, train_steps=1000):
    """tau_i for execution-order step i = 0..T-1 ("leading" spacing, no offset)."""
    return [(T - 1 - i) * (train_steps // T) for i in range(T)]


def alphas_cumprod(train_steps=1000, beta_start=0.00085, beta_end=0.012, kind="linear"):
    if kind == "linear":
        betas = np.linspace(beta_start, beta_end, train_steps, dtype=F)
    elif kind == "scaled_linear":
        betas = np.linspace(beta_start ** 0.5, beta_end ** 0.5, train_steps, dtype=F) ** 2
    else:
        raise ValueError(kind)
    return np.cumprod(1.0 - betas)


def cfg_combine(eps, scale):
    """eps rows: 0 = conditional, 1 = unconditional.  A single row passes through."""
    eps = np.asarray(eps, F)
    if eps.shape[0] == 1:
        return eps[0]
    return eps[1] + scale * (eps[0] - eps[1])


def ddim_step(x, eps, i, taus, acp):
    a = acp[taus[i]]
    a2 = acp[taus[i + 1]] if i + 1 < len(taus) else 1.0
    x0 = (np.asarray(x, F) - np.sqrt(1.0 - a) * eps) / np.sqrt(a)
    return np.sqrt(a2) * x0 + np.sqrt(1.0 - a2) * eps


def sigma(i, taus, acp):
    if i >= len(taus):
        return 0.0
    a = acp[taus[i]]
    return float(np.sqrt((1.0 - a) / a))


def euler_step(x, eps, i, taus, acp):
    return np.asarray(x, F) + (sigma(i + 1, taus, acp) - sigma(i, taus, acp)) * eps


def euler_input_scale(i, taus, acp):
    """Factor applied to the latent before it enters the noise predictor."""
    return 1.0 / np.sqrt(sigma(i, taus, acp) ** 2 + 1.0)


def euler_init_scale(taus, acp):
    return float(np.sqrt(sigma(0, taus, acp) ** 2 + 1.0))
