"""End-to-end oracle: UNet components + partition + asynchronous schedule + sampler.

Glue only; the arithmetic lives in primitives / unet / sampler, the wiring in schedule.
"""
import numpy as np

from . import sampler as SM
from . import schedule as SC
from .partition import component_ranges, segment_ranges_wrapped
from .unet import UNetConfig, build_units, component_io, run_units

F = np.float64


class Pipeline:
    def __init__(self, cfg: UNetConfig, wts, N, w, S, T, sampler="ddim", cfg_scale=7.5,
                 beta_kind="linear", time_shift=False, cuts=None, wrap=False):
        """cuts: optional explicit partition (first unit of components 2..N); default: the FLOP-balanced one.
        wrap: wrapped segmentation (N+1 segments, the first and the last are one component; then `cuts` has N
        entries and the evaluations are numbered 1..N+1, see schedule.py)."""
        self.cfg, self.N, self.w, self.S, self.T = cfg, N, w, S, T
        self.wrap = wrap
        self.wts = {k: np.asarray(v, F) for k, v in wts.items()}
        self.units = build_units(cfg)
        if wrap:
            self.ranges = segment_ranges_wrapped(cfg, N, cuts)
        elif cuts is None:
            self.ranges = component_ranges(cfg, N)
        else:
            edges = [0] + list(cuts) + [len(self.units)]
            assert len(cuts) == N - 1 and all(a < b for a, b in zip(edges, edges[1:])), "bad cuts"
            self.ranges = [(edges[k], edges[k + 1] - 1) for k in range(N)]
        self.sampler, self.cfg_scale, self.time_shift = sampler, cfg_scale, time_shift
        self.taus = SM.timesteps(T)
        self.acp = SM.alphas_cumprod(kind=beta_kind)
        self.rows = SC.build_schedule(T, N, w, S, time_shift, wrap)
        # producer component of every unit, and which components feed which
        self.owner = {}
        for n, (a, b) in enumerate(self.ranges, start=1):
            for i in range(a, b + 1):
                self.owner[i] = n
        self.io = {n: component_io(self.units, a, b) for n, (a, b) in enumerate(self.ranges, start=1)}
        self.feeds = {n: sorted({self.owner[i] for i in self.io[n][0] if i >= 0}) for n in self.io}

    def initial_latent(self, noise):
        noise = np.asarray(noise, F)
        return noise * SM.euler_init_scale(self.taus, self.acp) if self.sampler == "euler" else noise

    def comp_fn(self, ctx, pooled=None):
        def fn(n, stored, x, tau_step):
            a, b = self.ranges[n - 1]
            avail = {}
            for i in self.io[n][0]:
                if i < 0:
                    xin = np.asarray(x, F)
                    if self.sampler == "euler":
                        # the latent's noise level is that of the step it belongs to
                        xin = xin * SM.euler_input_scale(self._latent_step, self.taus, self.acp)
                    # image model: the guidance rows share the latent; video model: one latent per frame
                    avail[-1] = xin.copy() if self.cfg.frames else np.broadcast_to(xin, (self.cfg.batch,) + xin.shape).copy()
                else:
                    avail[i] = stored[self.owner[i]][i]
            return run_units(self.cfg, self.units, a, b, self.wts, avail, self.taus[tau_step], ctx, pooled)
        return fn

    def eps_fn(self, bundle):
        eps = bundle[len(self.units) - 1]
        return np.asarray(eps, F) if self.cfg.frames else SM.cfg_combine(eps, self.cfg_scale)

    def sampler_fn(self, x, eps, i):
        step = SM.ddim_step if self.sampler == "ddim" else SM.euler_step
        return step(x, eps, i, self.taus, self.acp)

    def run(self, noise, ctx, pooled=None, mode="table", trace=None):
        """mode: table (double-buffered table), recursive (definition), sequential (plain loop)."""
        base = self.comp_fn(np.asarray(ctx, F), pooled)

        # component 1 needs to know which latent it was handed (Euler input scaling); the
        # evaluators pass x itself, so recover the step from the row via a small wrapper.
        if mode == "table":
            rows_by_key = {}
            def fn(n, stored, x, tau_step, _rows=iter(self.rows)):
                r = next(_rows)
                assert r.comp == n and r.tau_step == tau_step
                self._latent_step = r.latent_step
                return base(n, stored, x, tau_step)
            return SC.run_table(self.rows, self.feeds, fn, self.eps_fn, self.sampler_fn,
                                self.initial_latent(noise), self.N, trace)
        if self.sampler == "euler":
            raise NotImplementedError("recursive/sequential evaluators are used with DDIM only")
        self._latent_step = 0
        if mode == "recursive":
            return SC.run_recursive(self.T, self.N, self.w, self.S, self.feeds, base, self.eps_fn,
                                    self.sampler_fn, self.initial_latent(noise), self.time_shift, self.wrap)
        if mode == "sequential":
            return SC.run_sequential(self.T, len(self.ranges), self.feeds, base, self.eps_fn, self.sampler_fn,
                                     self.initial_latent(noise))
        raise ValueError(mode)
