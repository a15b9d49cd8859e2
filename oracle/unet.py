"""SD-shaped UNet noise predictor as an ordered list of units, evaluated unit range by unit range.

The paper treats the denoiser as a stack of sequential blocks that is cut into N components
(Section 3.2, Eq. 4; Appendix A "Model Segmentation") and notes that a component may also need
residual (skip) features produced by earlier components (Section 3.2 "Multi-Device
Communication").  This module supplies exactly that view: `build_units` lists the blocks in
execution order with their wiring, `run_units` evaluates a contiguous range given the tensors
it needs from earlier units.  The block definitions are the standard ones (ResBlock,
spatial transformer with self/cross attention and GEGLU, strided-conv downsample,
nearest-2x + conv upsample).
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import primitives as P

F = np.float64


@dataclass
class UNetConfig:
    latent_channels: int = 4
    height: int = 16
    width: int = 16
    batch: int = 1
    channels: List[int] = field(default_factory=lambda: [32, 64])
    layers_per_block: int = 1
    # transformer depth per level (0 = no attention at that level), used for down and up path
    transformer_depth: List[int] = field(default_factory=lambda: [0, 0])
    mid_depth: int = 1
    head_dim: int = 16
    gn_groups: int = 8
    ctx_len: int = 8
    ctx_dim: int = 32
    pooled_dim: int = 0
    # video model: `frames` > 0 makes the batch axis the frame axis (batch == frames, one latent per frame, no
    # guidance, one text embedding shared by all frames); `temporal_heads` > 0 adds a temporal attention layer
    # after every spatial transformer
    frames: int = 0
    temporal_heads: int = 0
    gn_eps: float = 1e-5
    ln_eps: float = 1e-5

    @property
    def temb_dim(self):
        return 4 * self.channels[0]


@dataclass
class Unit:
    kind: str            # conv_in | res | tfm | down | up | out
    name: str
    c_in: int            # channels of the main input
    c_skip: int          # channels of the concatenated skip (res in the up path), else 0
    c_out: int
    h_in: int            # spatial size of the main input
    w_in: int
    h_out: int
    w_out: int
    depth: int = 0       # transformer layers
    skip_from: int = -1  # index of the unit whose output is concatenated, or -1


def build_units(cfg: UNetConfig) -> List[Unit]:
    units: List[Unit] = []
    skips: List[int] = []
    h, w = cfg.height, cfg.width
    ch = cfg.channels
    nl = len(ch)

    def add(u):
        units.append(u)
        return len(units) - 1

    skips.append(add(Unit("conv_in", "conv_in", cfg.latent_channels, 0, ch[0], h, w, h, w)))
    c = ch[0]
    for l in range(nl):
        for j in range(cfg.layers_per_block):
            idx = add(Unit("res", f"d{l}.{j}.res", c, 0, ch[l], h, w, h, w))
            c = ch[l]
            if cfg.transformer_depth[l] > 0:
                idx = add(Unit("tfm", f"d{l}.{j}.tfm", c, 0, c, h, w, h, w, depth=cfg.transformer_depth[l]))
            skips.append(idx)
        if l < nl - 1:
            skips.append(add(Unit("down", f"d{l}.ds", c, 0, c, h, w, h // 2, w // 2)))
            h, w = h // 2, w // 2
    add(Unit("res", "mid.res0", c, 0, c, h, w, h, w))
    if cfg.mid_depth > 0:
        add(Unit("tfm", "mid.tfm", c, 0, c, h, w, h, w, depth=cfg.mid_depth))
    add(Unit("res", "mid.res1", c, 0, c, h, w, h, w))
    for l in range(nl - 1, -1, -1):
        for j in range(cfg.layers_per_block + 1):
            s = skips.pop()
            add(Unit("res", f"u{l}.{j}.res", c, units[s].c_out, ch[l], h, w, h, w, skip_from=s))
            c = ch[l]
            if cfg.transformer_depth[l] > 0:
                add(Unit("tfm", f"u{l}.{j}.tfm", c, 0, c, h, w, h, w, depth=cfg.transformer_depth[l]))
        if l > 0:
            add(Unit("up", f"u{l}.us", c, 0, c, h, w, 2 * h, 2 * w))
            h, w = 2 * h, 2 * w
    assert not skips
    add(Unit("out", "out", c, 0, cfg.latent_channels, h, w, h, w))
    return units


def weight_manifest(cfg: UNetConfig):
    """Canonical (name, shape) list.  Conv weights [O,I,k,k], linear weights [O,I]."""
    m = []
    c0, td = cfg.channels[0], cfg.temb_dim
    m += [("time.lin1.w", (td, c0)), ("time.lin1.b", (td,)), ("time.lin2.w", (td, td)), ("time.lin2.b", (td,))]
    if cfg.pooled_dim:
        pd = cfg.pooled_dim
        m += [("pool.lin1.w", (td, pd)), ("pool.lin1.b", (td,)), ("pool.lin2.w", (td, td)), ("pool.lin2.b", (td,))]
    for u in build_units(cfg):
        n = u.name
        if u.kind in ("conv_in", "down", "up"):
            m += [(f"{n}.conv.w", (u.c_out, u.c_in, 3, 3)), (f"{n}.conv.b", (u.c_out,))]
        elif u.kind == "out":
            m += [(f"{n}.gn.g", (u.c_in,)), (f"{n}.gn.b", (u.c_in,)),
                  (f"{n}.conv.w", (u.c_out, u.c_in, 3, 3)), (f"{n}.conv.b", (u.c_out,))]
        elif u.kind == "res":
            ci = u.c_in + u.c_skip
            m += [(f"{n}.gn1.g", (ci,)), (f"{n}.gn1.b", (ci,)),
                  (f"{n}.conv1.w", (u.c_out, ci, 3, 3)), (f"{n}.conv1.b", (u.c_out,)),
                  (f"{n}.temb.w", (u.c_out, td)), (f"{n}.temb.b", (u.c_out,)),
                  (f"{n}.gn2.g", (u.c_out,)), (f"{n}.gn2.b", (u.c_out,)),
                  (f"{n}.conv2.w", (u.c_out, u.c_out, 3, 3)), (f"{n}.conv2.b", (u.c_out,))]
            if ci != u.c_out:
                m += [(f"{n}.short.w", (u.c_out, ci, 1, 1)), (f"{n}.short.b", (u.c_out,))]
        elif u.kind == "tfm":
            c = u.c_in
            m += [(f"{n}.gn.g", (c,)), (f"{n}.gn.b", (c,)), (f"{n}.proj_in.w", (c, c)), (f"{n}.proj_in.b", (c,))]
            for k in range(u.depth):
                p = f"{n}.{k}"
                m += [(f"{p}.ln1.g", (c,)), (f"{p}.ln1.b", (c,)),
                      (f"{p}.attn1.q.w", (c, c)), (f"{p}.attn1.k.w", (c, c)), (f"{p}.attn1.v.w", (c, c)),
                      (f"{p}.attn1.o.w", (c, c)), (f"{p}.attn1.o.b", (c,)),
                      (f"{p}.ln2.g", (c,)), (f"{p}.ln2.b", (c,)),
                      (f"{p}.attn2.q.w", (c, c)), (f"{p}.attn2.k.w", (c, cfg.ctx_dim)),
                      (f"{p}.attn2.v.w", (c, cfg.ctx_dim)),
                      (f"{p}.attn2.o.w", (c, c)), (f"{p}.attn2.o.b", (c,)),
                      (f"{p}.ln3.g", (c,)), (f"{p}.ln3.b", (c,)),
                      (f"{p}.ff1.w", (8 * c, c)), (f"{p}.ff1.b", (8 * c,)),
                      (f"{p}.ff2.w", (c, 4 * c)), (f"{p}.ff2.b", (c,))]
            m += [(f"{n}.proj_out.w", (c, c)), (f"{n}.proj_out.b", (c,))]
            if cfg.temporal_heads:
                m += [(f"{n}.temp.ln.g", (c,)), (f"{n}.temp.ln.b", (c,)),
                      (f"{n}.temp.q.w", (c, c)), (f"{n}.temp.k.w", (c, c)), (f"{n}.temp.v.w", (c, c)),
                      (f"{n}.temp.o.w", (c, c)), (f"{n}.temp.o.b", (c,))]
    return m


def time_embedding(cfg: UNetConfig, wts, tau, pooled=None):
    """temb[b,:] = Lin2(SiLU(Lin1(sinusoid(tau)))) (+ pooled-embedding MLP when configured)."""
    e = P.timestep_embedding(tau, cfg.channels[0])
    t = P.linear(P.silu(P.linear(e, wts["time.lin1.w"], wts["time.lin1.b"])), wts["time.lin2.w"], wts["time.lin2.b"])
    t = np.broadcast_to(t, (cfg.batch, cfg.temb_dim)).copy()
    if cfg.pooled_dim:
        t = t + P.linear(P.silu(P.linear(np.asarray(pooled, F), wts["pool.lin1.w"], wts["pool.lin1.b"])),
                         wts["pool.lin2.w"], wts["pool.lin2.b"])
    return t


def _res(cfg, u, wts, x, temb):
    n = u.name
    h = P.conv2d(P.silu(P.group_norm(x, cfg.gn_groups, wts[f"{n}.gn1.g"], wts[f"{n}.gn1.b"], cfg.gn_eps)),
                 wts[f"{n}.conv1.w"], wts[f"{n}.conv1.b"])
    h = h + P.linear(P.silu(temb), wts[f"{n}.temb.w"], wts[f"{n}.temb.b"])[:, :, None, None]
    h = P.conv2d(P.silu(P.group_norm(h, cfg.gn_groups, wts[f"{n}.gn2.g"], wts[f"{n}.gn2.b"], cfg.gn_eps)),
                 wts[f"{n}.conv2.w"], wts[f"{n}.conv2.b"])
    if f"{n}.short.w" in wts:
        x = P.conv2d(x, wts[f"{n}.short.w"], wts[f"{n}.short.b"])
    return x + h


def _temporal(cfg, u, wts, z):
    """Temporal attention layer of the video model: at every spatial position the frames are the tokens.
    z: [frames, C, H, W] -> z + Out(MHA_over_frames(LN(z))); no positional term, no feed-forward."""
    n = u.name
    f, c, hh, ww = z.shape
    # [positions, frames, C]: batch = position (copied into that order: matmul on the strided view leaves the BLAS path)
    t = np.ascontiguousarray(z.reshape(f, c, hh * ww).transpose(2, 0, 1))
    y = P.layer_norm(t, wts[f"{n}.temp.ln.g"], wts[f"{n}.temp.ln.b"], cfg.ln_eps)
    a = P.attention(P.linear(y, wts[f"{n}.temp.q.w"]), P.linear(y, wts[f"{n}.temp.k.w"]),
                    P.linear(y, wts[f"{n}.temp.v.w"]), cfg.temporal_heads)
    t = t + P.linear(a, wts[f"{n}.temp.o.w"], wts[f"{n}.temp.o.b"])
    return t.transpose(1, 2, 0).reshape(f, c, hh, ww)


def _tfm(cfg, u, wts, x, ctx):
    n = u.name
    b, c, hh, ww = x.shape
    heads = c // cfg.head_dim
    if ctx.shape[0] != b:                                      # one text embedding shared by all frames
        ctx = np.broadcast_to(ctx, (b,) + ctx.shape[1:])
    h = P.group_norm(x, cfg.gn_groups, wts[f"{n}.gn.g"], wts[f"{n}.gn.b"], cfg.gn_eps)
    h = h.reshape(b, c, hh * ww).transpose(0, 2, 1)            # [B, L, C] tokens
    h = P.linear(h, wts[f"{n}.proj_in.w"], wts[f"{n}.proj_in.b"])
    for k in range(u.depth):
        p = f"{n}.{k}"
        y = P.layer_norm(h, wts[f"{p}.ln1.g"], wts[f"{p}.ln1.b"], cfg.ln_eps)
        a = P.attention(P.linear(y, wts[f"{p}.attn1.q.w"]), P.linear(y, wts[f"{p}.attn1.k.w"]),
                        P.linear(y, wts[f"{p}.attn1.v.w"]), heads)
        h = h + P.linear(a, wts[f"{p}.attn1.o.w"], wts[f"{p}.attn1.o.b"])
        y = P.layer_norm(h, wts[f"{p}.ln2.g"], wts[f"{p}.ln2.b"], cfg.ln_eps)
        a = P.attention(P.linear(y, wts[f"{p}.attn2.q.w"]), P.linear(ctx, wts[f"{p}.attn2.k.w"]),
                        P.linear(ctx, wts[f"{p}.attn2.v.w"]), heads)
        h = h + P.linear(a, wts[f"{p}.attn2.o.w"], wts[f"{p}.attn2.o.b"])
        y = P.layer_norm(h, wts[f"{p}.ln3.g"], wts[f"{p}.ln3.b"], cfg.ln_eps)
        h = h + P.geglu_ff(y, wts[f"{p}.ff1.w"], wts[f"{p}.ff1.b"], wts[f"{p}.ff2.w"], wts[f"{p}.ff2.b"])
    h = P.linear(h, wts[f"{n}.proj_out.w"], wts[f"{n}.proj_out.b"])
    z = x + h.transpose(0, 2, 1).reshape(b, c, hh, ww)
    return _temporal(cfg, u, wts, z) if cfg.temporal_heads else z


def run_unit(cfg, units, i, wts, x, skip, temb, ctx):
    """Evaluate unit i on main input x (NCHW) and optional skip tensor."""
    u = units[i]
    n = u.name
    if u.kind == "conv_in":
        return P.conv2d(x, wts[f"{n}.conv.w"], wts[f"{n}.conv.b"])
    if u.kind == "res":
        if u.skip_from >= 0:
            x = np.concatenate([x, skip], axis=1)
        return _res(cfg, u, wts, x, temb)
    if u.kind == "tfm":
        return _tfm(cfg, u, wts, x, ctx)
    if u.kind == "down":
        return P.conv2d(x, wts[f"{n}.conv.w"], wts[f"{n}.conv.b"], stride=2)
    if u.kind == "up":
        return P.conv2d(P.upsample_nearest2x(x), wts[f"{n}.conv.w"], wts[f"{n}.conv.b"])
    if u.kind == "out":
        return P.conv2d(P.silu(P.group_norm(x, cfg.gn_groups, wts[f"{n}.gn.g"], wts[f"{n}.gn.b"], cfg.gn_eps)),
                        wts[f"{n}.conv.w"], wts[f"{n}.conv.b"])
    raise ValueError(u.kind)


def component_io(units, first, last):
    """Which earlier tensors a unit range [first,last] reads, and which of its tensors later units read.

    Tensors are named by the index of the unit that produces them (-1 = the latent).
    Returns (inputs, outputs), each a sorted list of unit indices; the main hidden state
    (unit first-1, resp. unit last) is always included.
    """
    ins = {first - 1}
    for i in range(first, last + 1):
        s = units[i].skip_from
        if 0 <= s < first:
            ins.add(s)
    outs = {last}
    for i in range(last + 1, len(units)):
        s = units[i].skip_from
        if first <= s <= last:
            outs.add(s)
    return sorted(ins), sorted(outs)


def run_units(cfg, units, first, last, wts, avail, tau, ctx, pooled=None):
    """Evaluate units first..last.  `avail` maps producer index -> tensor for everything read from
    before `first` (key -1 is the model input).  Returns {unit index: tensor} for the range's outputs."""
    temb = time_embedding(cfg, wts, tau, pooled)
    local = dict(avail)
    for i in range(first, last + 1):
        u = units[i]
        skip = local[u.skip_from] if u.skip_from >= 0 else None
        local[i] = run_unit(cfg, units, i, wts, local[i - 1], skip, temb, ctx)
    _, outs = component_io(units, first, last)
    return {i: local[i] for i in outs}


def unet_forward(cfg, wts, x, tau, ctx, pooled=None):
    """Whole noise predictor eps_theta(x, tau): all units in order (Eq. 4 with N = 1)."""
    units = build_units(cfg)
    out = run_units(cfg, units, 0, len(units) - 1, wts, {-1: np.asarray(x, F)}, tau, ctx, pooled)
    return out[len(units) - 1]
