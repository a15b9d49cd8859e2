"""Model segmentation: cut the unit list into N contiguous components of near-equal compute.

Section 3.2 asks for components of comparable computational load so that the slowest one,
which sets the cost of a parallel step (Eq. 7), is as small as possible; Appendix A
("Model Segmentation") says the split is sequential.  Reading used here: cost = exact
integer FLOPs (2 per multiply-accumulate) of the convolutions, linear layers and attention
matmuls of a unit; minimise the maximum component cost over all contiguous cuts; among
optimal cuts take the lexicographically smallest vector of cut positions.
"""
from typing import List

from .unet import UNetConfig, Unit, build_units


def unit_flops(cfg: UNetConfig, u: Unit) -> int:
    b = cfg.batch
    conv = lambda ci, co, k, ho, wo: 2 * b * ho * wo * co * ci * k * k
    if u.kind in ("conv_in", "down", "up", "out"):
        return conv(u.c_in, u.c_out, 3, u.h_out, u.w_out)
    if u.kind == "res":
        ci = u.c_in + u.c_skip
        f = conv(ci, u.c_out, 3, u.h_out, u.w_out) + conv(u.c_out, u.c_out, 3, u.h_out, u.w_out)
        f += 2 * b * cfg.temb_dim * u.c_out
        if ci != u.c_out:
            f += conv(ci, u.c_out, 1, u.h_out, u.w_out)
        return f
    if u.kind == "tfm":
        c, l, lk = u.c_in, u.h_in * u.w_in, cfg.ctx_len
        lin = 2 * b * l * c * c
        f = 2 * lin                                   # proj_in, proj_out
        per = 4 * lin + 4 * b * l * l * c             # self: q,k,v,o + QK^T and PV over all heads
        bt = 1 if cfg.frames else b                   # rows of the text embedding (shared by the frames of a video)
        per += 2 * lin + 2 * (2 * bt * lk * c * cfg.ctx_dim) + 4 * b * l * lk * c  # cross
        per += 24 * b * l * c * c                     # GEGLU: C->8C and 4C->C
        f += u.depth * per
        if cfg.temporal_heads:                        # q,k,v,o + QK^T and PV over the frame axis at every position
            f += 4 * lin + 4 * b * l * cfg.frames * c
        return f
    raise ValueError(u.kind)


def unit_score_flops(cfg: UNetConfig, u: Unit) -> int:
    """The part of unit_flops spent in QK^T and PV (module-level MAC counters leave it out)."""
    if u.kind != "tfm":
        return 0
    c, l = u.c_in, u.h_in * u.w_in
    return u.depth * (4 * cfg.batch * l * l * c + 4 * cfg.batch * l * cfg.ctx_len * c)


def partition(costs: List[int], n: int) -> List[int]:
    """Return the N-1 cut positions (component k ends before cuts[k]); minimax, then lexicographic."""
    m = len(costs)
    assert 1 <= n <= m
    pre = [0]
    for c in costs:
        pre.append(pre[-1] + c)
    seg = lambda a, b: pre[b] - pre[a]               # units a..b-1
    inf = float("inf")
    # best[k][i] = minimal max-load splitting units i..m-1 into k parts
    best = [[inf] * (m + 1) for _ in range(n + 1)]
    best[0][m] = 0
    for k in range(1, n + 1):
        for i in range(m - k, -1, -1):
            v = inf
            for e in range(i + 1, m - (k - 1) + 1):
                v = min(v, max(seg(i, e), best[k - 1][e]))
            best[k][i] = v
    opt = best[n][0]
    cuts, i = [], 0
    for k in range(n, 1, -1):
        for e in range(i + 1, m - (k - 1) + 1):
            if seg(i, e) <= opt and best[k - 1][e] <= opt:
                cuts.append(e)
                i = e
                break
    return cuts


def partition_wrapped(costs: List[int], n: int) -> List[int]:
    """Wrapped segmentation (Appendix A, "Model Segmentation": for SDXL the first and the last blocks form one
    segment, the rest is split sequentially).  Reading: the unit list is cut into n+1 contiguous segments; the
    first and the last segment together are component 1, segments 1..n-1 are components 2..n.  Returns the n cut
    positions that minimise the largest component cost; ties -> lexicographically smallest cut vector.
    Exhaustive search (the unit lists here have a few dozen entries)."""
    from itertools import combinations
    m = len(costs)
    assert n >= 2 and n + 1 <= m
    pre = [0]
    for c in costs:
        pre.append(pre[-1] + c)
    best, best_cuts = None, None
    for cuts in combinations(range(1, m), n):
        edges = (0,) + cuts + (m,)
        loads = [pre[edges[k + 1]] - pre[edges[k]] for k in range(n + 1)]
        worst = max([loads[0] + loads[n]] + loads[1:n])
        if best is None or worst < best:          # combinations() come in lexicographic order
            best, best_cuts = worst, list(cuts)
    return best_cuts


def segment_ranges_wrapped(cfg: UNetConfig, n: int, cuts=None):
    """[(first_unit, last_unit)] of the n+1 segments of the wrapped segmentation (segments 0 and n = component 1)."""
    units = build_units(cfg)
    if cuts is None:
        cuts = partition_wrapped([unit_flops(cfg, u) for u in units], n)
    edges = [0] + list(cuts) + [len(units)]
    assert len(cuts) == n and all(a < b for a, b in zip(edges, edges[1:])), "bad cuts"
    return [(edges[k], edges[k + 1] - 1) for k in range(n + 1)]


def component_ranges(cfg: UNetConfig, n: int):
    """[(first_unit, last_unit)] for the N components."""
    units = build_units(cfg)
    cuts = partition([unit_flops(cfg, u) for u in units], n)
    edges = [0] + cuts + [len(units)]
    return [(edges[k], edges[k + 1] - 1) for k in range(n)]
