"""Profile-guided partition: time every unit of the UNet on the device (each unit run alone as its own
component through ad_component_forward) and split the units into N components of comparable measured time
with the library's own partition rule (ad_balance_cuts).  Section 3.2 of the paper asks for components of
comparable load; FLOPs are the default measure (ad_create), measured time is the better one on a device
whose small layers run far below its peak.  The components of a round share the GPU, so the split that balances
the units' times in isolation is refined by timing whole asynchronous rounds for neighbouring splits."""
import time

import torch

from .binding import AD_BF16, AsyncDiff, balance_cuts


def measure_unit_times(cfg_dict, dtype, weights, device="cuda:0", reps=5):
    """Microseconds per unit (list of ints), one stream, inputs of the right shape filled with noise."""
    probe = AsyncDiff(cfg_dict, 1, 0, 1, dtype)
    nu = len(probe.units())
    probe.close()
    m = AsyncDiff(cfg_dict, nu, 1, 1, dtype, cuts=list(range(1, nu)))
    m.allocate(device)
    m.load_weights(weights)
    m.reset(50)
    tdt = torch.bfloat16 if dtype == AD_BF16 else torch.float32
    frames = cfg_dict.get("frames", 0)           # video model: one latent per frame, one text embedding for all frames
    text = torch.randn(1 if frames else cfg_dict["batch"], cfg_dict["ctx_len"], cfg_dict["ctx_dim"], device=device).to(tdt)
    pooled = torch.randn(cfg_dict["batch"], cfg_dict["pooled_dim"], device=device) if cfg_dict.get("pooled_dim") else None
    latent = torch.randn(max(1, frames), cfg_dict["latent_channels"], cfg_dict["height"], cfg_dict["width"], device=device)

    def alloc(u):
        (b, h, w, c), _ = m.tensor_shape(u)
        if u == nu - 1:
            return torch.zeros(b, c, h, w, device=device)
        return (torch.randn(b, h, w, c, device=device) * 0.5).to(tdt)

    s = torch.cuda.Stream(device=device)
    m.precompute_text(text, s)
    torch.cuda.synchronize()
    out = []
    for comp in range(1, nu + 1):
        ins, outs = m.component_io(comp)
        tin = [latent if u < 0 else alloc(u) for u in ins]
        tout = [alloc(u) for u in outs]
        m.component_forward(comp, tin, 10, text, tout, s, pooled=pooled)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            m.component_forward(comp, tin, 10, text, tout, s, pooled=pooled)
        torch.cuda.synchronize()
        out.append(max(1, int(round((time.perf_counter() - t0) / reps * 1e6))))
    m.close()
    return out


def time_balanced_cuts(cfg_dict, n_components, dtype, weights, device="cuda:0"):
    """Cuts for AsyncDiff(..., cuts=...) that balance the measured unit times; also returns the times."""
    times = measure_unit_times(cfg_dict, dtype, weights, device)
    return balance_cuts(times, n_components), times


def time_rounds(cfg_dict, n_components, warmup, stride, dtype, weights, cuts, device="cuda:0", rounds=12, settle=2, edges=False):
    """Milliseconds per asynchronous round (graph replay, one stream per concurrent evaluation) for a given split;
    edges: in per-edge mode (no barrier between rounds; stride 1)."""
    m = AsyncDiff(cfg_dict, n_components, warmup, stride, dtype, cuts=cuts)
    m.allocate(device)
    m.load_weights(weights)
    m.set_graph_mode(True)
    m.set_edge_mode(bool(edges))
    m.reset(warmup + (settle + rounds + 2) * stride)
    tdt = torch.bfloat16 if dtype == AD_BF16 else torch.float32
    frames = cfg_dict.get("frames", 0)
    text = torch.randn(1 if frames else cfg_dict["batch"], cfg_dict["ctx_len"], cfg_dict["ctx_dim"], device=device).to(tdt)
    pooled = torch.randn(cfg_dict["batch"], cfg_dict["pooled_dim"], device=device) if cfg_dict.get("pooled_dim") else None
    latent = torch.randn(max(1, frames), cfg_dict["latent_channels"], cfg_dict["height"], cfg_dict["width"], device=device)
    if not frames:
        latent = latent[0].contiguous()
    streams = [torch.cuda.Stream(device=device) for _ in range(n_components + stride - 1)]
    torch.cuda.synchronize()
    for _ in range(warmup + settle):
        m.step(latent, text, streams, pooled=pooled)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(rounds):
        m.step(latent, text, streams, pooled=pooled)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / rounds * 1e3
    m.close()
    del m
    torch.cuda.empty_cache()
    return ms


def refine_cuts(cfg_dict, n_components, warmup, stride, dtype, weights, cuts, device="cuda:0", max_evals=40, gain=0.0005, edges=False,
                other_starts=()):
    """Steepest descent around `cuts`: every split with one cut moved by one or two units is timed, the best one is
    taken while the measured round time drops by more than `gain` (relative) and fewer than `max_evals` splits
    have been timed.  other_starts: further splits (the FLOP-balanced one, say) that are timed first; the descent starts
    from the best of them and `cuts`.  Returns (cuts, ms per round, {cuts tuple: ms})."""
    probe = AsyncDiff(cfg_dict, 1, 0, 1, dtype)
    nu = len(probe.units())
    probe.close()
    seen = {}

    def measure(c):
        key = tuple(c)
        if key not in seen:
            # without a barrier the rounds overlap: more of them, and a longer run-in, for a steady figure
            seen[key] = time_rounds(cfg_dict, n_components, warmup, stride, dtype, weights, list(c), device, edges=edges,
                                    rounds=24 if edges else 12, settle=6 if edges else 2)
        return seen[key]

    best = list(cuts)
    best_ms = measure(best)
    for other in other_starts:
        if measure(list(other)) < best_ms:
            best, best_ms = list(other), measure(list(other))
    while len(seen) < max_evals:
        # steepest descent: time every neighbour of the current split (one cut moved by one or two units)
        cand_best, cand_ms = None, best_ms
        for k in range(len(best)):
            for step in (-1, 1, -2, 2):
                cand = list(best)
                cand[k] += step
                bounds = [0] + cand + [nu]
                if any(a >= b for a, b in zip(bounds, bounds[1:])) or (tuple(cand) not in seen and len(seen) >= max_evals):
                    continue
                ms = measure(cand)
                if ms < cand_ms:
                    cand_best, cand_ms = cand, ms
        if cand_best is None or cand_ms > best_ms * (1.0 - gain):
            break
        best, best_ms = cand_best, cand_ms
    return best, best_ms, seen


def pick_stream_placement(model, reset_fn, latent_fn, text, pooled, pool, n_eval, rounds=12, settle=5, max_eval=4):
    """Which stream of `pool` each of the n_eval evaluations of a round should use (evaluation e of a round runs on
    streams[e % len(streams)]).  The hardware queues behind the streams of a process are not equivalent: on the system this
    was written on, two of the four execute like one queue, and the round is up to 15 % slower when the wrong two
    components meet on them (and a few percent faster when the right two do, the last two of the FLOP partition).  Every
    assignment of the evaluations to distinct streams of the pool is timed over a few rounds; returns the fastest as a
    list of streams, and {assignment tuple: ms per round}.  More than max_eval evaluations: the pool in its own order."""
    import itertools
    if n_eval > max_eval or len(pool) < n_eval or n_eval < 2:
        return list(pool[:max(1, n_eval)]), {}
    tried = {}
    for perm in itertools.permutations(range(len(pool)), n_eval):
        streams = [pool[i] for i in perm]
        reset_fn(settle + rounds + 2)
        latent = latent_fn()
        torch.cuda.synchronize()
        for _ in range(model.warmup + settle):
            model.step(latent, text, streams, pooled=pooled)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(rounds):
            model.step(latent, text, streams, pooled=pooled)
        torch.cuda.synchronize()
        tried[perm] = (time.perf_counter() - t0) / rounds * 1e3
    best = min(tried, key=tried.get)
    return [pool[i] for i in best], tried

