"""Benchmark of the hot path on one MI355X: asynchronous denoising steps per second of the SD2.1-shaped
UNet at 768px (latent 4x96x96, guidance batch 2, N=4 components on 4 HIP streams, bf16).

A step = one parallel round of the schedule: the N component evaluations (each with the inputs stored
by the previous round) plus the sampler update.  Inputs are synthetic and resident in HBM before the
timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


# HBM-side traffic per launch (bytes: fetched + written) of the kernel classes of the sd21_768 workload, from two
# `rocprofv3 --pmc` runs of this file (FETCH_SIZE, WRITE_SIZE; KiB per dispatch scaled by the factors 2.00 and 1.00 that the
# same counters show for the 2^26-element sampler launch).  Commands and tables: profiles/bench_sd21_768_all_kernels.md.
MEASURED_TRAFFIC = {"sd21_768": {
    "igemm_bf16_128x128_p3": 91935451, "igemm_bf16_128x128_dma": 56090270, "igemm_bf16_256x128_p3": 75437418,
    "igemm_bf16_64x64_p3": 25701165, "igemm_bf16_128x128_p3_splitk": 52878129,
    "igemm_bf16_256x128_p3_splitk": 118992536, "splitk_reduce": 18418391, "attn_mfma2_bf16": 33263038,
    "attn_mfma_bf16": 14635399, "gn_apply": 17514426, "gn_partial": 7291156, "layernorm": 13106944,
    "igemm_bf16_64x64_splitk": 51769835, "linear_rows": 5541171, "gn_small": 3033703}}


TRAFFIC_SOURCE = "not measured in this run: FETCH_SIZE + WRITE_SIZE of two rocprofv3 --pmc runs of this file, profiles/bench_sd21_768_all_kernels.md"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


POOLED = None


def run_rounds(m, latent, text, streams, n):
    for _ in range(n):
        if m.step(latent, text, streams, pooled=POOLED) is None:
            raise RuntimeError("schedule exhausted")


def study_saturation(ad, torch, d, r, dtype, wts, dev, cuts, K):
    """One context (N streams, graph replay, barrier rounds) against two independent contexts enqueued alternately on 2N streams.
    The second context's kernels are free to fill whatever the first leaves idle, at round boundaries in particular.  It was
    meant as a bound on what overlap across rounds can gain and gave 1.00-1.02x; the per-edge mode, measured directly, gains
    2.7 % - two contexts also compete for caches and hardware queues, which hides what the filled gaps win."""
    import synthetic_inputs as SI
    N, w, S = r["N"], r["w"], r["S"]
    sampler = ad.AD_DDIM if r["sampler"] == "ddim" else ad.AD_EULER
    tdt = torch.bfloat16 if dtype == ad.AD_BF16 else torch.float32

    def make(seed):
        m = ad.AsyncDiff(d, N, w, S, dtype, cuts=cuts)
        m.allocate(dev); m.load_weights(wts); m.set_graph_mode(True)
        m.reset(w + 8 + 3 * K * S, sampler=sampler, cfg_scale=r["cfg_scale"])
        lat = torch.from_numpy(SI.make_latent(d["latent_channels"], d["height"], d["width"], seed=seed)).to(dev)
        text = torch.from_numpy(SI.make_text(d["batch"], d["ctx_len"], d["ctx_dim"], seed=seed + 1)).to(dev).to(tdt)
        return m, lat, text, [torch.cuda.Stream(device=dev) for _ in range(N + S - 1)]

    A, B2 = make(2000), make(2100)
    for m, lat, text, ss in (A, B2):
        run_rounds(m, lat, text, ss, w + 4)
    torch.cuda.synchronize()

    def timed(ctxs):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            for m, lat, text, ss in ctxs:
                run_rounds(m, lat, text, ss, 1)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / K * 1e3

    one = min(timed([A]), timed([A]))
    two = timed([A, B2])
    out = {"metric": "round time, one context vs two independent contexts side by side (saturation study)", "unit": "ms",
           "config": {"workload": "sd21_768" if d["height"] == 96 else "other", "component_first_units": [a for a, _ in A[0].partition()]},
           "one_context_ms_per_round": round(one, 4), "two_contexts_ms_per_pair": round(two, 4),
           "lower_bound_ms_per_round_with_overlap": round(two / 2, 4), "headroom": round(one / (two / 2), 4)}
    log(f"one context {one:.3f} ms per round; two contexts side by side {two:.3f} ms per pair = {two / 2:.3f} per round; headroom x{one / (two / 2):.3f}")
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", default="sd21_768")
    ap.add_argument("--refine", type=int, default=1, help="with --cuts auto: refine the time-balanced split by timing whole rounds of neighbouring splits")
    ap.add_argument("--streams", type=int, default=0, help="HIP streams for the timed region (0 = one per concurrent evaluation)")
    ap.add_argument("--graphs", type=int, default=1, help="1 (default): replay full asynchronous rounds from HIP graphs; 0: launch every kernel directly")
    ap.add_argument("--cuts", default="flops", help="partition of the units into components for the headline value: 'flops' (default: FLOP-balanced, the "
                    "library default and what the metric configuration names), 'auto' (balanced by unit times measured on this GPU before the "
                    "timed region) or N-1 comma-separated first units of components 2..N")
    ap.add_argument("--tuned", type=int, default=1, help="1 (default, with --cuts flops): after the headline measurement also time the partition balanced by "
                    "measured unit times and refined by whole-round timings, and report it as tuned_partition")
    ap.add_argument("--repeats", type=int, default=10, help="the timed region of --steps rounds is repeated this many times; value is the median")
    ap.add_argument("--edges", type=int, default=-1, help="per-edge mode for the timed region (no barrier between asynchronous rounds: events per producer / "
                    "consumer edge, three copies of the stored tensors; same results bit for bit).  -1 (default): on except with --wrap 1, and the barrier rounds are timed beside it; 0: barrier rounds only; 1: per-edge only")
    ap.add_argument("--place", type=int, default=1, help="1 (default): before a timed region with one stream per concurrent evaluation, time every assignment "
                    "of the evaluations to the streams over a few rounds and use the fastest (the hardware queues behind the streams are "
                    "not equivalent); 0: evaluation e on stream e")
    ap.add_argument("--wrap", type=int, default=0, help="1: wrapped segmentation (first and last segment in one component; stride 1, FLOP-balanced cuts)")
    ap.add_argument("--tile", type=int, default=-1, help="GEMM kernel family override for measurements (ad_tune_conv_tile); -1 = automatic")
    ap.add_argument("--order", type=int, default=-1, help="GEMM workgroup order override for measurements (ad_tune_conv_order); -1 = automatic")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--shapes", action="store_true", help="print the per-shape GEMM/attention timings of the instrumented round to stderr")
    ap.add_argument("--study", default="", help="'saturation': instead of the benchmark, time one context against two independent contexts run side by side "
                    "(twice the streams): what the second context's rounds gain is an upper bound on what any overlap of consecutive rounds of one "
                    "context (per-edge events instead of the round barrier) could gain")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the N components on ONE GPU (separate HIP streams); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2406_06911_amd as ad
    import synthetic_inputs as SI
    from configs import CONFIGS, RUNS

    d, r = CONFIGS[args.config], RUNS[args.config]
    dtype = ad.AD_BF16 if r["dtype"] == "bf16" else ad.AD_F32
    N, w, S = r["N"], r["w"], r["S"]
    if args.wrap:
        S = 1
    K, W = args.steps, args.warmup
    dev = "cuda:0"
    t0 = time.time()
    if args.tile != -1:
        ad.binding.check(ad.lib.ad_tune_conv_tile(args.tile))
    if args.order != -1:
        ad.binding.check(ad.lib.ad_tune_conv_order(args.order))
    probe = ad.AsyncDiff(d, 1, 0, 1, dtype)
    wts = SI.make_weights(probe.weight_manifest(), bf16_exact=(dtype == ad.AD_BF16))
    probe.close()
    if args.study == "saturation":
        study_saturation(ad, torch, d, r, dtype, wts, dev, None if args.cuts in ("flops", "auto") else [int(x) for x in args.cuts.split(",")], K)
        return
    if args.study:
        raise SystemExit("unknown --study")
    unit_us = None
    if args.wrap:
        cuts = None if args.cuts in ("auto", "flops") else [int(x) for x in args.cuts.split(",")]
    elif args.cuts == "auto":
        # components of comparable measured time: every unit is timed alone on this GPU, then split by the library's rule
        from paper_2406_06911_amd.tuning import time_balanced_cuts
        cuts, unit_us = time_balanced_cuts(d, N, dtype, wts, dev) if N > 1 else (None, None)
        log(f"unit times measured in {time.time() - t0:.1f}s; time-balanced cuts {cuts}")
        if N > 1 and args.refine:
            # the components share the GPU: neighbouring splits are timed as whole asynchronous rounds
            from paper_2406_06911_amd.tuning import refine_cuts
            t1 = time.time()
            cuts, ms_round, tried = refine_cuts(d, N, w, S, dtype, wts, cuts, dev, edges=(args.edges == 1 or (args.edges == -1 and not args.wrap)))
            log(f"partition refined in {time.time() - t1:.1f}s over {len(tried)} splits: cuts {cuts}, {ms_round:.3f} ms per round")
            log("  splits tried: " + ", ".join(f"{list(k)}: {v:.3f}" for k, v in tried.items()))
    else:
        cuts = None if args.cuts == "flops" else [int(x) for x in args.cuts.split(",")]
    m = ad.AsyncDiff(d, N, w, S, dtype, cuts=cuts, wrap=bool(args.wrap))
    m.allocate(dev)
    m.load_weights(wts)
    log(f"model ready in {time.time() - t0:.1f}s; arenas {[round(b / 2**20) for b in m.device_bytes()]} MiB")
    tdt = torch.bfloat16 if dtype == ad.AD_BF16 else torch.float32
    frames = d.get("frames", 0)     # video model: one latent per frame, one text embedding for all frames, no guidance
    text = torch.from_numpy(SI.make_text(1 if frames else d["batch"], d["ctx_len"], d["ctx_dim"])).to(dev).to(tdt)
    noise = torch.from_numpy(SI.make_video_latent(frames, d["latent_channels"], d["height"], d["width"]) if frames
                             else SI.make_latent(d["latent_channels"], d["height"], d["width"])).to(dev)
    global POOLED
    POOLED = torch.from_numpy(SI.make_pooled(d["batch"], d["pooled_dim"])).to(dev) if d.get("pooled_dim") else None
    units = m.units()
    flops_step = float(sum(u.flops for u in units))
    sampler = ad.AD_DDIM if r["sampler"] == "ddim" else ad.AD_EULER
    n_par = N + S - 1
    n_streams = args.streams if args.streams > 0 else n_par
    R = max(1, args.repeats)
    T = w + max(W + K * R, min(K, 10) + 2) * S
    if T > 1000:
        R = max(1, (1000 // S - w - W) // K)
        T = w + max(W + K * R, min(K, 10) + 2) * S
        log(f"repeats reduced to {R} so that one schedule (T <= 1000) holds every timed round")

    placement_log = {}

    def timed_rounds(model, graphs, streams, k, reps, edges=False, place=False, tag=""):
        """w warm-up rounds of the method and W untimed rounds, then reps x (exactly k rounds bracketed by device synchronisation).
        place: first choose which stream each evaluation of a round uses by timing every assignment over a few rounds.
        Returns the list of seconds per repetition and the host enqueue time of the first one."""
        model.set_graph_mode(bool(graphs))
        ss = [torch.cuda.Stream(device=dev) for _ in range(streams)]
        if place and streams == n_par:
            from paper_2406_06911_amd.tuning import pick_stream_placement

            def reset_for(nrounds):
                model.reset(w + nrounds * S, sampler=sampler, cfg_scale=r["cfg_scale"])
                model.set_edge_mode(bool(edges))
            t1 = time.time()
            ss, tried = pick_stream_placement(model, reset_for, noise.clone, text, POOLED, ss, n_par)
            if tried:
                best = min(tried, key=tried.get)
                placement_log[tag] = dict(assignment=list(best), ms_per_round=round(tried[best], 3), natural_order_ms=round(tried[tuple(range(n_par))], 3),
                                          worst_ms=round(max(tried.values()), 3), assignments_timed=len(tried), seconds=round(time.time() - t1, 1))
                log(f"stream placement ({tag}): evaluation -> stream {list(best)}, {tried[best]:.3f} ms per round (natural order "
                    f"{tried[tuple(range(n_par))]:.3f}, worst {max(tried.values()):.3f}; {len(tried)} assignments in {time.time() - t1:.1f}s)")
        model.reset(T, sampler=sampler, cfg_scale=r["cfg_scale"])
        model.set_edge_mode(bool(edges))
        lat = noise.clone()
        torch.cuda.synchronize()
        run_rounds(model, lat, text, ss, w + W)
        secs, host = [], None
        for _ in range(reps):
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            run_rounds(model, lat, text, ss, k)
            th = time.perf_counter() - t1
            torch.cuda.synchronize()
            secs.append(time.perf_counter() - t1)
            host = th if host is None else host
        assert bool(torch.isfinite(lat).all()), "latent is not finite"
        return secs, host, lat, ss

    # ---- timed region: concurrent components -----------------------------------------------------
    use_edges = args.edges == 1 or (args.edges == -1 and not args.wrap)     # wrapped segmentation: measured 1 % slower per-edge
    secs, t_host, lat, ss = timed_rounds(m, args.graphs, n_streams, K, R, edges=use_edges, place=bool(args.place), tag="headline")
    sec = float(np.median(secs))
    steps_per_s = K * S / sec
    ms_per_step = sec / (K * S) * 1e3
    spread = dict(repeats=R, timed_seconds=round(float(sum(secs)), 3), ms_per_step_min=round(min(secs) / (K * S) * 1e3, 4),
                  ms_per_step_max=round(max(secs) / (K * S) * 1e3, 4))
    log(f"concurrent ({n_streams} streams{', per-edge mode' if use_edges else ''}): {steps_per_s:.2f} steps/s, {ms_per_step:.3f} ms/step "
        f"(median of {R} x {K} rounds, {spread['ms_per_step_min']:.3f} .. {spread['ms_per_step_max']:.3f})")
    barrier = None
    if use_edges and args.edges == -1:
        # the same rounds with a barrier around every round (the mode of every other configuration), for comparison
        secs_b, host_b, _, _ = timed_rounds(m, args.graphs, n_streams, K, max(1, R // 2), edges=False)
        sec_b = float(np.median(secs_b))
        barrier = dict(steps_per_s=round(K * S / sec_b, 3), ms_per_step=round(sec_b / (K * S) * 1e3, 4), per_edge_over_barrier=round(sec_b / sec, 4),
                       host_enqueue_ms_per_step=round(host_b / (K * S) * 1e3, 3))
        log(f"barrier rounds: {barrier['steps_per_s']:.2f} steps/s ({barrier['per_edge_over_barrier']:.3f}x with per-edge mode)")
    # ---- the same rounds on one stream (sequential UNet with the same kernels): graph replay and direct launches ----
    K2 = min(K, 10)
    R2 = min(R, 5)
    seq = {}
    for mode, graphs in (("graph_replay", 1), ("direct_launches", 0)):
        secs2, _, lat, ss = timed_rounds(m, graphs, 1, K2, R2)
        seq[mode] = K2 * S / float(np.median(secs2))
    seq_steps_per_s = max(seq.values())
    log("one stream: " + ", ".join(f"{k} {v:.2f} steps/s" for k, v in seq.items()))
    m.set_graph_mode(False)
    # ---- per-kernel durations: HIP events around every launch of one more round, one stream ----------
    m.profile(True)
    run_rounds(m, lat, text, ss, 1)
    torch.cuda.synchronize()
    recs = m.profile_records()
    m.profile(False)
    agg = {}
    shapes = {}
    for name, fl, by, ms, mnk in recs:
        if mnk[0]:
            sh = shapes.setdefault((name,) + tuple(mnk), [0, 0.0, 0.0])
            sh[0] += 1; sh[1] += ms; sh[2] += fl
        a = agg.setdefault(name, dict(calls=0, ms=0.0, flops=0.0, bytes=0.0))
        a["calls"] += 1; a["ms"] += ms; a["flops"] += fl; a["bytes"] += by
    kernels = {}
    for name, a in sorted(agg.items(), key=lambda kv: -kv[1]["ms"]):
        e = dict(calls=a["calls"], total_ms=round(a["ms"], 4), avg_us=round(a["ms"] / a["calls"] * 1e3, 2))
        if a["bytes"] > 0:
            e["algorithmic_mb_per_launch"] = round(a["bytes"] / a["calls"] / 1e6, 2)
        if a["flops"] > 0 and name.startswith(("igemm", "attn")):
            e["tflops"] = round(a["flops"] / (a["ms"] * 1e-3) / 1e12, 2)
            e["frac_mfma_peak"] = round(e["tflops"] / PEAK_BF16_TFLOPS, 4)
        elif a["bytes"] > 0:
            e["gbs"] = round(a["bytes"] / (a["ms"] * 1e-3) / 1e9, 1)
            e["frac_hbm_peak"] = round(e["gbs"] / PEAK_HBM_GBS, 4)
        kernels[name] = e
    if args.shapes:
        for key, (cnt, ms, fl) in sorted(shapes.items(), key=lambda kv: -kv[1][1]):
            log(f"{key[0]:22s} M={key[1]:6d} N={key[2]:5d} K={key[3]:6d} calls={cnt:3d} total_ms={ms:8.3f} avg_us={ms / cnt * 1e3:8.1f} TFLOP/s={fl / (ms * 1e-3) / 1e12:7.1f}")
    dom = max(agg.items(), key=lambda kv: kv[1]["ms"])
    dname, da = dom
    if da["flops"] > 0:
        ach = da["flops"] / (da["ms"] * 1e-3) / 1e12
        roofline = dict(kernel=dname, bound="mfma", achieved=round(ach, 2), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                        frac=round(ach / PEAK_BF16_TFLOPS, 4), traffic=MEASURED_TRAFFIC.get(args.config, {}).get(dname), traffic_source=TRAFFIC_SOURCE,
                        launches=da["calls"],
                        avg_launch_us=round(da["ms"] / da["calls"] * 1e3, 2),
                        flops_per_launch=round(da["flops"] / da["calls"]),
                        algorithmic_bytes_per_launch=round(da["bytes"] / da["calls"]))
    else:
        ach = da["bytes"] / (da["ms"] * 1e-3) / 1e9
        roofline = dict(kernel=dname, bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(ach / PEAK_HBM_GBS, 4), traffic=MEASURED_TRAFFIC.get(args.config, {}).get(dname), traffic_source=TRAFFIC_SOURCE,
                        launches=da["calls"],
                        avg_launch_us=round(da["ms"] / da["calls"] * 1e3, 2),
                        bytes_per_launch=round(da["bytes"] / da["calls"]))
    # ---- the sampler kernel at a bandwidth-bound size (same kernel, synthetic size) ---------------------
    n_big = 1 << 26
    xb = torch.randn(n_big, device=dev)
    eb = torch.randn(2, n_big, device=dev)
    import ctypes as C
    s0 = torch.cuda.current_stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for it in range(3):
        if it == 1:
            ev[0].record(s0)
        ad.binding.check(ad.lib.ad_sampler_update_raw(C.c_void_p(xb.data_ptr()), C.c_void_p(eb.data_ptr()), n_big, 2, 1.0, 0.0, 7.5,
                                                      C.c_void_p(s0.cuda_stream)))
    ev[1].record(s0)
    torch.cuda.synchronize()
    samp_ms = ev[0].elapsed_time(ev[1]) / 2
    samp_gbs = n_big * 16 / (samp_ms * 1e-3) / 1e9
    del xb, eb
    # ---- GroupNorm + SiLU (statistics pass + apply pass) at a bandwidth-bound size: 2^26 bf16 elements ----------
    gb, ghw, gc = 2, 512 * 256, 256
    gx = torch.randn(gb, ghw, gc, device=dev).to(torch.bfloat16)
    gy = torch.empty_like(gx)
    gg, gbt = torch.ones(gc, device=dev), torch.zeros(gc, device=dev)
    gscr = torch.zeros(ad.lib.ad_groupnorm_scratch_bytes(gb, ghw, gc), dtype=torch.uint8, device=dev)
    vp = lambda t: C.c_void_p(t.data_ptr())
    for it in range(3):
        if it == 1:
            ev[0].record(s0)
        ad.binding.check(ad.lib.ad_groupnorm_forward(ad.AD_BF16, vp(gx), None, gc, 0, gb, ghw, 32, vp(gg), vp(gbt), 1e-5, 1, vp(gy), vp(gscr),
                                                     C.c_void_p(s0.cuda_stream)))
    ev[1].record(s0)
    torch.cuda.synchronize()
    gn_ms = ev[0].elapsed_time(ev[1]) / 2
    gn_gbs = gx.numel() * 4 / (gn_ms * 1e-3) / 1e9
    del gx, gy, gscr
    # ---- CPU oracle on a bounded sample of the same workload ---------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle.unet import UNetConfig, build_units, run_units, weight_manifest
        from oracle.partition import unit_flops
        ocfg = UNetConfig(**d)
        ounits = build_units(ocfg)
        # bounded sample: the first of four FLOP-balanced components (about a quarter of a step, 10-20 s of CPU time)
        from oracle.partition import component_ranges
        last = component_ranges(ocfg, 4)[0][1] if len(ounits) > 12 else len(ounits) - 1
        prefixes = ("time.", "pool.") + tuple(u.name + "." for u in ounits[:last + 1])
        names = {nm for nm, _ in weight_manifest(ocfg) if nm.startswith(prefixes)}
        sub = [(nm, sh) for nm, sh in weight_manifest(ocfg) if nm in names]
        ow = {k: v.astype(np.float64) for k, v in SI.make_weights(sub).items()}
        if frames:
            xin = SI.make_video_latent(frames, d["latent_channels"], d["height"], d["width"]).astype(np.float64)
        else:
            x = SI.make_latent(d["latent_channels"], d["height"], d["width"]).astype(np.float64)
            xin = np.broadcast_to(x, (d["batch"],) + x.shape).copy()
        ctx = SI.make_text(1 if frames else d["batch"], d["ctx_len"], d["ctx_dim"]).astype(np.float64)
        pooled = SI.make_pooled(d["batch"], d["pooled_dim"]) if d["pooled_dim"] else None
        tc = time.perf_counter()
        run_units(ocfg, ounits, 0, last, ow, {-1: xin}, 500, ctx, pooled)
        cpu_sec = time.perf_counter() - tc
        sample_flops = sum(unit_flops(ocfg, u) for u in ounits[:last + 1])
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        cpu = dict(value=round(1.0 / (cpu_sec * flops_step / sample_flops), 6), unit="steps/s", cores=int(cores),
                   kind=f"oracle: NumPy fp64, its matmul steps run in the BLAS library on {int(cores)} threads; a quarter of a step timed, scaled by FLOPs",
                   sample=f"units {ounits[0].name}..{ounits[last].name} of one UNet forward ({sample_flops / 1e9:.0f} of "
                          f"{flops_step / 1e9:.0f} GFLOP) in {cpu_sec:.1f}s, scaled by FLOPs to a full step",
                   sample_seconds=round(cpu_sec, 2))
    # ---- the same measurement with the partition balanced by measured unit times (profile-guided; a study, not the headline) ----
    tuned = None
    if args.tuned and args.cuts == "flops" and not args.wrap and N > 1:
        from paper_2406_06911_amd.tuning import refine_cuts, time_balanced_cuts
        headline_cuts = [a for a, _ in m.partition()]
        m.close()
        torch.cuda.empty_cache()
        t1 = time.time()
        tcuts, unit_us = time_balanced_cuts(d, N, dtype, wts, dev)
        if args.refine:
            tcuts, _, tried = refine_cuts(d, N, w, S, dtype, wts, tcuts, dev, edges=use_edges, other_starts=[headline_cuts[1:]])
        tune_s = time.time() - t1
        m2 = ad.AsyncDiff(d, N, w, S, dtype, cuts=tcuts)
        m2.allocate(dev)
        m2.load_weights(wts)
        secs_t, _, _, _ = timed_rounds(m2, args.graphs, n_streams, K, R, edges=use_edges, place=bool(args.place), tag="tuned_partition")
        sec_t = float(np.median(secs_t))
        tuned = dict(component_first_units=[a for a, _ in m2.partition()], steps_per_s=round(K * S / sec_t, 3),
                     ms_per_step=round(sec_t / (K * S) * 1e3, 4), over_flops_partition=round(sec / sec_t, 4),
                     tuning_seconds=round(tune_s, 1),
                     note="units timed alone on this GPU, split by the library's rule, refined by timing whole rounds of neighbouring splits")
        log(f"tuned partition {tuned['component_first_units']} (found in {tune_s:.0f}s): {tuned['steps_per_s']:.2f} steps/s vs {steps_per_s:.2f} with FLOP cuts {headline_cuts}")
        part_units = headline_cuts
        m2.close()
    else:
        part_units = [a for a, _ in m.partition()]
    del wts
    out = {
        "metric": "UNet denoising steps/sec, 768px SD2.1-shape N=4, 1 GPU; % bf16 MFMA peak" if args.config == "sd21_768" and not args.wrap
                  else f"UNet denoising steps/sec, {args.config}, N={N}{' wrapped' if args.wrap else ''}, 1 GPU",
        "value": round(steps_per_s, 3), "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dtype == ad.AD_BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.config}: latent {d['latent_channels']}x{d['height']}x{d['width']}, batch {d['batch']} ({'frames' if frames else 'guidance'}), "
                               f"N={N} components on {n_streams} HIP streams, warm-up {w}, stride {S}, {r['sampler']}",
                   "n_components": N, "stride": S, "streams": n_streams, "hip_graphs": bool(args.graphs), "per_edge_mode": bool(use_edges), "partition": ("wrapped, " if args.wrap else "") + (("flops" if args.wrap else args.cuts) if args.cuts in ("auto", "flops") else "given"),
                   "component_first_units": part_units, "flops_per_step": flops_step},
        "timing": spread,
        "component_evals_per_s": round(steps_per_s / S * n_par, 2),
        "sequential_steps_per_s": round(seq_steps_per_s, 3),
        "sequential_one_stream": {k: round(v, 3) for k, v in seq.items()},
        "concurrent_over_sequential": round(steps_per_s / seq_steps_per_s, 4),
        "barrier_rounds": barrier,
        "stream_placement": placement_log or None,
        "tuned_partition": tuned,
        "host_enqueue_ms_per_step": round(t_host / (K * S) * 1e3, 3),
        "mfma_frac_whole_step": round(flops_step / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline,
        "kernels": kernels,
        "sampler_large": {"n": n_big, "gbs": round(samp_gbs, 1), "frac_hbm_peak": round(samp_gbs / PEAK_HBM_GBS, 4),
                          "note": "same kernel on 2^26 latent elements (synthetic size); 16 bytes per element"},
        "gn_large": {"elements": gb * ghw * gc, "gbs": round(gn_gbs, 1), "frac_hbm_peak": round(gn_gbs / PEAK_HBM_GBS, 4), "us": round(gn_ms * 1e3, 1),
                     "note": "GroupNorm(32)+SiLU, statistics pass + apply pass, bf16 [2][131072][256] (synthetic size); 4 bytes per element"},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
