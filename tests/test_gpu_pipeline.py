"""End-to-end parity: component evaluations and whole asynchronous trajectories against the oracle."""
import numpy as np
import pytest
import torch

import paper_2406_06911_amd as ad
import synthetic_inputs as SI
from configs import CONFIGS, RUNS
from gpu_util import DEV, dev, dev_f32, host, nchw_to_nhwc, nhwc_to_nchw, quantize, rel_l2, tdtype
from oracle.asyncdiff import Pipeline
from oracle.unet import UNetConfig, weight_manifest
from paper_2406_06911_amd import binding as B
from progress import progress

pytestmark = pytest.mark.gpu


class Case:
    """A model instance on the GPU plus the oracle pipeline over the same seeded inputs."""

    def __init__(self, name, dtype, N, w, S, T, sampler="ddim", cfg_scale=1.0, std=0.02, time_shift=False, cuts=None, wrap=False, wts=None):
        d = CONFIGS[name]
        self.d, self.dtype, self.N, self.S, self.T = d, dtype, N, S, T
        ocfg = UNetConfig(**d)
        self.wts = wts if wts is not None else SI.make_weights(weight_manifest(ocfg), std=std, bf16_exact=(dtype == B.AD_BF16))
        frames = d.get("frames", 0)
        # video model: one latent per frame, one text embedding for all frames
        self.noise = (SI.make_video_latent(frames, d["latent_channels"], d["height"], d["width"]) if frames
                      else SI.make_latent(d["latent_channels"], d["height"], d["width"]))
        self.text = quantize(SI.make_text(1 if frames else d["batch"], d["ctx_len"], d["ctx_dim"]), dtype)
        self.pooled = SI.make_pooled(d["batch"], d["pooled_dim"]) if d["pooled_dim"] else None
        self.oracle = Pipeline(ocfg, self.wts, N=N, w=w, S=S, T=T, sampler=sampler, cfg_scale=cfg_scale, time_shift=time_shift, cuts=cuts, wrap=wrap)
        self.m = ad.AsyncDiff(d, N, w, S, dtype, cuts=cuts, wrap=wrap)
        self.m.allocate(DEV)
        self.m.load_weights(self.wts)
        self.m.reset(T, sampler=B.AD_DDIM if sampler == "ddim" else B.AD_EULER, cfg_scale=cfg_scale, time_shift=time_shift)
        self.d_text = dev(self.text, dtype)
        self.d_pooled = dev_f32(self.pooled) if self.pooled is not None else None

    def init_latent(self):
        return dev_f32(self.oracle.initial_latent(self.noise).astype(np.float32))

    def alloc_unit(self, unit):
        (b, h, w, c), nbytes = self.m.tensor_shape(unit)
        nu = len(self.oracle.units)
        if unit == nu - 1:
            return torch.full((b, c, h, w), float("nan"), device=DEV, dtype=torch.float32)
        return torch.full((b, h, w, c), float("nan"), device=DEV, dtype=tdtype(self.dtype))

    def to_nchw(self, unit, t):
        a = host(t)
        return a if unit == len(self.oracle.units) - 1 else nhwc_to_nchw(a)


def run_components_isolated(case, log=None):
    """Per-component parity: every evaluation of the table gets the oracle's own stored inputs and latent
    (rounded to the storage type), so the error measured is that of one component evaluation."""
    m, orc = case.m, case.oracle
    trace = []
    xs = orc.run(case.noise, case.text, case.pooled, trace=trace)
    nu = len(orc.units)
    stream = torch.cuda.current_stream()
    ostore = [dict(), dict()]          # the oracle's stored tensors, by slot and unit
    worst = 0.0
    k = 0
    while k < len(trace):
        rnd = trace[k][0].round
        group = []
        while k < len(trace) and trace[k][0].round == rnd:
            group.append(trace[k]); k += 1
        pending, heads = [], 0
        this_round = {}                    # evaluation -> its oracle bundle of this round (wrapped segmentation)
        for row, obundle in group:
            ins, outs = m.component_io(row.comp)
            this_round[row.comp] = obundle
            hin = []
            for u in ins:
                if u < 0:
                    hin.append(dev_f32(xs[row.latent_step].astype(np.float32)))
                elif row.fresh_from and row.write_slot != row.read_slot and orc.owner[u] == row.fresh_from:
                    hin.append(dev(nchw_to_nhwc(this_round[row.fresh_from][u]), case.dtype))
                else:
                    hin.append(dev(nchw_to_nhwc(ostore[row.read_slot][u]), case.dtype))
            hout = [case.alloc_unit(u) for u in outs]
            lane = 0
            if row.comp == len(orc.ranges):
                lane, heads = heads, heads + 1
            scale = m.sampler_coeffs(row.latent_step)[2] if row.latent_step >= 0 else 1.0
            m.component_forward(row.comp, hin, row.tau_step, case.d_text, hout, stream, lane=lane, latent_scale=scale, pooled=case.d_pooled)
            torch.cuda.synchronize()
            for u, t in zip(outs, hout):
                err = rel_l2(case.to_nchw(u, t), obundle[u])
                worst = max(worst, err)
                if log is not None:
                    log.append((row.round, row.comp, u, err))
                assert err < (1e-4 if case.dtype == B.AD_F32 else 2e-2), f"round {row.round} comp {row.comp} unit {u}: rel L2 {err:.3e}"
                if u != nu - 1 and row.write_slot >= 0:
                    if row.write_slot == row.read_slot:
                        ostore[row.write_slot][u] = obundle[u]
                    else:
                        pending.append((row.write_slot, u, obundle[u]))
        for (slot, u, a) in pending:
            ostore[slot][u] = a
    return worst


def run_steps(case, streams):
    """Whole trajectory through ad_step; returns the final latent (host) and the number of rounds."""
    latent = case.init_latent()
    ss = [torch.cuda.Stream(device=DEV) for _ in range(streams)]
    torch.cuda.synchronize()
    rounds = 0
    while case.m.step(latent, case.d_text, ss, pooled=case.d_pooled) is not None:
        rounds += 1
    torch.cuda.synchronize()
    return host(latent), rounds


def run_components_along_schedule(case, max_rows=None):
    """Drive ad_component_forward row by row exactly as the table says, with test-owned buffers, and
    compare every evaluation's outputs with the oracle's trace of the same table."""
    m, orc = case.m, case.oracle
    trace = []
    orc.run(case.noise, case.text, case.pooled, trace=trace)
    rows = m.schedule()
    assert [tuple(r) for r in rows] == [(r.round, r.comp, r.tau_step, r.read_slot, r.write_slot, r.latent_step, r.eps_step, r.fresh_from)
                                        for r, _ in trace]
    nu = len(orc.units)
    slots = [dict(), dict()]
    latent = case.init_latent()
    stream = torch.cuda.current_stream()
    worst = 0.0
    eps_bufs = {}
    heads_in_round = 0
    last_round = -1
    pending = []
    for idx, (row, (orow, obundle)) in enumerate(zip(rows, trace)):
        if max_rows is not None and idx >= max_rows:
            break
        rnd, comp, tau_step, rd, wr, lat, eps_step, _fresh = row
        if rnd != last_round:
            for (slot, unit, t) in pending:
                slots[slot][unit] = t
            pending, heads_in_round, last_round = [], 0, rnd
        ins, outs = m.component_io(comp)
        hin = [latent if u < 0 else slots[rd][u] for u in ins]
        hout = [case.alloc_unit(u) for u in outs]
        lane = 0
        if comp == case.N:
            lane, heads_in_round = heads_in_round, heads_in_round + 1
        scale = m.sampler_coeffs(lat)[2] if lat >= 0 else 1.0
        m.component_forward(comp, hin, tau_step, case.d_text, hout, stream, lane=lane, latent_scale=scale, pooled=case.d_pooled)
        torch.cuda.synchronize()
        for u, t in zip(outs, hout):
            err = rel_l2(case.to_nchw(u, t), obundle[u])
            worst = max(worst, err)
            assert err < (1e-4 if case.dtype == B.AD_F32 else 2e-2), f"row {idx} comp {comp} unit {u}: rel L2 {err:.3e}"
            if u == nu - 1:
                eps_bufs[eps_step] = t
            elif wr >= 0:
                if wr == rd:
                    slots[wr][u] = t
                else:
                    pending.append((wr, u, t))
        # sampler updates become due when the round's evaluations are done
        last_of_round = idx + 1 == len(rows) or rows[idx + 1][0] != rnd
        if last_of_round:
            for i in sorted(eps_bufs):
                m.ddim_update(latent, eps_bufs[i], i, orc.cfg_scale, stream)
            eps_bufs = {}
            torch.cuda.synchronize()
    return worst, latent


def test_tiny_fp32_components_and_trajectory():
    r = RUNS["tiny"]
    case = Case("tiny", B.AD_F32, r["N"], r["w"], r["S"], r["T"], cfg_scale=r["cfg_scale"])
    worst, latent = run_components_along_schedule(case)
    xs = case.oracle.run(case.noise, case.text)
    assert rel_l2(host(latent), xs[-1]) < 1e-4
    print(f"tiny fp32: worst per-component rel L2 {worst:.2e}, final latent {rel_l2(host(latent), xs[-1]):.2e}")


@pytest.mark.parametrize("N,w,S,sampler,streams", [(2, 1, 1, "ddim", 2), (3, 2, 2, "ddim", 4), (3, 1, 2, "euler", 4), (1, 0, 1, "ddim", 1),
                                                   (4, 2, 3, "ddim", 3)])
def test_tiny_fp32_ad_step_matches_oracle(N, w, S, sampler, streams):
    T = 10
    case = Case("tiny", B.AD_F32, N, w, S, T, sampler=sampler, std=0.1)
    xs = case.oracle.run(case.noise, case.text)
    latent = case.init_latent()
    ss = [torch.cuda.Stream(device=DEV) for _ in range(streams)]
    torch.cuda.synchronize()
    done, rounds = 0, 0
    while True:
        r = case.m.step(latent, case.d_text, ss)
        if r is None:
            break
        done, rounds = r, rounds + 1
        torch.cuda.synchronize()
        assert rel_l2(host(latent), xs[done]) < 1e-4, f"after step {done}"
    assert done == T
    assert rounds == len({r[0] for r in case.m.schedule()})


def test_concurrent_streams_equal_serial_order_bitwise():
    T = 8
    outs = []
    for streams in (1, 4):
        case = Case("tiny", B.AD_F32, 3, 1, 2, T, std=0.1)
        latent = case.init_latent()
        ss = [torch.cuda.Stream(device=DEV) for _ in range(streams)]
        torch.cuda.synchronize()
        while case.m.step(latent, case.d_text, ss) is not None:
            pass
        torch.cuda.synchronize()
        outs.append(latent.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.parametrize("name,dtype,N,w,S,T,sampler,shift", [
    ("tiny", B.AD_F32, 3, 1, 2, 14, "ddim", False),
    ("tiny", B.AD_F32, 2, 2, 1, 9, "euler", True),
    # no warm-up, one component, time shifting: the first round's timestep offset differs from every later round's,
    # so a graph captured in round 0 must not be replayed for round 2
    ("tiny", B.AD_F32, 1, 0, 1, 7, "ddim", True),
    ("tiny", B.AD_F32, 1, 0, 2, 9, "ddim", True),
    ("sd21_narrow", B.AD_BF16, 4, 1, 1, 8, "ddim", False),
])
def test_graph_replay_equals_direct_launch_bitwise(name, dtype, N, w, S, T, sampler, shift):
    """Captured rounds replayed from a HIP graph give the bits of the directly launched rounds, replay after
    replay, with synchronisation and host reads of the latent between the replays; a second run on the same
    context (new table, new latent buffer) re-captures and matches again."""
    case = Case(name, dtype, N, w, S, T, sampler=sampler, cfg_scale=3.0, time_shift=shift, std=0.1 if name == "tiny" else 0.02)
    smp = B.AD_DDIM if sampler == "ddim" else B.AD_EULER

    def trajectory(graphs):
        case.m.set_graph_mode(graphs)
        case.m.reset(T, sampler=smp, cfg_scale=3.0, time_shift=shift)
        latent = case.init_latent()
        ss = [torch.cuda.Stream(device=DEV) for _ in range(N + S - 1)]
        torch.cuda.synchronize()
        snaps = []
        while case.m.step(latent, case.d_text, ss, pooled=case.d_pooled) is not None:
            torch.cuda.synchronize()
            snaps.append(latent.cpu().numpy().copy())
        return snaps

    direct = trajectory(False)
    for attempt in range(2):
        replayed = trajectory(True)
        assert len(replayed) == len(direct)
        for r, (a, b) in enumerate(zip(direct, replayed)):
            assert np.array_equal(a, b), f"run {attempt}, round {r}"
    assert np.isfinite(direct[-1]).all()
    case.m.set_graph_mode(False)


@pytest.mark.parametrize("name,dtype,N,w,S,T,sampler,shift,wrap", [(*p, False) if len(p) == 8 else p for p in [
    ("tiny", B.AD_F32, 2, 1, 1, 9, "ddim", False),
    ("tiny", B.AD_F32, 3, 2, 1, 12, "euler", True),
    ("tiny", B.AD_F32, 4, 1, 1, 14, "ddim", False),
    ("tiny", B.AD_F32, 1, 0, 1, 6, "ddim", True),
    # wrapped segmentation: the tail follows the head of its own round and reads it from the copy being written
    ("tiny", B.AD_F32, 2, 1, 1, 9, "ddim", False, True),
    ("tiny", B.AD_F32, 3, 2, 1, 11, "euler", True, True),
    ("sdxl_narrow", B.AD_BF16, 4, 1, 1, 9, "euler", False, True),
    # stride denoising: the last component is evaluated S times per round on streams of its own; T - w not a multiple
    # of S ends with a partial round, which is a barrier round
    ("tiny", B.AD_F32, 3, 1, 2, 14, "ddim", False),
    ("tiny", B.AD_F32, 2, 2, 3, 16, "euler", True),
    ("tiny", B.AD_F32, 1, 0, 2, 9, "ddim", False),
    ("sd21_narrow", B.AD_BF16, 4, 1, 1, 10, "ddim", False),
    ("sd21_narrow", B.AD_BF16, 3, 2, 1, 9, "ddim", True),
    ("sdxl_narrow", B.AD_BF16, 4, 1, 2, 10, "euler", False),
]])
def test_edge_mode_equals_barrier_rounds_bitwise(name, dtype, N, w, S, T, sampler, shift, wrap):
    """Per-edge mode (no barrier between asynchronous rounds, three copies of the stored tensors, events per
    producer / consumer edge) gives the bits of the barrier rounds: round by round when the caller synchronises
    between rounds, and at the end of a free-running trajectory in which components of different rounds overlap -
    with direct launches and with one replayed graph per (component, copy), on as many streams as components, on two
    and on one."""
    case = Case(name, dtype, N, w, S, T, sampler=sampler, cfg_scale=3.0, time_shift=shift, std=0.1 if name == "tiny" else 0.02, wrap=wrap)
    smp = B.AD_DDIM if sampler == "ddim" else B.AD_EULER
    P = N + S - 1                                          # evaluations that run side by side

    def trajectory(edges, graphs, streams, sync_every_round, profiled_round=-1):
        case.m.set_edge_mode(edges)
        case.m.set_graph_mode(graphs)
        case.m.reset(T, sampler=smp, cfg_scale=3.0, time_shift=shift)
        latent = case.init_latent()
        ss = [torch.cuda.Stream(device=DEV) for _ in range(streams)]
        torch.cuda.synchronize()
        snaps = []
        rounds = 0
        while True:
            # a round with per-launch timing on is enqueued as a barrier round in the middle of the per-edge rounds
            case.m.profile(rounds == profiled_round)
            if case.m.step(latent, case.d_text, ss, pooled=case.d_pooled) is None:
                break
            rounds += 1
            if sync_every_round:
                torch.cuda.synchronize()
                snaps.append(latent.cpu().numpy().copy())
        torch.cuda.synchronize()
        snaps.append(latent.cpu().numpy().copy())
        return snaps

    ref = trajectory(False, False, P, True)
    assert np.isfinite(ref[-1]).all()
    for graphs in (False, True):
        stepwise = trajectory(True, graphs, P, True)
        assert len(stepwise) == len(ref)
        for r, (a, b) in enumerate(zip(ref, stepwise)):
            assert np.array_equal(a, b), f"graphs {graphs}, round {r}"
        for streams in sorted({P, 2, 1}):
            for attempt in range(2):
                free = trajectory(True, graphs, streams, False, profiled_round=w + 2 if attempt else -1)
                assert np.array_equal(free[-1], ref[-1]), f"graphs {graphs}, {streams} streams, free-running, run {attempt}"
    case.m.set_edge_mode(False)
    case.m.set_graph_mode(False)
    # and back: the barrier rounds still give the same bits on the context that has run per-edge rounds
    again = trajectory(False, True, P, False)
    assert np.array_equal(again[-1], ref[-1])
    case.m.set_graph_mode(False)


def test_edge_mode_cannot_change_in_the_middle_of_a_run():
    case = Case("tiny", B.AD_F32, 2, 1, 1, 6, std=0.1)
    latent = case.init_latent()
    ss = [torch.cuda.Stream(device=DEV) for _ in range(2)]
    case.m.step(latent, case.d_text, ss)
    with pytest.raises(ad.AsyncDiffError):
        case.m.set_edge_mode(True)
    torch.cuda.synchronize()
    case.m.reset(6)
    case.m.set_edge_mode(True)          # at the start of a run it may
    case.m.set_edge_mode(False)


@pytest.mark.parametrize("cuts,graphs", [([1, 2], False), ([3, 9], True), ([2], True)])
def test_caller_given_partition_matches_oracle(cuts, graphs):
    """A partition supplied by the caller (for instance one balanced by measured time) changes which tensors are
    stale, so the trajectory differs from the default one; the oracle run with the same cuts must agree."""
    T, N = 9, len(cuts) + 1
    case = Case("tiny", B.AD_F32, N, 1, 1, T, cfg_scale=2.0, std=0.1, cuts=cuts)
    case.m.set_graph_mode(graphs)
    assert [a for a, _ in case.m.partition()][1:] == cuts
    xs = case.oracle.run(case.noise, case.text, mode="table")
    got, rounds = run_steps(case, N)
    assert rel_l2(got, xs[-1]) < 1e-4
    default = Case("tiny", B.AD_F32, N, 1, 1, T, cfg_scale=2.0, std=0.1)
    if [a for a, _ in default.m.partition()][1:] != cuts:
        assert rel_l2(default.oracle.run(default.noise, default.text, mode="table")[-1], xs[-1]) > 1e-6


def test_full_warmup_equals_single_component_bitwise():
    """Warm-up covering every step is plain sequential denoising (Section 3.2): same kernels, same order."""
    T = 5
    outs = []
    for (N, w) in ((1, 0), (3, T)):
        case = Case("tiny", B.AD_F32, N, w, 1, T, std=0.1)
        latent = case.init_latent()
        ss = [torch.cuda.Stream(device=DEV) for _ in range(2)]
        torch.cuda.synchronize()
        while case.m.step(latent, case.d_text, ss) is not None:
            pass
        torch.cuda.synchronize()
        outs.append(latent.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])


def test_narrow_sd_bf16_components():
    """Reduced-width clone of the metric model (same topology, N=4, w=3), bf16: warm-up + two async rounds."""
    r = RUNS["sd21_narrow"]
    case = Case("sd21_narrow", B.AD_BF16, r["N"], r["w"], r["S"], 6, cfg_scale=r["cfg_scale"])
    log = []
    worst = run_components_isolated(case, log)
    xs = case.oracle.run(case.noise, case.text)
    latent, _ = run_steps(case, 4)
    err = rel_l2(latent, xs[-1])
    print(f"narrow bf16: worst per-component rel L2 {worst:.2e}, latent after 6 steps {err:.2e}")
    print("per-evaluation errors:", " ".join(f"r{a}c{b}u{c}:{d:.1e}" for a, b, c, d in log))
    assert err < 5e-2


def test_narrow_sd_bf16_two_components_one_warmup_step():
    """The run parameters of the 512px configuration (N=2, one warm-up step, stride 1, guidance 7.5) on the
    reduced-width clone: per-component parity, then the trajectory through the round driver with graph replay."""
    r = RUNS["sd_512"]
    T = 10
    case = Case("sd21_narrow", B.AD_BF16, r["N"], r["w"], r["S"], T, cfg_scale=r["cfg_scale"])
    worst = run_components_isolated(case)
    xs = case.oracle.run(case.noise, case.text)
    case.m.set_graph_mode(True)
    case.m.reset(T, cfg_scale=r["cfg_scale"])
    latent, rounds = run_steps(case, r["N"])
    err = rel_l2(latent, xs[-1])
    print(f"narrow bf16 N=2 w=1: worst per-component rel L2 {worst:.2e}, latent after {T} steps {err:.2e}")
    assert rounds == T and err < 5e-2


def test_narrow_sd_bf16_full_trajectory():
    """All 50 steps of the reduced-width clone (N=4, w=3, guidance 7.5): final latent within 5e-2."""
    r = RUNS["sd21_narrow"]
    case = Case("sd21_narrow", B.AD_BF16, r["N"], r["w"], r["S"], r["T"], cfg_scale=r["cfg_scale"])
    xs = case.oracle.run(case.noise, case.text)
    latent, rounds = run_steps(case, 4)
    err = rel_l2(latent, xs[-1])
    print(f"narrow bf16 50 steps: final latent rel L2 {err:.2e} after {rounds} rounds")
    assert err < 5e-2


def test_narrow_sdxl_bf16_stride2_euler_pooled():
    """Reduced-width clone of the SDXL-shaped configuration: pooled-embedding branch, transformer depth 1/2, Euler
    sampler, stride 2, N=4, w=3: per-component parity over warm-up and the first rounds, then a short trajectory."""
    r = RUNS["sdxl_narrow"]
    case = Case("sdxl_narrow", B.AD_BF16, r["N"], r["w"], r["S"], 9, sampler=r["sampler"], cfg_scale=r["cfg_scale"])
    log = []
    worst = run_components_isolated(case, log)
    xs = case.oracle.run(case.noise, case.text, case.pooled)
    latent, rounds = run_steps(case, 5)
    err = rel_l2(latent, xs[-1])
    print(f"sdxl narrow bf16: worst per-component rel L2 {worst:.2e}, latent after 9 steps ({rounds} rounds) {err:.2e}")
    assert rounds == len({row[0] for row in case.m.schedule()})
    assert err < 5e-2


def test_time_shift_fp32():
    """Appendix A "Time Shifting": the time embedding lags one step after warm-up; table and arithmetic match the oracle."""
    T = 8
    case = Case("tiny", B.AD_F32, 3, 2, 1, T, std=0.1, time_shift=True)
    xs = case.oracle.run(case.noise, case.text)
    latent, _ = run_steps(case, 3)
    assert rel_l2(latent, xs[-1]) < 1e-4
    plain = Case("tiny", B.AD_F32, 3, 2, 1, T, std=0.1, time_shift=False)
    assert rel_l2(run_steps(plain, 3)[0], xs[-1]) > 1e-3        # the shift really changes the result


def test_state_errors():
    m = ad.AsyncDiff(CONFIGS["tiny"], 2, 1, 1, B.AD_F32)
    m.reset(4)
    x = torch.zeros(4, 16, 16, device=DEV)
    with pytest.raises(ad.AsyncDiffError) as e:
        m.step(x, x, [torch.cuda.current_stream()])
    assert e.value.status == B.AD_ERR_STATE
    m.close()


# ---------------------------------------------------------------------------------------------------
# The metric configuration at full size (768px SD2.1 shape, 866M parameters, N = 4, bf16)
# ---------------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def full_size_weights():
    d = CONFIGS["sd21_768"]
    progress("drawing the weights of sd21_768")
    return SI.make_weights(weight_manifest(UNetConfig(**d)), bf16_exact=True)


def test_full_size_first_units_match_oracle(full_size_weights):
    """One evaluation of the first three units at the real shape (first convolution, ResBlock, transformer block
    with the 9216-token self-attention): the layers that hold the largest GEMMs and the dominant attention
    launch, in the tile / split-K configuration the full-size shapes select.  The oracle computes the same
    units from the same seeded inputs (about 360 GFLOP in fp64)."""
    from oracle.unet import build_units, run_units
    d = CONFIGS["sd21_768"]
    ocfg = UNetConfig(**d)
    units = build_units(ocfg)
    last = 2
    prefixes = tuple(units[i].name + "." for i in range(last + 1)) + ("time.",)
    sub = {k: np.asarray(v, np.float64) for k, v in full_size_weights.items() if k.startswith(prefixes)}
    noise = SI.make_latent(d["latent_channels"], d["height"], d["width"])
    text = quantize(SI.make_text(d["batch"], d["ctx_len"], d["ctx_dim"]), B.AD_BF16)
    taus = __import__("oracle.sampler", fromlist=["timesteps"]).timesteps(50)
    x = np.broadcast_to(noise.astype(np.float64), (d["batch"],) + noise.shape).copy()
    progress("oracle: first three units of sd21_768")
    ref = run_units(ocfg, units, 0, last, sub, {-1: x}, taus[0], text.astype(np.float64), None)

    progress("gpu: loading the weights")
    m = ad.AsyncDiff(d, 4, 3, 1, B.AD_BF16, cuts=[last + 1, 28, 39])
    m.allocate(DEV)
    m.load_weights(full_size_weights)
    m.reset(50)
    ins, outs = m.component_io(1)
    assert ins == [-1] and sorted(ref.keys()) == sorted(outs)
    d_text = dev(text, B.AD_BF16)
    hout = []
    for u in outs:
        (b, h, w, c), _ = m.tensor_shape(u)
        hout.append(torch.full((b, h, w, c), float("nan"), device=DEV, dtype=torch.bfloat16))
    m.component_forward(1, [dev_f32(noise.astype(np.float32))], 0, d_text, hout, torch.cuda.current_stream())
    torch.cuda.synchronize()
    for u, t in zip(outs, hout):
        err = rel_l2(nhwc_to_nchw(host(t)), ref[u])
        assert err < 2e-2, f"unit {u}: rel L2 {err:.3e}"
    m.close()


def test_full_size_bench_configuration_properties(full_size_weights):
    """The launch configuration bench.py times (time-balanced partition, four streams, graph replay) at full
    size: every round gives bit for bit what direct launches on one stream give, the warm-up steps equal plain
    sequential denoising by a single component, and the latent stays finite."""
    d = CONFIGS["sd21_768"]
    T, w = 8, 3
    noise = dev_f32(SI.make_latent(d["latent_channels"], d["height"], d["width"]).astype(np.float32))
    d_text = dev(quantize(SI.make_text(d["batch"], d["ctx_len"], d["ctx_dim"]), B.AD_BF16), B.AD_BF16)

    def trajectory(n, cuts, warm, streams, graphs, rounds=None, edges=False, free_running=False):
        progress(f"gpu: trajectory with {n} component(s) on {streams} stream(s), graphs {graphs}, per-edge {edges}")
        m = ad.AsyncDiff(d, n, warm, 1, B.AD_BF16, cuts=cuts)
        m.allocate(DEV)
        m.load_weights(full_size_weights)
        m.set_graph_mode(graphs)
        m.set_edge_mode(edges)
        m.reset(T, cfg_scale=7.5)
        latent = noise.clone()
        ss = [torch.cuda.Stream(device=DEV) for _ in range(streams)]
        torch.cuda.synchronize()
        snaps = []
        while (rounds is None or len(snaps) < rounds) and m.step(latent, d_text, ss) is not None:
            if not free_running:
                torch.cuda.synchronize()
                snaps.append(latent.cpu().numpy().copy())
        torch.cuda.synchronize()
        if free_running:
            snaps.append(latent.cpu().numpy().copy())
        m.close()
        return snaps

    cuts = [11, 28, 39]
    direct = trajectory(4, cuts, w, 1, False)
    replay = trajectory(4, cuts, w, 4, True)
    assert len(direct) == len(replay) == T
    for r, (a, b) in enumerate(zip(direct, replay)):
        assert np.array_equal(a, b), f"round {r}"
    assert np.isfinite(replay[-1]).all()
    # per-edge mode (what bench.py times by default): no barrier between rounds, same bits - round by round, and at the end
    # of a run in which nothing synchronises and components of different rounds overlap
    edge = trajectory(4, cuts, w, 4, True, edges=True)
    assert len(edge) == T
    for r, (a, b) in enumerate(zip(direct, edge)):
        assert np.array_equal(a, b), f"per-edge round {r}"
    free = trajectory(4, cuts, w, 4, True, edges=True, free_running=True)
    assert np.array_equal(free[-1], direct[-1])
    single = trajectory(1, None, 0, 1, False, rounds=w)
    for r in range(w):
        assert np.array_equal(single[r], direct[r]), f"warm-up step {r}"
    # the asynchronous steps differ from sequential denoising (stale inputs), but only slightly (Section 3.2)
    full = trajectory(1, None, 0, 1, False)
    dev_async = rel_l2(direct[-1], full[-1])
    assert 0 < dev_async < 0.2, dev_async


# ---------------------------------------------------------------------------------------------------
# Wrapped segmentation (Appendix A "Model Segmentation": first and last segment in one component)
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,w,graphs,streams,shift", [(2, 1, False, 2, False), (3, 2, True, 3, False), (3, 1, False, 2, True), (4, 1, True, 4, False)])
def test_wrapped_tiny_fp32_matches_oracle(N, w, graphs, streams, shift):
    T = 9
    case = Case("tiny", B.AD_F32, N, w, 1, T, cfg_scale=2.0, std=0.1, wrap=True, time_shift=shift)
    case.m.set_graph_mode(graphs)
    assert case.m.partition() == case.oracle.ranges
    worst = run_components_isolated(case)
    xs = case.oracle.run(case.noise, case.text)
    case.m.reset(T, cfg_scale=2.0, time_shift=shift)
    latent = case.init_latent()
    ss = [torch.cuda.Stream(device=DEV) for _ in range(streams)]
    torch.cuda.synchronize()
    done = 0
    while True:
        r = case.m.step(latent, case.d_text, ss)
        if r is None:
            break
        done = r
        torch.cuda.synchronize()
        assert rel_l2(host(latent), xs[done]) < 1e-4, f"after step {done}"
    assert done == T
    # the fresh skip features matter: the sequential segmentation with the same number of components ends elsewhere
    plain = Case("tiny", B.AD_F32, N, w, 1, T, cfg_scale=2.0, std=0.1, time_shift=shift)
    assert rel_l2(plain.oracle.run(plain.noise, plain.text)[-1], xs[-1]) > 1e-6


def test_wrapped_narrow_sdxl_bf16():
    """SDXL-shaped reduced-width model (the case the paper names), N = 4 wrapped, Euler, pooled branch."""
    r = RUNS["sdxl_narrow"]
    T = 12
    case = Case("sdxl_narrow", B.AD_BF16, r["N"], r["w"], 1, T, sampler=r["sampler"], cfg_scale=r["cfg_scale"], wrap=True)
    worst = run_components_isolated(case)
    xs = case.oracle.run(case.noise, case.text, case.pooled)
    case.m.set_graph_mode(True)
    case.m.reset(T, sampler=B.AD_EULER, cfg_scale=r["cfg_scale"])
    got, rounds = run_steps(case, r["N"])
    assert rounds == T
    assert rel_l2(got, xs[-1]) < 5e-2
    print(f"wrapped sdxl_narrow bf16: worst per-evaluation rel L2 {worst:.2e}, final latent {rel_l2(got, xs[-1]):.2e}")


# ---- video model: frames as the batch axis, temporal attention after every spatial transformer ----------------

def test_video_tiny_fp32_components_and_trajectory():
    r = RUNS["video_tiny"]
    case = Case("video_tiny", B.AD_F32, r["N"], r["w"], r["S"], r["T"], std=0.1)
    worst, latent = run_components_along_schedule(case)
    xs = case.oracle.run(case.noise, case.text)
    assert host(latent).shape == xs[-1].shape == (3, 4, 8, 8)
    assert rel_l2(host(latent), xs[-1]) < 1e-4
    # the round driver: three components on three streams, with and without graph replay
    for graphs in (0, 1):
        c2 = Case("video_tiny", B.AD_F32, 3, 1, 1, 8, std=0.1)
        c2.m.set_graph_mode(graphs)
        got, _ = run_steps(c2, 3)
        assert rel_l2(got, c2.oracle.run(c2.noise, c2.text)[-1]) < 1e-4
    print(f"video tiny fp32: worst per-component rel L2 {worst:.2e}")


def test_video_narrow_bf16_components_and_trajectory():
    """Reduced-width clone of the video configuration (16 frames, 8 temporal heads, N=4, 2 warm-up steps, DDIM)."""
    r = RUNS["video_narrow"]
    T = 5
    case = Case("video_narrow", B.AD_BF16, r["N"], r["w"], r["S"], T)
    worst = run_components_isolated(case)
    assert worst < 2e-2
    got, rounds = run_steps(case, r["N"])
    xs = case.oracle.run(case.noise, case.text)
    assert rounds == T
    err = rel_l2(got, xs[-1])
    assert err < 5e-2, f"final latent rel L2 {err:.3e}"
    print(f"video narrow bf16: worst per-component rel L2 {worst:.2e}, final latent {err:.2e}")


def test_video_full_size_first_units_and_properties():
    """The video configuration at its real shape (16 frames of 64x64 latents).  Against the oracle on the same
    seeded inputs: the first convolution, the first ResBlock and the temporal layer over all 65536 tokens (the
    spatial transformer in front of it is switched off by a zero output projection, so that the oracle does not
    have to evaluate sixteen 4096-token self-attentions in fp64; that part runs at full size in the test of the
    768px model).  Then the launch configuration the benchmark uses (four streams, graph replay), with the real
    weights, against direct launches on one stream, bit for bit."""
    from oracle.unet import _temporal, build_units, run_units
    d = CONFIGS["video_16f"]
    ocfg = UNetConfig(**d)
    units = build_units(ocfg)
    last = 2
    assert units[last].kind == "tfm"
    progress("drawing weights")
    wts = SI.make_weights(weight_manifest(ocfg), bf16_exact=True)
    off = dict(wts)
    tname = units[last].name
    off[tname + ".proj_out.w"] = np.zeros_like(wts[tname + ".proj_out.w"])
    off[tname + ".proj_out.b"] = np.zeros_like(wts[tname + ".proj_out.b"])
    prefixes = tuple(units[i].name + "." for i in range(last + 1)) + ("time.",)
    sub = {k: np.asarray(v, np.float64) for k, v in off.items() if k.startswith(prefixes)}
    noise = SI.make_video_latent(d["frames"], d["latent_channels"], d["height"], d["width"])
    text = quantize(SI.make_text(1, d["ctx_len"], d["ctx_dim"]), B.AD_BF16)
    taus = __import__("oracle.sampler", fromlist=["timesteps"]).timesteps(25)
    progress("oracle: first two units")
    ref = run_units(ocfg, units, 0, 1, sub, {-1: noise.astype(np.float64)}, taus[0], text.astype(np.float64), None)
    # the temporal layer never mixes positions: its reference is evaluated on a sample of them (corners included)
    progress("oracle: temporal layer on sampled positions")
    hw = d["height"] * d["width"]
    pos = np.unique(np.concatenate([[0, d["width"] - 1, hw - d["width"], hw - 1],
                                    np.random.default_rng(11).integers(0, hw, 252)]))
    z = ref[1].reshape(d["frames"], -1, hw)[:, :, pos][..., None]             # [frames, C, n, 1]
    ref_t = _temporal(ocfg, units[last], sub, z)[..., 0]                        # [frames, C, n]
    progress("gpu")

    cuts = [last + 1, 28, 39]
    d_text = dev(text, B.AD_BF16)
    m = ad.AsyncDiff(d, 4, 2, 1, B.AD_BF16, cuts=cuts)
    m.allocate(DEV)
    m.load_weights(off)
    m.reset(25)
    ins, outs = m.component_io(1)
    assert ins == [-1] and outs == [0, 2]        # the ResBlock's output stays inside; it is checked through the temporal layer
    hout = []
    for u in outs:
        (b, h, w, c), _ = m.tensor_shape(u)
        hout.append(torch.full((b, h, w, c), float("nan"), device=DEV, dtype=torch.bfloat16))
    m.component_forward(1, [dev_f32(noise)], 0, d_text, hout, torch.cuda.current_stream())
    torch.cuda.synchronize()
    err = rel_l2(nhwc_to_nchw(host(hout[0])), ref[0])
    assert err < 2e-2, f"unit 0: rel L2 {err:.3e}"
    got_t = nhwc_to_nchw(host(hout[1])).reshape(d["frames"], -1, hw)
    assert np.isfinite(got_t).all()
    err = rel_l2(got_t[:, :, pos], ref_t)
    assert err < 2e-2, f"temporal layer on sampled positions: rel L2 {err:.3e}"
    del hout
    m.load_weights(wts)

    def trajectory(streams, graphs, T=5):
        m.set_graph_mode(graphs)
        m.reset(T)
        latent = dev_f32(noise)
        ss = [torch.cuda.Stream(device=DEV) for _ in range(streams)]
        torch.cuda.synchronize()
        snaps = []
        while m.step(latent, d_text, ss) is not None:
            torch.cuda.synchronize()
            snaps.append(latent.cpu().numpy().copy())
        return snaps

    direct, replay = trajectory(1, False), trajectory(4, True)
    assert len(direct) == len(replay) == 5
    for r, (a, b) in enumerate(zip(direct, replay)):
        assert np.array_equal(a, b), f"round {r}"
    assert np.isfinite(replay[-1]).all() and replay[-1].shape == (16, 4, 64, 64)
    m.close()


@pytest.mark.parametrize("N,w,S,sampler,wrap,shift", [(2, 1, 2, "euler", False, False), (3, 2, 1, "ddim", True, False),
                                                      (3, 1, 3, "ddim", False, True)])
def test_video_tiny_schedule_variants(N, w, S, sampler, wrap, shift):
    """The video model under stride denoising, the Euler sampler, time shifting and the wrapped segmentation:
    the latent of every completed step against the oracle."""
    T = 9
    case = Case("video_tiny", B.AD_F32, N, w, S, T, sampler=sampler, std=0.1, wrap=wrap, time_shift=shift)
    xs = case.oracle.run(case.noise, case.text)
    latent = case.init_latent()
    ss = [torch.cuda.Stream(device=DEV) for _ in range(N + S - 1)]
    torch.cuda.synchronize()
    done = 0
    while True:
        r = case.m.step(latent, case.d_text, ss)
        if r is None:
            break
        done = r
        torch.cuda.synchronize()
        assert rel_l2(host(latent), xs[done]) < 1e-4, f"after step {done}"
    assert done == T


@pytest.mark.parametrize("name", ["sd21_768", "sd_512"])
def test_full_size_whole_unet_matches_oracle(full_size_weights, name):
    """The complete noise prediction of the 768px and of the 512px model (all 46 units as one component; 4.3 and 1.9
    TFLOP in fp64 on the oracle side, up to half a minute of CPU time) against the GPU's first denoising step,
    element by element.  The two configurations share the architecture and therefore the weights."""
    from oracle.unet import unet_forward
    d = CONFIGS[name]
    ocfg = UNetConfig(**d)
    noise = SI.make_latent(d["latent_channels"], d["height"], d["width"])
    text = quantize(SI.make_text(d["batch"], d["ctx_len"], d["ctx_dim"]), B.AD_BF16)
    taus = __import__("oracle.sampler", fromlist=["timesteps"]).timesteps(50)
    m = ad.AsyncDiff(d, 1, 0, 1, B.AD_BF16)
    m.allocate(DEV)
    m.load_weights(full_size_weights)
    m.reset(50)
    nu = len(m.units())
    (b, h, w, c), _ = m.tensor_shape(nu - 1)
    eps = torch.full((b, c, h, w), float("nan"), device=DEV, dtype=torch.float32)
    m.component_forward(1, [dev_f32(noise)], 0, dev(text, B.AD_BF16), [eps], torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = host(eps)
    m.close()
    torch.cuda.empty_cache()
    progress("oracle: whole UNet forward")
    x = np.broadcast_to(noise.astype(np.float64), (d["batch"],) + noise.shape).copy()
    ref = unet_forward(ocfg, full_size_weights, x, taus[0], text.astype(np.float64))
    err = rel_l2(got, ref)
    progress(f"whole UNet at full size ({name}): rel L2 {err:.3e}")
    assert got.shape == ref.shape and err < 2e-2


def test_partition_tuning_helpers():
    """Profile-guided partition: measured unit times balanced by the library's rule, then refined by timing whole
    rounds; the result is a valid split that the library accepts and the oracle reproduces."""
    from paper_2406_06911_amd.tuning import refine_cuts, time_balanced_cuts
    d = CONFIGS["sd21_narrow"]
    wts = SI.make_weights(weight_manifest(UNetConfig(**d)), bf16_exact=True)
    cuts, times = time_balanced_cuts(d, 3, B.AD_BF16, wts, DEV)
    nu = len(times)
    assert len(cuts) == 2 and 0 < cuts[0] < cuts[1] < nu and all(t > 0 for t in times)
    assert cuts == ad.balance_cuts(times, 3)
    best, ms, tried = refine_cuts(d, 3, 1, 1, B.AD_BF16, wts, cuts, DEV, max_evals=6)
    assert tuple(cuts) in tried and tuple(best) in tried and ms == tried[tuple(best)] <= tried[tuple(cuts)]
    assert 0 < best[0] < best[1] < nu and len(tried) <= 6
    case = Case("sd21_narrow", B.AD_BF16, 3, 1, 1, 5, cuts=best)
    got, _ = run_steps(case, 3)
    assert rel_l2(got, case.oracle.run(case.noise, case.text)[-1]) < 5e-2


def test_full_size_sdxl_first_units_match_oracle():
    """The SDXL-shaped configuration at its real shape (1024px: latent 128x128, text width 2048, pooled branch):
    the first seven units (first convolution, three ResBlocks, the strided convolution and a depth-2 transformer
    over 4096 tokens) against the oracle on the same seeded inputs."""
    from oracle.unet import build_units, run_units
    d = CONFIGS["sdxl_1024"]
    ocfg = UNetConfig(**d)
    units = build_units(ocfg)
    last = 6
    assert [u.kind for u in units[:last + 1]] == ["conv_in", "res", "res", "down", "res", "tfm", "res"]
    progress("drawing the weights of sdxl_1024")
    wts = SI.make_weights(weight_manifest(ocfg), bf16_exact=True)
    prefixes = tuple(units[i].name + "." for i in range(last + 1)) + ("time.", "pool.")
    sub = {k: np.asarray(v, np.float64) for k, v in wts.items() if k.startswith(prefixes)}
    noise = SI.make_latent(d["latent_channels"], d["height"], d["width"])
    text = quantize(SI.make_text(d["batch"], d["ctx_len"], d["ctx_dim"]), B.AD_BF16)
    pooled = SI.make_pooled(d["batch"], d["pooled_dim"])
    taus = __import__("oracle.sampler", fromlist=["timesteps"]).timesteps(50)
    x = np.broadcast_to(noise.astype(np.float64), (d["batch"],) + noise.shape).copy()
    progress("oracle: first seven units")
    ref = run_units(ocfg, units, 0, last, sub, {-1: x}, taus[0], text.astype(np.float64), pooled)

    progress("gpu: loading the weights")
    m = ad.AsyncDiff(d, 4, 3, 2, B.AD_BF16, cuts=[last + 1, 15, 27])
    m.allocate(DEV)
    m.load_weights(wts)
    m.reset(50, sampler=B.AD_EULER)
    ins, outs = m.component_io(1)
    assert ins == [-1] and sorted(ref.keys()) == sorted(outs)
    hout = []
    for u in outs:
        (b, h, w, c), _ = m.tensor_shape(u)
        hout.append(torch.full((b, h, w, c), float("nan"), device=DEV, dtype=torch.bfloat16))
    m.component_forward(1, [dev_f32(noise)], 0, dev(text, B.AD_BF16), hout, torch.cuda.current_stream(), pooled=dev_f32(pooled))
    torch.cuda.synchronize()
    for u, t in zip(outs, hout):
        err = rel_l2(nhwc_to_nchw(host(t)), ref[u])
        assert err < 2e-2, f"unit {u}: rel L2 {err:.3e}"
    m.close()


# ---------------------------------------------------------------------------------------------------
# Asynchronous rounds and the deep / wide units at full size against the oracle
# ---------------------------------------------------------------------------------------------------
def test_full_size_async_round_components_match_oracle(full_size_weights):
    """The metric configuration at its real shape with the FLOP-balanced partition of four components: the last
    warm-up step and the first asynchronous round, every component evaluation against the oracle's evaluation of the
    same schedule row.  Each evaluation is fed the oracle's stored tensors of the round before (rounded to bf16), so
    the asynchronous round runs on genuinely stale inputs of real size: 2 x 4 component evaluations, two UNet
    forwards in fp64 on the oracle side.  (One warm-up step instead of the configuration's three: the warm-up steps
    are the same computation, and step w - 1 is the one that seeds the asynchronous phase.)"""
    case = Case("sd21_768", B.AD_BF16, 4, 1, 1, 2, cfg_scale=7.5, wts=full_size_weights)
    assert [a for a, _ in case.m.partition()] == [0, 10, 31, 40]          # conv_in.. | d1.ds.. | u2.us.. | u0.0.tfm..out
    log = []
    progress("oracle: two steps of four components")
    worst = run_components_isolated(case, log)
    rounds = sorted({r for r, _, _, _ in log})
    assert rounds == [0, 1] and sorted({c for _, c, _, _ in log}) == [1, 2, 3, 4]
    progress(f"full-size warm-up step and first asynchronous round: worst per-tensor rel L2 {worst:.3e}")
    for r in rounds:
        progress(f"  round {r} " + " ".join(f"c{c}/u{u}:{e:.1e}" for rr, c, u, e in log if rr == r))
    case.m.close()


def _single_unit_against_oracle(name, unit, N, cuts, comp, T, sampler, seed):
    """One unit of a full-size model as a component of its own: seeded N(0,1) hidden state in, oracle's run_units on the
    same (bf16-rounded) input and the weights of that unit."""
    from oracle.unet import build_units, run_units
    d = CONFIGS[name]
    ocfg = UNetConfig(**d)
    units = build_units(ocfg)
    u = units[unit]
    progress("drawing weights")
    wts = SI.make_weights(weight_manifest(ocfg), bf16_exact=True)
    prefixes = (u.name + ".", "time.", "pool.")
    sub = {k: np.asarray(v, np.float64) for k, v in wts.items() if k.startswith(prefixes)}
    frames = d.get("frames", 0)
    text = quantize(SI.make_text(1 if frames else d["batch"], d["ctx_len"], d["ctx_dim"]), B.AD_BF16)
    pooled = SI.make_pooled(d["batch"], d["pooled_dim"]) if d["pooled_dim"] else None
    x = quantize(SI.make_array((d["batch"], u.c_in, u.h_in, u.w_in), seed), B.AD_BF16)
    taus = __import__("oracle.sampler", fromlist=["timesteps"]).timesteps(T)
    step = 3
    progress(f"oracle: unit {u.name}")
    ref = run_units(ocfg, units, unit, unit, sub, {unit - 1: x.astype(np.float64)}, taus[step], text.astype(np.float64), pooled)[unit]
    progress("gpu: loading the weights")
    m = ad.AsyncDiff(d, N, 1, 1, B.AD_BF16, cuts=cuts)
    m.allocate(DEV)
    m.load_weights(wts)
    del wts
    progress("gpu: forward")
    m.reset(T, sampler=sampler)
    assert m.partition()[comp - 1] == (unit, unit)
    ins, outs = m.component_io(comp)
    assert ins == [unit - 1] and outs == [unit]
    (b, h, w, c), _ = m.tensor_shape(unit)
    out = torch.full((b, h, w, c), float("nan"), device=DEV, dtype=torch.bfloat16)
    m.component_forward(comp, [dev(nchw_to_nhwc(x), B.AD_BF16)], step, dev(text, B.AD_BF16), [out], torch.cuda.current_stream(),
                        pooled=dev_f32(pooled) if pooled is not None else None)
    torch.cuda.synchronize()
    got = nhwc_to_nchw(host(out))
    m.close()
    assert got.shape == ref.shape and np.isfinite(got).all()
    err = rel_l2(got, ref)
    # the residual path passes x through unchanged: also compare what the unit adds
    err_delta = rel_l2(got - x, ref - x)
    progress(f"{name} unit {u.name}: rel L2 {err:.3e}, of the unit's own contribution {err_delta:.3e}")
    assert err < 2e-2
    return err, err_delta


def test_full_size_sdxl_depth10_transformer_matches_oracle():
    """The deepest transformer of the SDXL-shaped model at its real width: 1280 channels, 32x32 = 1024 tokens, 20 heads,
    ten layers (self-attention, cross-attention to the 77x2048 text embedding, GEGLU feed-forward each)."""
    from oracle.unet import build_units
    units = build_units(UNetConfig(**CONFIGS["sdxl_1024"]))
    unit = 10
    assert (units[unit].name, units[unit].depth, units[unit].c_in, units[unit].h_in) == ("d2.0.tfm", 10, 1280, 32)
    err, err_delta = _single_unit_against_oracle("sdxl_1024", unit, 3, [unit, unit + 1], 2, 50, B.AD_EULER, 9100)
    assert err_delta < 5e-2          # ten layers of three residual branches each, every one rounded to bf16


def test_full_size_video_level1_transformer_and_temporal_layer_match_oracle():
    """The level-1 transformer of the video model at full width and its temporal layer: 16 frames of 32x32 tokens,
    640 channels; spatial self / cross attention per frame, then attention over the 16 frames at each of the 1024
    positions - every output element against the oracle."""
    from oracle.unet import build_units
    units = build_units(UNetConfig(**CONFIGS["video_16f"]))
    unit = 7
    assert (units[unit].name, units[unit].c_in, units[unit].h_in) == ("d1.0.tfm", 640, 32)
    err, err_delta = _single_unit_against_oracle("video_16f", unit, 3, [unit, unit + 1], 2, 25, B.AD_DDIM, 9200)
    assert err_delta < 3e-2
