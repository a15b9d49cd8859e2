"""Pins for oracle/schedule.py: values the paper prints, closed-form wiring rule, two derivations."""
import json
import os

import numpy as np
import pytest

from oracle import schedule as SC

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))

P = 1_000_003  # tag arithmetic base


def chain_feeds(N, extra=()):
    feeds = {n: ([n - 1] if n > 1 else []) for n in range(1, N + 1)}
    for m, n in extra:
        feeds[n] = sorted(set(feeds[n]) | {m})
    return feeds


def symbolic_fns():
    """Components as symbolic records: the bundle is the nested expression itself."""
    comp = lambda n, stored, x, tau: ("c", n, tau, x, tuple(sorted(stored.items())))
    eps = lambda bundle: ("eps", bundle)
    samp = lambda x, e, i: ("x", i + 1, x, e)
    return comp, eps, samp


def deps(expr, acc=None):
    """All latent indices and (component, tau) pairs an expression depends on, not descending into latents."""
    acc = {"x": set(), "c": set()} if acc is None else acc
    if expr[0] == "c":
        _, n, tau, x, stored = expr
        acc["c"].add((n, tau))
        if x is not None:
            acc["x"].add(x[1] if x[0] == "x" else 0)
        for _, b in stored:
            deps(b, acc)
    return acc


def latent_index(x):
    return x[1] if isinstance(x, tuple) and x[0] == "x" else 0


@pytest.mark.parametrize("N,w,S,T", [(4, 1, 1, 12), (3, 2, 1, 9), (2, 1, 1, 6), (3, 1, 2, 11), (4, 3, 2, 14), (3, 2, 3, 13)])
def test_table_equals_recursive_definition(N, w, S, T):
    comp, eps, samp = symbolic_fns()
    for feeds in (chain_feeds(N), chain_feeds(N, [(1, N)]) if N > 2 else chain_feeds(N)):
        rows = SC.build_schedule(T, N, w, S)
        a = SC.run_table(rows, feeds, comp, eps, samp, "x0", N)
        b = SC.run_recursive(T, N, w, S, feeds, comp, eps, samp, "x0")
        assert a == b and len(a) == T + 1


@pytest.mark.parametrize("N", [1, 2, 3, 4])
def test_eq5_dependency_rule_on_a_chain(N):
    """Eq. 5: eps of step i is built from component n evaluated at step i-N+n, reading x_{i-N+1}."""
    T, w = 12, 1
    comp, eps, samp = symbolic_fns()
    trace = []
    SC.run_table(SC.build_schedule(T, N, w, 1), chain_feeds(N), comp, eps, samp, ("x", 0), N, trace)
    heads = {r.eps_step: b for r, b in trace if r.eps_step >= 0}
    for i in range(w + N - 1, T):
        d = deps(heads[i])
        assert d["c"] == {(n, i - N + n) for n in range(1, N + 1)}
        assert d["x"] == {i - N + 1}
    # "component n computed at step t contributes to the prediction of step t-N+n" (counted downwards),
    # i.e. in execution order: the evaluation of component n made at step i ends up in eps of step i+N-n
    for r, b in trace:
        if r.round >= w + N - 1 and r.round + N - r.comp < T:
            assert (r.comp, r.tau_step) in deps(heads[r.round + N - r.comp])["c"]


def test_skip_edge_adds_older_latent_dependency():
    N, T, w = 4, 12, 1
    comp, eps, samp = symbolic_fns()
    trace = []
    SC.run_table(SC.build_schedule(T, N, w, 1), chain_feeds(N, [(1, 4), (2, 4)]), comp, eps, samp, ("x", 0), N, trace)
    heads = {r.eps_step: b for r, b in trace if r.eps_step >= 0}
    for i in range(w + N - 1, T):
        # chain gives x_{i-3}; edge 1->4 gives component 1 of step i-1 (reads x_{i-1}); edge 2->4 gives x_{i-2}
        assert deps(heads[i])["x"] == {i - 3, i - 2, i - 1}


@pytest.mark.parametrize("N,S", [(1, 1), (1, 2), (3, 1)])
def test_sequential_special_cases(N, S):
    comp, eps, samp = symbolic_fns()
    T = 7
    seq = SC.run_sequential(T, N, chain_feeds(N), comp, eps, samp, "x0")
    # warm-up covering every step is plain sequential denoising (Section 3.2)
    assert SC.run_table(SC.build_schedule(T, N, T, S), chain_feeds(N), comp, eps, samp, "x0", N) == seq
    assert SC.run_table(SC.build_schedule(T, N, T + 3, S), chain_feeds(N), comp, eps, samp, "x0", N) == seq
    if N == 1 and S == 1:
        assert SC.run_table(SC.build_schedule(T, 1, 0, 1), chain_feeds(1), comp, eps, samp, "x0", 1) == seq


def test_components_that_ignore_their_hidden_input():
    """If no component looks at what the previous one handed over, asynchronous == sequential."""
    comp = lambda n, stored, x, tau: ("c", n, tau, x if n == 1 else None)
    eps = lambda b: b
    samp = lambda x, e, i: ("x", i + 1, e[2])          # sampler looks only at the time step of eps
    T, N = 9, 3
    a = SC.run_table(SC.build_schedule(T, N, 1, 1), chain_feeds(N), comp, eps, samp, "x0", N)
    assert a == SC.run_sequential(T, N, chain_feeds(N), comp, eps, samp, "x0")


def test_stride_batch_printed_in_the_paper():
    """Section 3.2 / Figure 3: N=3, S=2: one batch computes eps^3(t), eps^1(t-1), eps^2(t-1), eps^3(t-1)."""
    g = GOLD["stride_batch_N3_S2"]["evaluations_relative_to_t"]
    T, N, w, S = 11, 3, 1, 2
    rows = SC.build_schedule(T, N, w, S)
    for rnd in range(w, w + (T - w) // S):
        group = [r for r in rows if r.round == rnd]
        b = min(r.tau_step for r in group)             # the paper's step "t" of this batch
        assert sorted((r.comp, r.tau_step - b) for r in group) == sorted(map(tuple, g))
        heads = [r for r in group if r.comp == N]
        assert len({r.read_slot for r in group}) == 1  # all read the previously broadcast states
        assert [r.eps_step for r in heads] == [b, b + 1]           # the batch yields x_{t-1} and x_{t-2}
        assert [r.write_slot for r in heads][0] == -1              # hidden states of step t are not kept
    # both eps^3 share the feature of eps^2 from the previous batch
    comp, eps, samp = symbolic_fns()
    trace = []
    SC.run_table(rows, chain_feeds(N), comp, eps, samp, ("x", 0), N, trace)
    by_round = {}
    for r, bdl in trace:
        if r.comp == N and r.round >= w:
            by_round.setdefault(r.round, []).append(bdl)
    for rnd, (b0, b1) in by_round.items():
        if rnd == w + (T - w) // S:
            continue
        assert b0[4] == b1[4] and b0[2] + 1 == b1[2]
    # steps {T-1, T-3, ..} (paper numbering) denoise alone; {T-2, T-4, ..} compute and broadcast (Appendix A)
    T2 = 9
    rows = SC.build_schedule(T2, 3, 1, 2)
    alone = sorted({r.tau_step for r in rows if r.round >= 1 and r.write_slot == -1})
    bcast = sorted({r.tau_step for r in rows if r.round >= 1 and r.comp == 1})
    assert alone == [1, 3, 5, 7] and bcast == [2, 4, 6, 8]


def test_round_and_device_counts_printed_in_the_paper():
    g = GOLD["broadcast_counts_T50"]
    rounds = lambda S: len({r.round for r in SC.build_schedule(50, 3, 1, S) if r.round >= 1})
    assert rounds(1) == g["stride1"] and rounds(2) == g["stride2"]
    # full rounds with stride 2 = (T - W) // 2 (Section 4.6)
    full = [r.round for r in SC.build_schedule(50, 3, 1, 2) if r.comp == 1 and r.round >= 1]
    assert len(full) == (50 - 1) // 2
    d = GOLD["devices"]
    per_round = lambda N, S: max(sum(1 for r in SC.build_schedule(50, N, 1, S) if r.round == k) for k in range(1, 20))
    assert per_round(2, 2) == d["N2_S2"] and per_round(3, 2) == d["N3_S2"] and per_round(4, 1) == d["N4_S1"]
    # evaluation count: w*N + R*(N+S-1) + rho
    for (T, N, w, S) in [(50, 4, 3, 2), (50, 4, 3, 1), (25, 4, 2, 1), (13, 3, 2, 3)]:
        R, rho = (T - w) // S, (T - w) % S
        assert len(SC.build_schedule(T, N, w, S)) == w * N + R * (N + S - 1) + rho
    assert len(SC.build_schedule(50, 4, 3, 2)) == 128


def test_time_shift_sequence_printed_in_the_paper():
    g = GOLD["time_shift_T50_w2_head"]
    rows = SC.build_schedule(50, 3, 2, 1, time_shift=True)
    label = lambda step: 50 - step                      # the paper numbers time embeddings 50..1
    seq = [label(r.tau_step) for r in rows if r.comp == 3]
    assert seq[:4] == g["shifted"] and seq[-2:] == g["shifted_tail"] and len(seq) == 50
    plain = [label(r.tau_step) for r in SC.build_schedule(50, 3, 2, 1) if r.comp == 3]
    assert plain[:4] == g["original"] and plain[-1] == 1


def test_slots_alternate_and_every_step_gets_one_eps():
    for (T, N, w, S) in [(10, 2, 1, 1), (50, 4, 3, 2), (13, 3, 2, 3), (5, 1, 0, 1)]:
        rows = SC.build_schedule(T, N, w, S)
        assert sorted(r.eps_step for r in rows if r.eps_step >= 0) == list(range(T))
        for r in rows:
            assert (r.eps_step >= 0) == (r.comp == N) and (r.latent_step >= 0) == (r.comp == 1)
            if r.round < w:
                assert r.read_slot == r.write_slot == r.round & 1
            else:
                assert r.read_slot == (r.round - 1) & 1 and r.write_slot in (-1, r.round & 1)


# ---- wrapped segmentation (Appendix A "Model Segmentation": first and last blocks in one segment) -------------

def wrap_feeds(N, extra=()):
    """Evaluations 1..N+1 on a chain; the tail (N+1) also reads the head's (1) skip features."""
    return chain_feeds(N + 1, [(1, N + 1)] + list(extra))


@pytest.mark.parametrize("N,w,T,shift", [(2, 1, 8, False), (3, 2, 10, False), (4, 1, 12, True)])
def test_wrapped_table_equals_recursive_definition(N, w, T, shift):
    comp, eps, samp = symbolic_fns()
    for feeds in (wrap_feeds(N), wrap_feeds(N, [(2, N + 1)]) if N > 2 else wrap_feeds(N)):
        rows = SC.build_schedule(T, N, w, 1, shift, wrap=True)
        a = SC.run_table(rows, feeds, comp, eps, samp, "x0", N)
        b = SC.run_recursive(T, N, w, 1, feeds, comp, eps, samp, "x0", shift, wrap=True)
        assert a == b and len(a) == T + 1


def test_wrapped_dependencies():
    """The tail reads the head of the SAME step (fresh latent through the skip features) and the middle segments
    one step behind each: eps_i is built from head and tail at step i, segment n (2..N) at step i-(N+1-n), and so
    from the latents x_i (head of this step) and x_{i-N+1} (the head whose output went down the chain)."""
    N, T, w = 3, 12, 1
    comp, eps, samp = symbolic_fns()
    trace = []
    SC.run_table(SC.build_schedule(T, N, w, 1, wrap=True), wrap_feeds(N), comp, eps, samp, ("x", 0), N, trace)
    heads = {r.eps_step: b for r, b in trace if r.eps_step >= 0}
    for i in range(w + N, T):
        d = deps(heads[i])
        expect = {(N + 1, i), (1, i)} | {(n, i - (N + 1 - n)) for n in range(2, N + 1)} | {(1, i - N)}
        assert d["c"] == expect
        assert d["x"] == {i, i - N}
    # per asynchronous round: N+1 evaluations, only the tail reads something of its own round, one eps
    rows = SC.build_schedule(T, N, w, 1, wrap=True)
    for g in range(w, T):
        grp = [r for r in rows if r.round == g]
        assert [r.comp for r in grp] == list(range(1, N + 2))
        assert [r.fresh_from for r in grp] == [0] * N + [1]
        assert [r.eps_step for r in grp] == [-1] * N + [g] and grp[0].latent_step == g
        assert all(r.read_slot == (g - 1) & 1 and r.write_slot == g & 1 for r in grp)


def test_wrapped_full_warmup_is_sequential():
    N, T = 3, 6
    comp, eps, samp = symbolic_fns()
    feeds = wrap_feeds(N)
    a = SC.run_table(SC.build_schedule(T, N, T, 1, wrap=True), feeds, comp, eps, samp, "x0", N)
    assert a == SC.run_sequential(T, N + 1, feeds, comp, eps, samp, "x0")


def test_wrapped_partition_rule():
    """Independent derivation: for every head end and tail start, the best split of the middle comes from the
    (separately pinned) sequential partition; the wrapped optimum is the best of those."""
    from oracle.partition import partition, partition_wrapped
    rng = np.random.default_rng(3)
    for trial in range(25):
        m = int(rng.integers(4, 13))
        n = int(rng.integers(2, min(4, m - 1) + 1))
        costs = [int(c) for c in rng.integers(1, 50, size=m)]
        cuts = partition_wrapped(costs, n)
        edges = [0] + cuts + [m]
        assert len(cuts) == n and all(a < b for a, b in zip(edges, edges[1:]))
        loads = [sum(costs[edges[k]:edges[k + 1]]) for k in range(n + 1)]
        got = max([loads[0] + loads[n]] + loads[1:n])
        best = None
        for c1 in range(1, m):
            for cn in range(c1 + n - 1, m):
                mid = costs[c1:cn]
                if n == 2:
                    worst_mid = sum(mid)
                else:
                    mc = [0] + partition(mid, n - 1) + [len(mid)]
                    worst_mid = max(sum(mid[mc[k]:mc[k + 1]]) for k in range(n - 1))
                v = max(sum(costs[:c1]) + sum(costs[cn:]), worst_mid)
                best = v if best is None else min(best, v)
        assert got == best, (costs, n)
