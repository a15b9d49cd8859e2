"""The asynchronous denoising schedule (Section 3.2 "Asynchronous Denoising", "Stride
Denoising"; Appendix A "Stride Denoising", "Time Shifting") as an explicit integer table,
plus three independent evaluators of it.

Steps are numbered i = 0..T-1 in execution order (the paper counts t downwards, so its
"t-1" is i+1 here).  x_0 is the initial noise and x_{i+1} = S(x_i, eps_i, i).

Rule (reading of the paper, with stride S >= 1 and warm-up w):
  * i < w: the N components run one after another on fresh inputs (plain sequential inference).
  * afterwards steps are grouped into rounds of S; the round starting at step b reads only what
    the previous round (or warm-up step w-1) stored:
      - the last component is evaluated for every step b..b+S-1 of the round, each time with that
        step's time embedding, all on the same stored inputs; evaluation j gives eps_{b+j};
      - components 1..N-1 are evaluated once, with the time embedding of the round's last step;
        component 1 reads the latent x_b available when the round starts;
      - a trailing round with fewer than S steps evaluates only the last component.
  * every cross-component input (main hidden state and skip features) is the stored one.

Wrapped segmentation (Appendix A "Model Segmentation", the SDXL case; stride 1 only - the paper does not say how
the two combine): the unit list has N+1 segments, numbered here as evaluations 1..N+1; segment 1 (head) and
segment N+1 (tail) are one component and run back to back on one device.  In an asynchronous round the head reads
the fresh latent, segments 2..N read stored inputs, and the tail reads the head's outputs of THIS round (they never
left the device) and stored inputs from everybody else; the tail yields eps.  Warm-up runs all N+1 in order.
"""
from dataclasses import dataclass
from typing import Callable, Dict, List


@dataclass(frozen=True)
class Row:
    round: int        # global round counter (warm-up steps are rounds 0..w-1)
    comp: int         # 1..N
    tau_step: int     # step index whose timestep feeds this evaluation's time embedding
    read_slot: int    # slot (0/1) the stored inputs are read from
    write_slot: int   # slot the outputs are stored in, -1 = outputs other than eps are dropped
    latent_step: int  # i of the latent x_i read by component 1, else -1
    eps_step: int     # step whose noise prediction this evaluation yields (last component), else -1
    fresh_from: int = 0  # wrapped segmentation: component whose outputs of this same round are read (0 = none)


def build_schedule(T: int, N: int, w: int, S: int, time_shift: bool = False, wrap: bool = False) -> List[Row]:
    assert T >= 1 and N >= 1 and S >= 1 and w >= 0 and (N == 1 or w >= 1)
    shift = lambda i: i - 1 if (time_shift and i >= w and i >= 1) else i
    rows: List[Row] = []
    g = 0
    if wrap:
        assert N >= 2 and S == 1
        P = N + 1                                    # evaluations per step: head, N-1 middle segments, tail
        for i in range(min(w, T)):
            for n in range(1, P + 1):
                rows.append(Row(g, n, i, g & 1, g & 1, i if n == 1 else -1, i if n == P else -1))
            g += 1
        for b in range(min(w, T), T):
            rd, wr = (g - 1) & 1, g & 1
            for n in range(1, P):
                rows.append(Row(g, n, shift(b), rd, wr, b if n == 1 else -1, -1))
            rows.append(Row(g, P, shift(b), rd, wr, -1, b, 1))
            g += 1
        return rows
    for i in range(min(w, T)):
        for n in range(1, N + 1):
            rows.append(Row(g, n, i, g & 1, g & 1, i if n == 1 else -1, i if n == N else -1))
        g += 1
    b = min(w, T)
    while b < T:
        s_r = min(S, T - b)
        full = s_r == S
        rd, wr = (g - 1) & 1, g & 1
        if full:
            for n in range(1, N):
                rows.append(Row(g, n, shift(b + S - 1), rd, wr, b if n == 1 else -1, -1))
        for j in range(s_r):
            keep = full and j == S - 1
            rows.append(Row(g, N, shift(b + j), rd, wr if keep else -1, b if N == 1 else -1, b + j))
        g += 1
        b += s_r
    return rows


# ----------------------------------------------------------------------------------------------
# Evaluators.  comp_fn(n, stored, x, tau_step) -> bundle, where `stored` maps producer component
# m -> the bundle m produced (only m in feeds[n]), x is the latent (component 1 only, else None).
# eps_fn(bundle of component N) -> eps.  sampler_fn(x, eps, i) -> next latent.
# ----------------------------------------------------------------------------------------------

def run_table(rows: List[Row], feeds: Dict[int, List[int]], comp_fn: Callable, eps_fn: Callable,
              sampler_fn: Callable, x0, N: int, trace=None):
    """Iterative double-buffered execution of the table.  Returns the list of latents x_0..x_T."""
    xs = [x0]
    slots = [dict(), dict()]
    k = 0
    while k < len(rows):
        g = rows[k].round
        group = []
        while k < len(rows) and rows[k].round == g:
            group.append(rows[k])
            k += 1
        pending, eps = [], {}
        for r in group:
            stored = {m: slots[r.read_slot][m] for m in feeds[r.comp]}
            if r.fresh_from and r.write_slot != r.read_slot:
                # the producer ran earlier in this round on the same device: its output has not been stored yet
                stored[r.fresh_from] = next(b for (_, n, b) in pending if n == r.fresh_from)
            x = xs[r.latent_step] if r.latent_step >= 0 else None
            bundle = comp_fn(r.comp, stored, x, r.tau_step)
            if trace is not None:
                trace.append((r, bundle))
            if r.eps_step >= 0:
                eps[r.eps_step] = eps_fn(bundle)
            if r.write_slot < 0:
                continue
            if r.write_slot == r.read_slot:      # warm-up: later components of this step see it
                slots[r.write_slot][r.comp] = bundle
            else:                                # asynchronous round: visible from the next round on
                pending.append((r.write_slot, r.comp, bundle))
        for (s, n, bundle) in pending:
            slots[s][n] = bundle
        for i in sorted(eps):
            assert i == len(xs) - 1
            xs.append(sampler_fn(xs[i], eps[i], i))
    return xs


def run_recursive(T, N, w, S, feeds, comp_fn, eps_fn, sampler_fn, x0, time_shift=False, wrap=False):
    """Memoised evaluation straight from the rule in the module docstring (no table, no slots)."""
    memo_out, memo_x = {}, {0: x0}
    shift = lambda i: i - 1 if (time_shift and i >= w and i >= 1) else i
    if wrap:
        assert S == 1
        P = N + 1

        def latent_w(i):
            if i not in memo_x:
                memo_x[i] = sampler_fn(latent_w(i - 1), eps_fn(out_w(P, i - 1)), i - 1)
            return memo_x[i]

        def out_w(n, i):
            if (n, i) not in memo_out:
                if i < w:
                    stored = {m: out_w(m, i) for m in feeds[n]}
                    tau = i
                else:       # stored inputs are one step old, except what the head hands to the tail
                    stored = {m: out_w(m, i if (n == P and m == 1) else i - 1) for m in feeds[n]}
                    tau = shift(i)
                memo_out[(n, i)] = comp_fn(n, stored, latent_w(i) if n == 1 else None, tau)
            return memo_out[(n, i)]

        return [latent_w(i) for i in range(T + 1)]

    def round_start(i):
        return w + ((i - w) // S) * S

    def latent(i):
        if i not in memo_x:
            memo_x[i] = sampler_fn(latent(i - 1), eps_fn(out(N, i - 1)), i - 1)
        return memo_x[i]

    def out(n, i):
        if (n, i) in memo_out:
            return memo_out[(n, i)]
        if i < w:
            stored = {m: out(m, i) for m in feeds[n]}
            val = comp_fn(n, stored, latent(i) if n == 1 else None, i)
        else:
            b = round_start(i)
            assert n == N or i == b + S - 1, "components 1..N-1 exist only at the last step of a full round"
            stored = {m: out(m, b - 1) for m in feeds[n]}
            val = comp_fn(n, stored, latent(b) if n == 1 else None, shift(i))
        memo_out[(n, i)] = val
        return val

    return [latent(i) for i in range(T + 1)]


def run_sequential(T, N, feeds, comp_fn, eps_fn, sampler_fn, x0):
    """Plain sequential denoising (Section 3.2, first paragraph): every component fresh, every step."""
    xs = [x0]
    for i in range(T):
        done = {}
        for n in range(1, N + 1):
            done[n] = comp_fn(n, {m: done[m] for m in feeds[n]}, xs[i] if n == 1 else None, i)
        xs.append(sampler_fn(xs[i], eps_fn(done[N]), i))
    return xs
