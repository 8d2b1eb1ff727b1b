"""Pins for the oracle's scheduler model -- CPU only.

What fixes it from outside: the four average completion times the paper prints
for its worked example (Section 3.1), hand-evaluated instances of equations
(1)-(3), the qualitative choices Section 2.3 states, a brute-force integration
of a simulated request's memory curve for the memory-over-time function (all
three strategies), hand-worked timelines for the out-of-memory discard and for
the iteration in which a starving request is served, the textbook optimality
of shortest-job-first on one machine, and the invariants of Algorithm 1
(memory budget, batch size, starvation bound).  The one statement of the paper
the rank does not meet -- the order it gives for its worked example -- is kept
as a strict expected failure with the numbers.

parity unpinned: the LAMPS branch of Simulator._rank on the paper's worked
example (the definition and the example's stated order disagree).
"""
import itertools
import os

import numpy as np
import pytest

import lamps_workloads as W
from oracle import scheduler as S

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _example_requests():
    # total length 6 / 2 / 3, API after 5 / 1 / 2 tokens, API duration 2 / 7 / 1,
    # Preserve / Discard / Swap (the example's table)
    return [S.Request(1, 0.0, 0, [(5, 2.0, 0), (1, None, 0)], [S.PRESERVE, None], priority=3),
            S.Request(2, 0.0, 0, [(1, 7.0, 0), (1, None, 0)], [S.DISCARD, None], priority=2),
            S.Request(3, 0.0, 0, [(2, 1.0, 0), (1, None, 0)], [S.SWAP, None], priority=1)]


def _printed():
    out = {}
    for line in open(os.path.join(GOLD, "worked_example_completion_times.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


@pytest.mark.parametrize("name,policy,total", [("FCFS", S.FCFS, 35), ("SJF", S.SJF, 31),
                                               ("SJF_TOTAL", S.SJF_TOTAL, 33),
                                               ("PREFERRED", S.FIXED, 30)])
def test_worked_example_average_completion_times(name, policy, total):
    sim = S.Simulator(_example_requests(), policy, max_batch=1, memory_tokens=6,
                      cost=S.CostModel(unit=True), recompute_chunk=1).run()
    mean = sim.mean_completion()
    assert abs(mean * 3 - total) < 1e-9
    printed = _printed()[name]
    assert abs(mean - printed) < 0.0067, (mean, printed)        # the paper truncates to 2 decimals
    assert sim.peak_memory <= 6


def test_worked_example_fcfs_timeline_matches_the_text():
    sim = S.Simulator(_example_requests(), S.FCFS, 1, 6, S.CostModel(unit=True), recompute_chunk=1).run()
    c = sim.completion_times()
    # R2's pre-API part runs during R1's API call, R3 cannot; R2 finishes last
    assert c == {1: 8.0, 3: 12.0, 2: 15.0}
    ran = {t: ids for t, ids in sim.trace}
    assert ran[6.0] == [2]                              # the unit from 5 to 6
    assert 7.0 not in ran                               # idle from 6 to 7: R3 does not fit


def test_worked_example_sjf_timeline_matches_the_text():
    sim = S.Simulator(_example_requests(), S.SJF, 1, 6, S.CostModel(unit=True), recompute_chunk=1).run()
    ran = {t: ids for t, ids in sim.trace}
    assert ran[9.0] == [1]          # at time 8 R2 is back but R1, also with two units left, goes on
    assert 10.0 not in ran and 11.0 not in ran          # R1 in its API holds 5 of 6: R2 (needs 2) waits
    assert sim.completion_times() == {3: 5.0, 1: 12.0, 2: 14.0}


def test_equations_by_hand():
    # T_INT = 3 s, C_i = 100 tokens, M = 2 bytes; T_fwd = 0.5 s, C_other = 900; T_swap = 0.1 s
    assert S.waste_preserve(3.0, 100, 2.0) == 600.0
    assert S.waste_discard(0.5, 100, 900, 2.0) == 0.5 * 100 * 2 + 0.5 * 900 * 2 == 1000.0
    assert S.waste_swap(0.1, 1000, 2.0) == 2 * 0.1 * 1000 * 2 == 400.0
    assert S.handling_strategy(3.0, 100, 900, 2.0, 0.5, 0.1) == S.SWAP
    assert S.handling_strategy(0.1, 100, 900, 2.0, 0.5, 0.1) == S.PRESERVE
    assert S.handling_strategy(3.0, 100, 900, 2.0, 0.05, 0.1) == S.DISCARD


def test_strategy_choices_follow_section_2_3():
    """Brief calls: Preserve.  Long calls: Discard if the context is short (cheap to
    recompute), Swap otherwise."""
    t_fwd = lambda C: 1e-3 + 4e-5 * C                          # recompute: cheap start, steep slope
    t_swap = lambda C: 2e-3 + 8e-6 * C                         # swap: costly start, shallow slope
    pick = lambda T, C: S.handling_strategy(T, C, 20000, 1.0, t_fwd(C), t_swap(C))
    assert pick(1e-4, 500) == S.PRESERVE and pick(1e-4, 4000) == S.PRESERVE    # math-like API
    assert pick(20.0, 20) == S.DISCARD                                          # long call, tiny context
    assert pick(20.0, 4000) == S.SWAP                                           # long call, long context


def test_waste_scales_as_the_equations_say():
    for f in (2.0, 5.0):
        assert S.waste_preserve(f * 3, 7, 11) == f * S.waste_preserve(3, 7, 11)
        assert S.waste_discard(0.3, 7, f * 13, 11) - S.waste_discard(0.3, 7, 0, 11) == \
            pytest.approx(f * (S.waste_discard(0.3, 7, 13, 11) - S.waste_discard(0.3, 7, 0, 11)))
        assert S.waste_swap(f * 0.2, 50, 11) == pytest.approx(f * S.waste_swap(0.2, 50, 11))


def test_memory_over_time_preserve_equals_integrated_simulation():
    """A single request alone in the system, Preserve: the integral of the memory it
    holds over time, summed iteration by iteration from the simulation's own record."""
    tau, T = 0.25, 3.0
    r = S.Request(1, 0.0, 0, [(6, T, 0), (4, None, 0)], [S.PRESERVE, None])
    cost = S.CostModel(it_a=tau)
    sim = S.Simulator([r], S.FCFS, 1, 100, cost)
    held = []

    class Spy(S.CostModel):
        def iteration(self, ctx_tokens, recomputed, swapped):
            held.append(ctx_tokens)
            return tau
    sim.cost = Spy(it_a=tau)
    sim.run()
    area = sum(h * tau for h in held) + T * 6
    assert S.memory_over_time(S.PRESERVE, 0, 6, T, 0, 4, tau, 0.0, 0.0) == pytest.approx(area)


class _Recorder(S.CostModel):
    """A cost model that also records, per executed iteration, what the simulator reports
    to it and how long the iteration's two phases last: the stall while blocks move
    (swapped tokens held), then the model's pass (the batch's context held)."""

    def __init__(self, **kw):
        super().__init__(**kw)
        self.phases = []                                # (seconds, tokens held) pieces, in order

    def iteration(self, ctx_tokens, recomputed, swapped):
        total = super().iteration(ctx_tokens, recomputed, swapped)
        stall = (self.sw_a + self.sw_b * swapped) if (self.swap_stalls and swapped > 0) else 0.0
        if ctx_tokens or recomputed or swapped:         # (0, 0, 0) is the rank asking for tau
            self.phases.append((stall, swapped))
            self.phases.append((total - stall, ctx_tokens))
        return total


def _integrated_alone(strategy, c0, n1, T, n2, cost):
    """Memory x time of one request that runs alone, summed piece by piece from what the
    simulator itself executed; the API call contributes T x (what the strategy leaves in memory)."""
    r = S.Request(1, 0.0, c0, [(n1, T, 0), (n2, None, 0)], [strategy, None])
    S.Simulator([r], S.FCFS, 1, 10 ** 6, cost).run()
    area = sum(dt * held for dt, held in cost.phases)
    first = cost.phases[1]                              # the prompt's own pass is not part of the rank:
    area -= first[0] * first[1]                         # the rank starts with c0 tokens already there
    if strategy == S.PRESERVE:
        area += T * (c0 + n1)
    return area


@pytest.mark.parametrize("strategy", [S.PRESERVE, S.DISCARD, S.SWAP])
def test_memory_over_time_equals_the_integrated_memory_curve_of_a_request_run_alone(strategy):
    """Section 4.2: the rank is the integral of the memory-over-time curve.  The curve here is
    the simulator's own record of a single request (iteration by iteration: how long, how many
    tokens held), not the closed form.  The cost model is a consistent one: the iteration that
    recomputes C tokens lasts T_fwd(C) (fwd_a = it_a, no per-context term), moving C tokens
    stalls the engine for T_swap(C), during which those C tokens are held."""
    c0, n1, T, n2 = 7, 6, 3.0, 4
    cost = _Recorder(it_a=0.25, it_b=0.0, fwd_a=0.25, fwd_b=0.01, sw_a=0.05, sw_b=0.002)
    C = c0 + n1
    got = S.memory_over_time(strategy, c0, n1, T, 0, n2, 0.25, cost.t_fwd(C), cost.t_swap(C))
    assert got == pytest.approx(_integrated_alone(strategy, c0, n1, T, n2, cost), rel=1e-12)
    # and the three differ where they should: by hand, C = 13
    mids = {S.PRESERVE: 3.0 * 13, S.DISCARD: (0.25 + 0.13) * 13, S.SWAP: 2 * (0.05 + 0.026) * 13}
    base = S.memory_over_time(S.PRESERVE, c0, n1, 0.0, 0, n2, 0.25, 0.0, 0.0)
    assert got - base == pytest.approx(mids[strategy], rel=1e-12)


def test_memory_over_time_orders_strategies_as_section_4_2_describes():
    # a longer API call costs a Preserve request more and the others nothing
    assert S.memory_over_time(S.PRESERVE, 10, 2, 9.0, 3, 2, 1.0, 0.7, 0.2) > \
        S.memory_over_time(S.PRESERVE, 10, 2, 5.0, 3, 2, 1.0, 0.7, 0.2)
    for strat in (S.DISCARD, S.SWAP):
        assert S.memory_over_time(strat, 10, 2, 9.0, 3, 2, 1.0, 0.7, 0.2) == \
            S.memory_over_time(strat, 10, 2, 5.0, 3, 2, 1.0, 0.7, 0.2)
    # the response's tokens are context of everything generated after the call
    assert S.memory_over_time(S.SWAP, 10, 2, 5.0, 3, 2, 1.0, 0.7, 0.2) - \
        S.memory_over_time(S.SWAP, 10, 2, 5.0, 0, 2, 1.0, 0.7, 0.2) == pytest.approx(3 * 2 * 1.0)


def _lamps_on_the_example():
    sim = S.Simulator(_example_requests(), S.LAMPS, max_batch=1, memory_tokens=6,
                      cost=S.CostModel(unit=True), recompute_chunk=1)
    for r in sim.reqs:
        sim._decide(r)
    return sim, {r.id: sim._rank(r) for r in sim.reqs}


def test_lamps_rank_on_the_worked_example_recorded_values():
    """What the area gives on the only instance the paper fixes, in the example's own units
    (one unit per iteration, one unit to recompute, swaps free):
      R1 Preserve: 1+2+3+4+5 before the call, 5 held for 2 units, 6 after        = 31
      R2 Discard : 1 before, nothing during, 1 while recomputing, 2 after         =  4
      R3 Swap    : 1+2 before, nothing during, 3 after                            =  6
    R1 is last, as Sections 3.1 and 4.3 say.  R2 comes out below R3; see the next test."""
    sim, rank = _lamps_on_the_example()
    assert rank == {1: 31.0, 2: 4.0, 3: 6.0}
    sim.run()
    # ranked by area the three finish at 14, 10, 5: a mean of 29/3, not above the 30/3 of the
    # schedule the figure calls preferred
    assert sim.completion_times() == {1: 14.0, 2: 10.0, 3: 5.0}
    assert sim.peak_memory <= 6


@pytest.mark.xfail(strict=True, reason=
                   "Sections 3.1 and 4.3 say R3 first, then R2, then R1, and the figure's caption gives "
                   "a mean of 10 for that order.  The integral of memory over time puts R2 (at most 4: "
                   "it never holds more than 2 tokens and holds nothing during its call) below R3 (at "
                   "least 6 = 1+2+3 even with free swaps) under every reading tried; only a curve that "
                   "keeps a Discard request's memory during its 7-unit call puts R3 first, which "
                   "Section 4.2 rules out (nothing is held during a Discard or Swap call).  Recorded as "
                   "a disagreement between the paper's definition and its example.")
def test_lamps_rank_gives_the_order_the_paper_states_for_its_example():
    sim, rank = _lamps_on_the_example()
    assert rank[3] < rank[2] < rank[1]
    assert sim.run().mean_completion() == pytest.approx(_printed()["PREFERRED"])


def test_blocked_queue_discards_its_worst_ranked_holder_before_idling():
    """Section 4.3 on full memory: jobs are discarded and recomputed when memory is there again.
    Worked by hand (FCFS, batch of 2, budget 12, unit iterations, recompute in one iteration):
      A, B: prompt 3, two tokens, a Preserve call of 1 unit, then four tokens.  Z: one token, arrives at 20.
      t 0-1  both prompts (3 + 3 held)      t 1-3  two tokens each (5 + 5 held), both calls end at 4
      t 4    both are back holding 5 and need 4 more each; 2 are free: nothing fits, and both
             waiting requests hold memory -> B (later id = worse FCFS rank) is discarded
      t 4-8  A generates its four tokens and finishes at 8 (held 9, freed)
      t 8-9  B recomputes its 5 tokens, t 9-13 generates four: finishes at 13
      t 20   Z arrives, runs, finishes at 21
    Had the engine idled until the next event instead (Z's arrival at 20), A could not have
    finished before 24."""
    def reqs():
        return [S.Request(1, 0.0, 3, [(2, 1.0, 0), (4, None, 0)], [S.PRESERVE, None]),
                S.Request(2, 0.0, 3, [(2, 1.0, 0), (4, None, 0)], [S.PRESERVE, None]),
                S.Request(3, 20.0, 0, [(1, None, 0)])]
    sim = S.Simulator(reqs(), S.FCFS, 2, 12, S.CostModel(unit=True)).run()
    assert sim.completion_times() == {1: 8.0, 2: 13.0, 3: 1.0}
    assert sim.preemptions == 1 and sim.peak_memory <= 12
    ran = dict(sim.trace)
    assert ran[9.0] == [2] and all(ran[float(t)] == [1] for t in range(5, 9))


def test_starving_request_runs_in_the_iteration_in_which_its_counter_reaches_the_threshold():
    """Algorithm 1's two loops, by hand (SJF, one request at a time, threshold 4, unit iterations):
    L needs 3 tokens; a 1-token request arrives at every time 0, 1, 2, ...
      iterations 0, 1, 2 (t 0-3): the short request of that time runs, L is left out: counter 1, 2, 3
      iteration 3 (t 3-4): counter 4 = threshold -> tagged while this batch is formed and put at
                           its head (Section 4.4), so L runs in this iteration, not the next
      L keeps its place until it completes: t 3-6, completion 6; the short requests that arrived
      at 3, 4, 5 wait behind it (their own counters stay below 4)."""
    reqs = [S.Request(0, 0.0, 0, [(3, None, 0)])]
    reqs += [S.Request(i, float(i - 1), 0, [(1, None, 0)]) for i in range(1, 13)]
    sim = S.Simulator(reqs, S.SJF, 1, 1000, S.CostModel(unit=True), starvation_threshold=4).run()
    ran = dict(sim.trace)
    assert [ran[float(t)] for t in range(1, 9)] == [[1], [2], [3], [0], [0], [0], [4], [5]]
    assert sim.completion_times()[0] == 6.0


def _plain(lengths, policy, max_batch=1, budget=10 ** 6):
    reqs = [S.Request(i, 0.0, 0, [(n, None, 0)]) for i, n in enumerate(lengths)]
    return S.Simulator(reqs, policy, max_batch, budget, S.CostModel(unit=True)).run()


def test_sjf_without_api_calls_is_optimal_on_one_machine():
    lengths = [5, 2, 7, 1, 3]
    best = min(sum(itertools.accumulate(p)) for p in itertools.permutations(lengths))
    assert _plain(lengths, S.SJF).mean_completion() * len(lengths) == best
    # without API calls the memory-over-time rank orders requests like their lengths
    assert _plain(lengths, S.LAMPS).completion_times() == _plain(lengths, S.SJF).completion_times()
    fc = _plain(lengths, S.FCFS).completion_times()
    assert [fc[i] for i in range(5)] == list(itertools.accumulate(lengths))


def _random_requests(seed, n):
    u = W.uniform01(seed, 8 * n)
    reqs = []
    for i in range(n):
        x = u[8 * i:8 * i + 8]
        segs = []
        for k in range(int(x[0] * 3)):                  # 0..2 API calls
            segs.append((1 + int(x[1 + k] * 12), 0.5 + 30 * x[3 + k], int(x[5] * 6)))
        segs.append((1 + int(x[6] * 15), None, 0))
        reqs.append(S.Request(i, float(int(x[7] * 40)), int(x[5] * 20), segs))
    return reqs


@pytest.mark.parametrize("policy", [S.FCFS, S.SJF, S.SJF_TOTAL, S.LAMPS])
def test_algorithm_1_invariants_on_random_workloads(policy):
    cost = S.CostModel(it_a=1.0, it_b=0.001, fwd_a=0.2, fwd_b=0.05, sw_a=0.1, sw_b=0.01)
    for seed in (1, 2, 3):
        reqs = _random_requests(seed, 40)
        sim = S.Simulator(reqs, policy, max_batch=4, memory_tokens=120, cost=cost,
                          starvation_threshold=25, c_other=60.0).run()
        assert all(r.state == S.DONE for r in reqs)
        assert sim.peak_memory <= 120
        assert all(len(ids) <= 4 for _, ids in sim.trace)
        for r in reqs:                                  # every token was generated exactly once
            assert r.completion >= r.arrival + sum(s[0] for s in r.segments) * 1.0
            assert r.first_token is not None and r.first_token <= r.completion


def test_starving_request_is_moved_to_the_head():
    """A long request under SJF with a stream of short arrivals would wait for all of
    them; the starvation counter bounds its wait."""
    reqs = [S.Request(0, 0.0, 0, [(15, None, 0)])]
    reqs += [S.Request(i, float(2 * (i - 1)), 0, [(2, None, 0)]) for i in range(1, 101)]
    free = S.Simulator([S.Request(r.id, r.arrival, 0, r.segments) for r in reqs], S.SJF, 1, 1000,
                       S.CostModel(unit=True), starvation_threshold=10 ** 9).run()
    guarded = S.Simulator(reqs, S.SJF, 1, 1000, S.CostModel(unit=True), starvation_threshold=20).run()
    assert free.completion_times()[0] >= 200            # served after the short ones
    # prioritised after 20 waits, then it runs to its end (before any short request has waited 20)
    assert guarded.completion_times()[0] <= 20 + 15 + 4
