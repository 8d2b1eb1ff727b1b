"""Pins for the oracle's scheduler model -- CPU only.

What fixes it from outside: the four average completion times the paper prints
for its worked example (Section 3.1), hand-evaluated instances of equations
(1)-(3), the qualitative choices Section 2.3 states, a brute-force integration
of a simulated request's memory curve for the memory-over-time function, the
textbook optimality of shortest-job-first on one machine, and the invariants
of Algorithm 1 (memory budget, batch size, starvation bound)."""
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


def test_memory_over_time_by_hand_and_ordering():
    # c0 = 10, n1 = 2, T = 5, rho = 3, n2 = 2, tau = 1
    pre = 11 + 12
    post = (12 + 3 + 1) + (12 + 3 + 2)
    assert S.memory_over_time(S.PRESERVE, 10, 2, 5.0, 3, 2, 1.0, 0.7, 0.2) == pre + 5.0 * 12 + post
    assert S.memory_over_time(S.DISCARD, 10, 2, 5.0, 3, 2, 1.0, 0.7, 0.2) == pytest.approx(pre + 0.7 * 12 + post)
    assert S.memory_over_time(S.SWAP, 10, 2, 5.0, 3, 2, 1.0, 0.7, 0.2) == pytest.approx(pre + 2 * 0.2 * 12 + post)
    # a longer API call costs a Preserve request more and the others nothing
    assert S.memory_over_time(S.PRESERVE, 10, 2, 9.0, 3, 2, 1.0, 0.7, 0.2) > \
        S.memory_over_time(S.PRESERVE, 10, 2, 5.0, 3, 2, 1.0, 0.7, 0.2)
    assert S.memory_over_time(S.SWAP, 10, 2, 9.0, 3, 2, 1.0, 0.7, 0.2) == \
        S.memory_over_time(S.SWAP, 10, 2, 5.0, 3, 2, 1.0, 0.7, 0.2)


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
