"""The C++ scheduler behind lamps_sched.h against the oracle's plain model -- CPU only
(no GPU call is made by any scheduler function).

Times are compared exactly: both sides evaluate the same formulas in the same order in
IEEE double precision."""
import os
import re

import pytest

import lamps_workloads as W
import paper_2410_18248_amd as P
from oracle import scheduler as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
POLICY = {S.FCFS: P.LAMPS_POLICY_FCFS, S.SJF: P.LAMPS_POLICY_SJF, S.SJF_TOTAL: P.LAMPS_POLICY_SJF_TOTAL,
          S.LAMPS: P.LAMPS_POLICY_LAMPS, S.FIXED: P.LAMPS_POLICY_FIXED}


def _cfg(policy, max_batch, memory, cost, starvation=100, refresh=1, chunk=1 << 30, c_other=0.0, M=1.0):
    cm = P.LampsCostModel(cost.it_a, cost.it_b, cost.fwd_a, cost.fwd_b, cost.sw_a, cost.sw_b,
                          1 if cost.swap_stalls else 0, 1 if cost.unit else 0)
    return P.LampsSchedConfig(POLICY[policy], max_batch, memory, starvation, refresh, chunk, c_other, M, cm)


def _both(make_requests, policy, max_batch, memory, cost, **kw):
    """Runs the oracle and the library on the same requests; returns (oracle sim, results by id)."""
    reqs = make_requests()
    sim = S.Simulator(reqs, policy, max_batch, memory, cost,
                      starvation_threshold=kw.get("starvation", 100), score_refresh=kw.get("refresh", 1),
                      recompute_chunk=kw.get("chunk", 1 << 30), c_other=kw.get("c_other", 0.0),
                      bytes_per_token=kw.get("M", 1.0)).run()
    sched = P.LampsSched(_cfg(policy, max_batch, memory, cost, **kw))
    for r in make_requests():
        segs = [(s[0], s[1], s[2], r.handling[k]) for k, s in enumerate(r.segments)]
        sched.add(r.id, r.arrival, r.prompt, segs, r.priority)
    sched.run()
    got = {r.id: sched.result(r.id, len(r.segments)) for r in reqs}
    stats = sched.stats()
    sched.destroy()
    return sim, got, stats


def _example():
    return [S.Request(1, 0.0, 0, [(5, 2.0, 0), (1, None, 0)], [S.PRESERVE, None], priority=3),
            S.Request(2, 0.0, 0, [(1, 7.0, 0), (1, None, 0)], [S.DISCARD, None], priority=2),
            S.Request(3, 0.0, 0, [(2, 1.0, 0), (1, None, 0)], [S.SWAP, None], priority=1)]


@pytest.mark.parametrize("policy,total", [(S.FCFS, 35), (S.SJF, 31), (S.SJF_TOTAL, 33), (S.FIXED, 30),
                                          (S.LAMPS, 29)])
def test_worked_example_through_the_c_abi(policy, total):
    """Section 3.1: average completion 11.66 / 10.33 / 11 / 10 = 35/3, 31/3, 33/3, 30/3; ranked by
    the memory-over-time area the example ends at 29/3 (the oracle's pins say why)."""
    sim, got, stats = _both(_example, policy, 1, 6, S.CostModel(unit=True), chunk=1)
    assert sum(c for c, _, _ in got.values()) == total
    assert {i: c for i, (c, _, _) in got.items()} == sim.completion_times()
    assert stats[1] <= 6


def _random_requests(seed, n):
    u = W.uniform01(seed, 8 * n)
    reqs = []
    for i in range(n):
        x = u[8 * i:8 * i + 8]
        segs = []
        for k in range(int(x[0] * 3)):
            segs.append((1 + int(x[1 + k] * 12), 0.5 + 30 * x[3 + k], int(x[5] * 6)))
        segs.append((1 + int(x[6] * 15), None, 0))
        reqs.append(S.Request(i, float(int(x[7] * 40)), int(x[5] * 20), segs))
    return reqs


def test_hand_worked_timelines_through_the_c_abi():
    """The two timelines the oracle's pins work out by hand: a blocked queue discards its
    worst-ranked holder before idling; a starving request runs in the iteration in which its
    counter reaches the threshold."""
    def blocked():
        return [S.Request(1, 0.0, 3, [(2, 1.0, 0), (4, None, 0)], [S.PRESERVE, None]),
                S.Request(2, 0.0, 3, [(2, 1.0, 0), (4, None, 0)], [S.PRESERVE, None]),
                S.Request(3, 20.0, 0, [(1, None, 0)])]
    _, got, stats = _both(blocked, S.FCFS, 2, 12, S.CostModel(unit=True))
    assert {i: c for i, (c, _, _) in got.items()} == {1: 8.0, 2: 13.0, 3: 21.0} and stats[2] == 1

    def starving():
        return [S.Request(0, 0.0, 0, [(3, None, 0)])] + \
               [S.Request(i, float(i - 1), 0, [(1, None, 0)]) for i in range(1, 13)]
    _, got, _ = _both(starving, S.SJF, 1, 1000, S.CostModel(unit=True), starvation=4)
    assert got[0][0] == 6.0 and got[4][0] == 7.0 and got[5][0] == 8.0


COSTS = [S.CostModel(it_a=1.0, it_b=0.001, fwd_a=0.2, fwd_b=0.05, sw_a=0.1, sw_b=0.01),
         S.CostModel(it_a=0.013, it_b=2.1e-6, fwd_a=3e-3, fwd_b=4.5e-5, sw_a=2e-3, sw_b=7e-6,
                     swap_stalls=False)]


@pytest.mark.parametrize("policy", [S.FCFS, S.SJF, S.SJF_TOTAL, S.LAMPS])
@pytest.mark.parametrize("cost", COSTS)
def test_library_equals_oracle_on_random_workloads(policy, cost):
    for seed, kw in ((1, dict(starvation=25, c_other=60.0)), (2, dict(starvation=7, refresh=4, chunk=5)),
                     (3, dict(c_other=300.0, M=2.5))):
        sim, got, stats = _both(lambda: _random_requests(seed, 60), policy, 4, 130, cost, **kw)
        for r in sim.reqs:
            c, f, h = got[r.id]
            assert c == r.completion and f == r.first_token, (seed, r.id)
            assert h == [x if x is not None else -1 for x in r.handling]
        assert stats == (sim.iteration, sim.peak_memory, sim.preemptions)


def test_step_interface_reports_what_the_driver_must_do():
    """One request, Swap: the batch entry says what to bring back, the event says how it left."""
    cost = S.CostModel(it_a=1.0)
    sched = P.LampsSched(_cfg(S.FCFS, 2, 100, cost))
    sched.add(7, 0.0, 4, [(2, 3.0, 5, P.LAMPS_SWAP), (1, None, 0, None)])
    b = sched.next_batch()
    assert b == [(7, 0, 4, 4)]                           # the prompt is run through the model first
    assert sched.commit() == []
    assert sched.next_batch() == [(7, 0, 0, 5)] and sched.commit() == []
    assert sched.next_batch() == [(7, 0, 0, 6)]
    assert sched.commit(0.5) == [(7, 0, P.LAMPS_SWAP, 6)]            # measured iteration time
    assert sched.now() == 2.5
    b = sched.next_batch()                               # time jumps to the API return at 5.5
    assert sched.now() == 5.5 and b == [(7, 6, 5, 11)]   # swap 6 back in, process the 5 response tokens
    assert sched.commit() == []
    assert sched.next_batch() == [(7, 0, 0, 12)]
    assert sched.commit() == [(7, 1, P.LAMPS_PRESERVE, 12)]
    assert sched.next_batch() == []
    c, f, h = sched.result(7, 2)
    assert c == 7.5 and f == 2.0 and h == [P.LAMPS_SWAP, -1]
    sched.destroy()


def test_out_of_memory_discards_are_reported_once_and_recomputed():
    """Two requests come back from Preserve calls holding 5 tokens each with room for neither's
    next segment: the worse-ranked one is discarded; the step interface names it once, and it
    recomputes its context when it runs again.  Totals equal the oracle's."""
    cost = S.CostModel(unit=True)

    def reqs():
        return [S.Request(i, 0.0, 3, [(2, 1.0, 0), (4, None, 0)], [S.PRESERVE, None]) for i in (1, 2)]
    sim = S.Simulator(reqs(), S.FCFS, 2, 12, cost).run()
    assert sim.preemptions >= 1
    sched = P.LampsSched(_cfg(S.FCFS, 2, 12, cost))
    for r in reqs():
        sched.add(r.id, r.arrival, r.prompt, [(s[0], s[1], s[2], r.handling[k]) for k, s in enumerate(r.segments)])
    dropped, recomputed = [], {}
    for _ in range(200):
        batch = sched.next_batch()
        got = sched.take_discards()
        assert sched.take_discards() == []            # each is reported once
        dropped += got
        if not batch:
            break
        for rid, swap_in, recompute, context in batch:
            if rid in dropped and recompute > 0:
                recomputed[rid] = recomputed.get(rid, 0) + recompute
        sched.commit()
    assert len(dropped) == sim.preemptions == sched.stats()[2]
    for rid in set(dropped):
        assert recomputed[rid] >= 5                   # prompt + the two generated tokens come back by recompute
    for r in sim.reqs:
        c, f, h = sched.result(r.id, len(r.segments))
        assert c == r.completion and f == r.first_token
    sched.destroy()


def test_closed_forms_equal_the_oracle():
    u = W.uniform01(99, 900)
    for k in range(100):
        a = u[9 * k:9 * k + 9]
        T, Ci, Co, M, tf, ts = 30 * a[0], int(4000 * a[1]), int(20000 * a[2]), 1 + 3 * a[3], a[4], 0.1 * a[5]
        lib = P.load_library()
        assert lib.lamps_waste_preserve(T, Ci, M) == S.waste_preserve(T, Ci, M)
        assert lib.lamps_waste_discard(tf, Ci, Co, M) == S.waste_discard(tf, Ci, Co, M)
        assert lib.lamps_waste_swap(ts, Ci + Co, M) == S.waste_swap(ts, Ci + Co, M)
        assert lib.lamps_handling_strategy(T, Ci, Co, M, tf, ts) == S.handling_strategy(T, Ci, Co, M, tf, ts)
        c0, n1, rho, n2, tau = int(500 * a[6]), int(60 * a[7]), int(20 * a[8]), int(40 * a[0]), 0.01 + a[1]
        for strat in (0, 1, 2):
            assert lib.lamps_memory_over_time(strat, c0, n1, T, rho, n2, tau, tf, ts) == \
                S.memory_over_time(strat, c0, n1, T, rho, n2, tau, tf, ts)


def test_argument_checks():
    cost = S.CostModel(it_a=1.0)
    bad = _cfg(S.FCFS, 0, 100, cost)
    with pytest.raises(P.LampsError):
        P.LampsSched(bad)
    sched = P.LampsSched(_cfg(S.FCFS, 2, 100, cost))
    with pytest.raises(P.LampsError):
        sched.add(1, 0.0, 0, [(1, 2.0, 0, None)])         # the last segment must have no call
    with pytest.raises(P.LampsError):
        sched.add(1, 0.0, 0, [(1, None, 0, None), (1, None, 0, None)])   # a middle segment needs one
    with pytest.raises(P.LampsError):
        sched.add(1, 0.0, 0, [(0, None, 0, None)])
    sched.add(1, 0.0, 0, [(1, None, 0, None)])
    with pytest.raises(P.LampsError) as e:
        sched.add(1, 0.0, 0, [(1, None, 0, None)])
    assert e.value.status == -3
    with pytest.raises(P.LampsError):
        sched.commit()                                   # no batch pending
    with pytest.raises(P.LampsError):
        sched.result(5)
    sched.destroy()
    big = P.LampsSched(_cfg(S.FCFS, 1, 3, cost))
    big.add(1, 0.0, 0, [(9, None, 0, None)])             # needs 9 tokens of a budget of 3
    with pytest.raises(P.LampsError) as e:
        big.next_batch()
    assert e.value.status == -6
    big.destroy()


def test_library_exports_every_symbol_of_the_scheduler_header():
    header = open(os.path.join(ROOT, "include", "lamps_sched.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = sorted(set(re.findall(r"\b(lamps_[a-z_]+)\s*\(", header)))
    assert len(names) >= 14
    lib = P.load_library()
    for n in names:
        assert hasattr(lib, n), n
