"""Pins for oracle/serving_sim.simulate that do not come from the simulation itself.

The model restates iteration-level scheduling over a block budget (paper Section 4.1's block manager under the
engine's first-come-first-served, one-token-per-iteration loop; whole-life reservation is this build's reading).
Pinned here by closed forms of special cases and by invariants recomputed from the returned trace:
  - equal requests that all wait from the start run in waves of floor(capacity / life) requests: admission and
    finish iterations have a closed form, and so has the makespan;
  - a budget that holds exactly one request serialises the stream: finish iterations are prefix sums;
  - a lone request that arrives late is admitted on arrival and the clock jumps over the idle gap;
  - under random streams: first come first served, never before arrival, exactly output_len consecutive
    iterations per request, the blocks held recounted from the definition, held <= promised <= capacity;
  - a shrink admits nobody until the promises fit again, and takes nothing from those running.
"""
import math

import numpy as np
import pytest

from oracle import serving_sim

T = 16


def life(p, o):
    return math.ceil((p + o) / T)


@pytest.mark.parametrize("n,p,o,cap,max_batch", [(10, 40, 12, 13, 1 << 30), (7, 5, 30, 9, 2), (25, 100, 7, 70, 1 << 30),
                                                 (4, 16, 1, 2, 1 << 30)])
def test_equal_requests_run_in_waves_with_closed_form_times(n, p, o, cap, max_batch):
    k = min(max_batch, cap // life(p, o))
    assert k >= 1
    trace, adm, fin = serving_sim.simulate([0] * n, [p] * n, [o] * n, cap, 0, lambda it: 0, T, max_batch=max_batch)
    for i in range(n):
        assert adm[i] == (i // k) * o and fin[i] == (i // k) * o + o - 1
    assert len(trace) == math.ceil(n / k) * o                       # makespan in iterations
    for it, ids, held, promised in trace:
        wave = it // o
        assert ids == list(range(wave * k, min(n, (wave + 1) * k)))
        assert promised == len(ids) * life(p, o)
        assert held == len(ids) * math.ceil((p + (it - wave * o) + 1) / T)


def test_a_budget_of_one_request_serialises_the_stream():
    rng = np.random.Generator(np.random.PCG64(5))
    o = rng.integers(1, 40, size=12).tolist()
    p = [T * 3 - x for x in o]                                      # every life is exactly 3 blocks
    trace, adm, fin = serving_sim.simulate([0] * 12, p, o, 3, 0, lambda it: 0, T)
    starts = np.concatenate([[0], np.cumsum(o)[:-1]]).tolist()
    assert adm == starts and fin == [s + x - 1 for s, x in zip(starts, o)]
    assert all(len(ids) == 1 for _, ids, _, _ in trace) and len(trace) == sum(o)


def test_a_late_arrival_is_admitted_on_arrival_and_idle_time_is_skipped():
    trace, adm, fin = serving_sim.simulate([3, 500], [10, 10], [5, 4], 8, 0, lambda it: 0, T)
    assert adm == [3, 500] and fin == [7, 503]
    assert [it for it, _, _, _ in trace] == [3, 4, 5, 6, 7, 500, 501, 502, 503]


@pytest.mark.parametrize("seed", range(6))
def test_invariants_recomputed_from_the_trace_on_random_streams(seed):
    rng = np.random.Generator(np.random.PCG64([11, seed]))
    n = 60
    arrival = np.sort(rng.integers(0, 200, size=n)).tolist()
    p = rng.integers(0, 300, size=n).tolist()
    o = rng.integers(1, 80, size=n).tolist()
    n_gpu, unit, level = 40, 8, int(rng.integers(0, 4))
    max_batch = int(rng.integers(2, 12))
    cap = n_gpu + level * unit
    trace, adm, fin = serving_sim.simulate(arrival, p, o, n_gpu, unit, lambda it: level, T, max_batch=max_batch)
    assert all(a >= arr for a, arr in zip(adm, arrival))            # never before arrival
    assert all(a <= b for a, b in zip(adm, adm[1:]))                # first come first served
    assert all(f - a + 1 == x for a, f, x in zip(adm, fin, o))      # output_len consecutive iterations
    ran = {i: [] for i in range(n)}
    for it, ids, held, promised in trace:
        assert ids == sorted(ids) and len(ids) <= max_batch
        for i in ids:
            ran[i].append(it)
        assert held == sum(math.ceil((p[i] + (it - adm[i]) + 1) / T) for i in ids)
        assert promised == sum(life(p[i], o[i]) for i in ids)
        assert held <= promised <= cap
    for i in range(n):
        assert ran[i] == list(range(adm[i], fin[i] + 1))
    # a request that waited did so for a reason: at its admission the one before it in line had just been
    # admitted too, or something ended in the iteration before (blocks or a batch place came free)
    its = {it: ids for it, ids, _, _ in trace}
    for i in range(1, n):
        if adm[i] > arrival[i]:
            assert adm[i - 1] == adm[i] or any(fin[j] == adm[i] - 1 for j in its.get(adm[i] - 1, []))


def test_a_shrink_stops_admissions_and_takes_nothing_from_running_requests():
    n = 30
    p, o = [20] * n, [10] * n                                       # life 2 blocks each
    level_at = lambda it: 2 if it < 15 else 0                       # 8 + 2 * 4 = 16 blocks, then 8
    trace, adm, fin = serving_sim.simulate([0] * n, p, o, 8, 4, level_at, T)
    by_it = {it: (ids, promised) for it, ids, _, promised in trace}
    assert len(by_it[0][0]) == 8 and by_it[14][1] == 16             # eight at a time while expanded
    assert by_it[15][0] == by_it[14][0]                             # the shrink preempts nobody
    for i in range(n):
        if adm[i] >= 15:
            assert by_it[adm[i]][1] <= 8                            # admitted only once the promises fit again
    assert max(len(ids) for it, (ids, _) in by_it.items() if it >= 20) == 4
    assert all(f - a + 1 == 10 for a, f in zip(adm, fin))
