"""Pins for oracle/controller_sim.py: the closed-form fixed point of the
transparency condition (Section 3.1), the worked example of Section 3.3, and the
behaviours Section 3.4.2 states in prose."""
import math

import pytest

from conftest import load_golden
from oracle.controller_sim import AdaptiveExpansion, Observation, linear_timing, simulate

G = load_golden("worked_example.txt")


def run(units, L, c, s, steps=600, **kw):
    tkw = {k: kw.pop(k) for k in ("tput_gain", "slow_from", "slow_until", "slow_factor") if k in kw}
    ctl = AdaptiveExpansion(units=units, k_max=units - 1, **kw)
    levels = simulate(ctl, linear_timing(L, units, c, s, **tkw), steps)
    return ctl, levels


def test_starts_with_everything_on_the_gpu():
    ctl, levels = run(32, 32, 1.0, 10.0)
    assert levels[0] == 0 and AdaptiveExpansion(units=4, k_max=3).host_fraction == 0.0


@pytest.mark.parametrize("units,c,s,rho", [(32, 1.0, 10.0, 0.9), (32, 1.0, 4.0, 0.9), (100, 0.288, 7.7, 0.9),
                                           (64, 2.0, 3.0, 1.0), (20, 1.0, 1.5, 0.5)])
def test_fixed_point_is_the_closed_form(units, c, s, rho):
    """t_in(f) = f*s, compute c per layer: largest level with (k/units)*s <= rho*c."""
    ctl, levels = run(units, 8, c, s, steps=2000, rho=rho, probe_period=10 ** 9, util_max=1.01)
    expect = min(units - 1, math.floor(rho * c * units / s + 1e-12))
    assert expect >= 1
    assert levels[-1] == expect
    assert levels[-200:] == [expect] * 200                      # settled, no oscillation
    assert (expect / units) * s <= rho * c < ((expect + 1) / units) * s or expect == units - 1
    assert max(levels) == expect                                # never overshoots in a noiseless model


def test_worked_example_level_is_four():
    n = int(G["n_layers"])
    # one unit = one layer; swapping a layer takes 2 compute times; per layer of compute
    # the link can move m*2/n of a layer: transparent while 2m <= n
    ctl, levels = run(n, n, 1.0, float(G["t_swap_over_t_compute"]) * 1.0, rho=1.0, probe_period=10 ** 9)
    assert levels[-1] == int(G["fifo_length"])
    ctl, levels = run(n, n, 1.0, float(G["t_swap_over_t_compute"]) * 1.0, rho=0.9, probe_period=10 ** 9)
    assert levels[-1] == 4


def test_growth_is_one_unit_at_a_time_after_k_up_clean_steps():
    ctl, levels = run(32, 4, 1.0, 2.0, steps=60, k_up=5)
    changes = [(i, levels[i - 1], levels[i]) for i in range(1, len(levels)) if levels[i] != levels[i - 1]]
    assert all(b - a == 1 for _, a, b in changes)
    assert [i for i, _, _ in changes][:3] == [5, 10, 15]


def test_shrinks_after_sustained_slowdown_and_not_on_a_spike():
    base = dict(units=32, L=4, c=1.0, s=4.0, probe_period=10 ** 9)
    ctl, lv = run(steps=400, **base)
    k0 = lv[-1]
    assert k0 == 7
    # one slow step (brief interference): tolerated
    ctl, lv = run(steps=400, slow_from=300, slow_until=301, slow_factor=2.0, **base)
    assert lv[300:] == [k0] * 100
    # sustained 2x slower link: comes down until compute no longer waits, i.e. to the largest level with
    # (k/32)*8 <= 1, which is 4 (the margin rho applies to growing, not to shrinking)
    ctl, lv = run(steps=400, slow_from=300, slow_until=None, slow_factor=2.0, **base)
    assert lv[-1] == 4
    first_drop = next(i for i in range(300, 400) if lv[i] < k0)
    assert first_drop - 300 <= 2 + 1                      # k_down = 2 bad steps, effective the step after
    assert all(b - a in (0, -1) for a, b in zip(lv[300:], lv[301:]))


def test_stall_alone_triggers_shrink():
    ctl = AdaptiveExpansion(units=10, k_max=9)
    ctl.k = 3
    ok = Observation([1.0] * 4, [0.1] * 4, [0.0] * 4, 0.1, 1.0)
    stalled = Observation([1.0] * 4, [0.1] * 4, [0.5, 0, 0, 0], 0.1, 1.0)
    assert ctl.observe(stalled) == 3
    assert ctl.observe(ok) == 3                           # streak broken
    assert ctl.observe(stalled) == 3
    assert ctl.observe(stalled) == 2
    assert ctl.ceiling == 3


def test_plateau_stops_growth_and_steps_back():
    # throughput does not improve with more memory: try one level, see no gain, go back and hold
    ctl, lv = run(32, 4, 1.0, 2.0, steps=300, tput_gain=0.0, probe_period=10 ** 9)
    assert max(lv) == 1 and lv[-1] == 0
    assert lv[-250:] == [0] * 250


def test_periodic_probe_retries_and_returns():
    ctl, lv = run(32, 4, 1.0, 2.0, steps=400, tput_gain=0.0, probe_period=50)
    ups = [i for i in range(1, len(lv)) if lv[i] > lv[i - 1]]
    assert len(ups) >= 4                                   # keeps probing
    assert all(50 <= b - a <= 70 for a, b in zip(ups[1:], ups[2:]))
    assert max(lv) == 1


def test_link_saturation_blocks_growth():
    ctl = AdaptiveExpansion(units=10, k_max=9)
    busy = Observation([1.0] * 2, [0.0] * 2, [0.0] * 2, 0.95, 1.0)
    for _ in range(20):
        ctl.observe(busy)
    assert ctl.k == 0
    free = Observation([1.0] * 2, [0.0] * 2, [0.0] * 2, 0.2, 1.0)
    for _ in range(4):
        ctl.observe(free)
    assert ctl.k == 1


def test_recovers_after_slowdown_ends():
    ctl, lv = run(32, 4, 1.0, 4.0, steps=900, slow_from=200, slow_until=400, slow_factor=3.0, probe_period=32)
    assert lv[199] == 7 and min(lv[200:420]) == 2 and lv[-1] == 7
