"""Adaptive expansion as a step-by-step simulation (paper Section 3.4.2, with
the three growth conditions of Section 1).

The paper gives the rules in prose and no constants; this is the reading taken:

  * The amount of swapping is an integer level k; the host-resident fraction is
    f = k / units (one unit = one layer's worth when units = n_layers, the
    paper moves a single layer per decision).  The run starts at k = 0.
  * After every decode step the controller is shown, per layer, the attention
    time, the swap-in time and the time compute waited for a swap, plus the
    link utilisation and the step's throughput.
  * A step is *bad* when swapping was not hidden: some layer's swap-in took
    longer than its compute, or the summed waits exceed stall_eps of the summed
    compute.  k_down consecutive bad steps move one unit back to the GPU and
    remember that level as a ceiling; fewer are tolerated as brief
    interference.
  * After k_up consecutive good steps the level counts as sustained and its mean
    throughput is recorded.  If the level was reached by growing and the record
    is not at least (1 + plateau_eps) times the record one level below, the
    workload has stopped scaling: go back one level and set the ceiling there.
  * Otherwise grow by one unit, provided (1) the link is not saturated
    (utilisation < util_max), (2) the swap-in time extrapolated linearly to the
    next level stays within rho x compute for every layer, (3) the next level is
    below the ceiling, or the ceiling is older than probe_period steps (then it
    is cleared: the periodic upward probe), and k < k_max.

It is a heuristic, so the GPU library's controller is compared with this
simulation decision by decision under an injected timing model; on hardware only
the invariant and the fixed point are checked.

TEST INFRASTRUCTURE ONLY - never imported by the product path.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence


@dataclass
class Observation:
    t_attn: Sequence[float]
    t_in: Sequence[float]
    t_stall: Sequence[float]
    link_util: float
    throughput: float


@dataclass
class AdaptiveExpansion:
    units: int
    k_max: int
    rho: float = 0.9
    k_up: int = 4
    k_down: int = 2
    probe_period: int = 64
    plateau_eps: float = 0.01
    util_max: float = 0.9
    stall_eps: float = 0.01

    k: int = 0
    clean: int = 0
    bad: int = 0
    ceiling: Optional[int] = None
    since_ceiling: int = 0
    grew: bool = False
    win_sum: float = 0.0
    win_n: int = 0
    rec: Dict[int, float] = field(default_factory=dict)

    @property
    def host_fraction(self) -> float:
        return self.k / self.units

    def _set_level(self, k: int, grew: bool) -> None:
        self.k = k
        self.grew = grew
        self.clean = 0
        self.bad = 0
        self.win_sum = 0.0
        self.win_n = 0

    def observe(self, o: Observation) -> int:
        """Feed one step's measurements; returns the level for the next step."""
        if self.ceiling is not None:
            self.since_ceiling += 1
        tot_attn = 0.0
        tot_stall = 0.0
        over = False
        for a, i, s in zip(o.t_attn, o.t_in, o.t_stall):
            tot_attn += a
            tot_stall += s
            if i > a:
                over = True
        is_bad = self.k > 0 and (over or tot_stall > self.stall_eps * tot_attn)
        if is_bad:
            self.bad += 1
            self.clean = 0
        else:
            self.clean += 1
            self.bad = 0
            self.win_sum += o.throughput
            self.win_n += 1

        if self.bad >= self.k_down:                      # shrink: compute had to wait
            self.ceiling = self.k
            self.since_ceiling = 0
            self._set_level(self.k - 1, False)
            return self.k
        if self.clean < self.k_up:
            return self.k

        self.rec[self.k] = self.win_sum / self.win_n     # level sustained
        if self.grew and (self.k - 1) in self.rec:
            if self.rec[self.k] < self.rec[self.k - 1] * (1.0 + self.plateau_eps):
                self.ceiling = self.k                    # stopped scaling: step back, hold
                self.since_ceiling = 0
                self._set_level(self.k - 1, False)
                return self.k
        self.grew = False

        if self.k >= self.k_max:
            return self.k
        if o.link_util >= self.util_max:
            return self.k
        if self.ceiling is not None and self.k + 1 >= self.ceiling:
            if self.since_ceiling < self.probe_period:
                return self.k
        if self.k > 0:
            for a, i in zip(o.t_attn, o.t_in):
                if i * (self.k + 1) / self.k > self.rho * a:
                    return self.k
        if self.ceiling is not None and self.k + 1 >= self.ceiling:
            self.ceiling = None                          # periodic upward probe
        self._set_level(self.k + 1, True)
        return self.k


def simulate(ctl: AdaptiveExpansion, timing: Callable[[int, int], Observation], n_steps: int) -> List[int]:
    """Run the controller against a timing model (level, step index) -> Observation.
    Returns the level in force during each step."""
    levels = []
    for step in range(n_steps):
        levels.append(ctl.k)
        ctl.observe(timing(ctl.k, step))
    return levels


def linear_timing(n_layers: int, units: int, c: float, s: float, tput_gain: float = 1.0,
                  slow_from: Optional[int] = None, slow_until: Optional[int] = None, slow_factor: float = 1.0):
    """Timing model for tests: every layer computes in c, a swap-in of the whole
    layer would take s (so a fraction f takes f*s), compute waits for whatever
    does not fit, and throughput follows 1/(1-f) scaled by tput_gain (0 = a
    workload that does not benefit from more memory).  Between steps slow_from
    and slow_until the link is slow_factor times slower."""
    def timing(k: int, step: int) -> Observation:
        f = k / units
        s_now = s * slow_factor if (slow_from is not None and slow_from <= step < (slow_until or 1 << 60)) else s
        t_in = f * s_now
        stall = max(0.0, t_in - c)
        step_time = n_layers * (c + stall)
        expansion = 1.0 / (1.0 - f) if f < 1.0 else float("inf")
        tput = (1.0 + tput_gain * (expansion - 1.0)) / step_time
        return Observation([c] * n_layers, [t_in] * n_layers, [stall] * n_layers,
                           min(1.0, t_in / (c + stall)), tput)
    return timing
