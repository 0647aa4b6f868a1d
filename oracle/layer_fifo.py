"""The paper's layer-granular swapping protocol as a discrete-event simulation.

Follows Section 3.2 (mapping table: logical layer -> CPU pointer, GPU pointer,
timestamps; two-phase update; presence check before a layer is computed) and
Section 3.3 (the protocol run at the beginning of every layer's computation):

  * if the previous swap-in has finished, start a swap-in of the hottest layer
    in CPU memory - the one that will be accessed soonest - provided a GPU
    layer slot is free;
  * if the previous swap-out has finished, start a swap-out of the coldest
    layer on the GPU - the one whose next access is farthest away, which is the
    layer that has just finished computing - provided a CPU layer slot is free;
    not if every layer currently in CPU memory is colder than that layer;
  * before computing layer k, if it is not physically present on the GPU, wait
    until it has been moved back completely.

Readings where the text is silent: the swap-in check is made first, then the
swap-out check, and a swap-out is only started when no GPU slot is free - its
purpose is to make room for the next swap-in (in the worked example the freed
space of layer 1 takes layer 8 while layer 3 starts to leave: both orders give
the example's trace, but only this one lets the layers drain back onto the GPU
when slots are added); "coldness" is the
number of layer computations until the next access, (j - k) mod n for layer j
while layer k computes; a layer in flight in either direction is neither a
swap-out candidate nor counted as "in CPU memory"; a swap-out's GPU slot is
released when the copy has completed (phase two), a swap-in's CPU slot
likewise; a layer that is needed while it is neither present nor on its way is
brought back at once (waiting for the link and, if necessary, for a slot), and
that wait is counted as stall.

Adaptive expansion in the paper's own unit (Section 3.4.2: start with all layers
on the GPU, put more layers into swapping while computation does not wait, move
one back when it does): the number of GPU layer slots in use can be changed
between tokens (set_gpu_slots).  Taking a slot away retires a free slot, or the
next one that a completed swap-out frees; while more GPU slots are occupied than
allowed, the swap-out exception ("everything in CPU memory is colder") is not
applied, since the point is to move a layer out.  Giving a slot back puts a
retired slot on the free list; the next swap-in fills it.

Time is in arbitrary units; one layer computes in t_compute, one layer moves
in t_in / t_out.  Layers are numbered 0 .. n-1 here (the paper's 1 .. n).

TEST INFRASTRUCTURE ONLY - never imported by the product path.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

GPU, HOST, MOVING_OUT, MOVING_IN = "gpu", "host", "out", "in"


@dataclass
class Entry:
    """One row of the mapping table."""
    state: str
    gpu_slot: Optional[int] = None
    host_slot: Optional[int] = None
    t_out_start: Optional[float] = None     # timestamps of the last moves
    t_out_done: Optional[float] = None
    t_in_start: Optional[float] = None
    t_in_done: Optional[float] = None


@dataclass
class Record:
    """What happened at the beginning of one layer's computation."""
    token: int
    layer: int
    t_begin: float                  # when the compute stream reached the layer
    t_start: float                  # when its computation started (after any wait)
    out_started: Optional[int] = None
    in_started: Optional[int] = None
    out_skipped: Optional[str] = None      # "busy" | "no_slot" | "colder_on_host" | "room_left" | "none"
    in_skipped: Optional[str] = None       # "busy" | "no_slot" | "none"
    forced_in: bool = False


@dataclass
class Result:
    records: List[Record] = field(default_factory=list)
    residences: List[tuple] = field(default_factory=list)    # (layer, t_out_start, t_in_done)
    stall: float = 0.0
    max_away: int = 0               # most layers simultaneously not plainly resident on the GPU
    table: Dict[int, Entry] = field(default_factory=dict)


class LayerFifo:
    def __init__(self, n_layers: int, n_gpu_slots: int, n_host_slots: int, on_host: List[int]):
        if n_layers <= 0 or n_gpu_slots <= 0 or n_host_slots < 0:
            raise ValueError("sizes")
        on_host = sorted(set(int(x) for x in on_host))
        if any(x < 0 or x >= n_layers for x in on_host):
            raise ValueError("layer out of range")
        if len(on_host) > n_host_slots or n_layers - len(on_host) > n_gpu_slots:
            raise ValueError("placement does not fit")
        self.n = n_layers
        self.free_gpu = list(range(n_gpu_slots))
        self.free_host = list(range(n_host_slots))
        self.table: Dict[int, Entry] = {}
        for j in range(n_layers):                    # lowest free slot first, in layer order
            if j in on_host:
                self.table[j] = Entry(HOST, host_slot=self.free_host.pop(0))
            else:
                self.table[j] = Entry(GPU, gpu_slot=self.free_gpu.pop(0))
        self.moving_in: Optional[int] = None         # at most one swap-in and one swap-out in flight
        self.moving_out: Optional[int] = None
        self.n_gpu_total = n_gpu_slots
        self.n_host_total = n_host_slots
        self.n_enabled = n_gpu_slots                 # GPU slots in use or on the free list
        self.target = n_gpu_slots                    # how many are allowed
        self.retired: List[int] = []

    # ---- changing the number of GPU layer slots ------------------------------
    def _rebalance(self):
        while self.n_enabled > self.target and self.free_gpu:
            self.retired.append(self.free_gpu.pop())         # highest free slot
            self.retired.sort()
            self.n_enabled -= 1
        while self.n_enabled < self.target and self.retired:
            self.free_gpu.append(self.retired.pop(0))        # lowest retired slot
            self.free_gpu.sort()
            self.n_enabled += 1

    def set_gpu_slots(self, n: int):
        # the layers that do not fit the GPU slots need a CPU slot each, plus the two in flight
        if n < 1 or n > self.n_gpu_total or self.n - n + 2 > self.n_host_total:
            raise ValueError("slot count")
        self.target = n
        self._rebalance()

    @property
    def oversubscribed(self) -> bool:
        return self.n_enabled > self.target

    # ---- phase two of a move -------------------------------------------------
    def complete_in(self, now: float):
        j = self.moving_in
        e = self.table[j]
        self.free_host.append(e.host_slot)
        self.free_host.sort()
        e.host_slot, e.state, e.t_in_done = None, GPU, now
        self.moving_in = None
        return j

    def complete_out(self, now: float):
        j = self.moving_out
        e = self.table[j]
        self.free_gpu.append(e.gpu_slot)
        self.free_gpu.sort()
        e.gpu_slot, e.state, e.t_out_done = None, HOST, now
        self.moving_out = None
        self._rebalance()
        return j

    # ---- phase one -------------------------------------------------------------
    def start_in(self, j: int, now: float):
        e = self.table[j]
        assert e.state == HOST and self.moving_in is None and self.free_gpu
        e.gpu_slot, e.state, e.t_in_start = self.free_gpu.pop(0), MOVING_IN, now
        self.moving_in = j

    def start_out(self, j: int, now: float):
        e = self.table[j]
        assert e.state == GPU and self.moving_out is None and self.free_host
        e.host_slot, e.state, e.t_out_start = self.free_host.pop(0), MOVING_OUT, now
        self.moving_out = j

    def distance(self, j: int, k: int) -> int:
        """Layer computations until layer j is accessed, counted while layer k computes."""
        return (j - k) % self.n

    def hottest_on_host(self, k: int) -> Optional[int]:
        c = [j for j, e in self.table.items() if e.state == HOST]
        return min(c, key=lambda j: self.distance(j, k)) if c else None

    def coldest_on_gpu(self, k: int) -> Optional[int]:
        c = [j for j, e in self.table.items() if e.state == GPU and j != k]
        return max(c, key=lambda j: self.distance(j, k)) if c else None


def simulate(n_layers: int, n_gpu_slots: int, n_host_slots: int, on_host: List[int], n_tokens: int,
             t_compute: float = 1.0, t_in: float = 2.0, t_out: float = 2.0, gpu_slots_for_token=None) -> Result:
    """gpu_slots_for_token: optional callable (token index, stall of the previous token) -> number of GPU
    layer slots allowed from this token on (None = unchanged); called at every token boundary."""
    f = LayerFifo(n_layers, n_gpu_slots, n_host_slots, on_host)
    res = Result()
    now = 0.0
    in_done_at = out_done_at = None
    stall_prev = 0.0

    def retire(t):
        nonlocal in_done_at, out_done_at
        if out_done_at is not None and out_done_at <= t:
            j = f.complete_out(out_done_at)
            out_done_at = None
        if in_done_at is not None and in_done_at <= t:
            j = f.complete_in(in_done_at)
            res.residences.append((j, f.table[j].t_out_start, f.table[j].t_in_done))
            in_done_at = None

    for token in range(n_tokens):
        retire(now)
        if gpu_slots_for_token is not None:
            want = gpu_slots_for_token(token, res.stall - stall_prev)
            if want is not None:
                f.set_gpu_slots(want)
        stall_prev = res.stall
        for k in range(n_layers):
            retire(now)
            rec = Record(token, k, now, now)
            e = f.table[k]
            # presence check
            if e.state != GPU:
                if e.state == MOVING_OUT:                   # pathological: leaving while it is needed
                    now = max(now, out_done_at)
                    retire(now)
                if e.state == HOST:                         # needed, and not even on its way
                    if f.moving_in is not None:
                        now = max(now, in_done_at)
                        retire(now)
                    while not f.free_gpu:                   # a freed slot may be retired: then another layer goes
                        if f.moving_out is None:
                            victim = f.coldest_on_gpu(k)
                            f.start_out(victim, now)
                            out_done_at = now + t_out
                        now = max(now, out_done_at)
                        retire(now)
                    f.start_in(k, now)
                    in_done_at = now + t_in
                    rec.forced_in = True
                if f.table[k].state == MOVING_IN:
                    now = max(now, in_done_at)
                    retire(now)
                assert f.table[k].state == GPU
            res.stall += now - rec.t_begin
            rec.t_start = now
            # swap-in of the hottest layer in CPU memory
            if f.moving_in is not None:
                rec.in_skipped = "busy"
            else:
                cand = f.hottest_on_host(k)
                if cand is None:
                    rec.in_skipped = "none"
                elif not f.free_gpu:
                    rec.in_skipped = "no_slot"
                else:
                    f.start_in(cand, now)
                    in_done_at = now + t_in
                    rec.in_started = cand
            # swap-out of the coldest layer on the GPU
            if f.moving_out is not None:
                rec.out_skipped = "busy"
            else:
                cand = f.coldest_on_gpu(k)
                on_host_now = [j for j, x in f.table.items() if x.state == HOST]
                if cand is None:
                    rec.out_skipped = "none"
                elif not f.oversubscribed and all(f.distance(j, k) > f.distance(cand, k) for j in on_host_now):
                    rec.out_skipped = "colder_on_host"      # also when nothing is in CPU memory at all
                elif f.free_gpu:
                    rec.out_skipped = "room_left"           # a GPU slot is free: nothing has to leave
                elif not f.free_host:
                    rec.out_skipped = "no_slot"
                else:
                    f.start_out(cand, now)
                    out_done_at = now + t_out
                    rec.out_started = cand
            away = sum(1 for x in f.table.values() if x.state != GPU)
            res.max_away = max(res.max_away, away)
            res.records.append(rec)
            now += t_compute
    res.table = f.table
    return res


def simulate_adaptive(n_layers: int, n_host_slots: int, n_tokens: int, t_compute: float = 1.0, t_in: float = 2.0,
                      t_out: float = 2.0, k_up: int = 4, k_down: int = 2, probe_period: int = 64):
    """Adaptive expansion over the protocol: all layers start on the GPU; after every token the controller of
    oracle.controller_sim (level = layers meant to live in CPU memory) sees whether computation waited, and
    the number of GPU layer slots follows its level.  The throughput signal is 1 / token time x n / (n - m):
    more layers in CPU memory mean proportionally larger per-layer caches (Section 3.1).
    Returns (levels per token, Result)."""
    from .controller_sim import AdaptiveExpansion, Observation
    ctl = AdaptiveExpansion(units=n_layers, k_max=n_host_slots - 2, k_up=k_up, k_down=k_down, probe_period=probe_period)
    levels: List[int] = []
    state = {"t_token": None}

    def hook(token, stall_last):
        if token > 0:
            t_token = n_layers * t_compute + stall_last
            m = ctl.k
            per_layer = stall_last / n_layers
            ctl.observe(Observation([t_compute] * n_layers, [0.0] * n_layers, [per_layer] * n_layers, 0.0,
                                    (1.0 / t_token) * n_layers / (n_layers - m)))
        levels.append(ctl.k)
        return n_layers - ctl.k

    res = simulate(n_layers, n_layers, n_host_slots, [], n_tokens, t_compute, t_in, t_out, gpu_slots_for_token=hook)
    return levels, res
