"""Iteration-level request scheduling over the split KV cache.

What the paper builds on top of its swapping layer (Section 4.1: a block
manager with a free list that hands blocks out on demand and takes them back
when a request ends; the scheduler sees more blocks when the cache is
expanded and fewer when it shrinks) reduced to what the decode path needs:
requests arrive (Evaluation setup: Poisson arrivals), wait first come first
served until the cache can hold them, decode one token per iteration together
with every other running request, and leave.  Expansion turns into batch size
here: the blocks a `BlockBudget` promises are the GPU pool plus `level` units
of host blocks.

Grow and shrink.  The paper makes new blocks visible only after every layer's
cache has been moved to its larger allocation, and on shrinking hides blocks
from the scheduler before it frees them.  A block-granular cache has no
contiguous per-layer allocation to move, so growth is visible at once; the
shrink rule is kept as stated: the budget drops at once (nothing new is
admitted against the hidden blocks), running requests keep what they hold, and
host blocks are given up as requests end or as their blocks find room in the
GPU pool (`Scheduler.promote`).

There is no model and no prefill here: a request's prompt is taken as already
in the cache (its blocks hold whatever the pool was filled with), and every
iteration appends one synthetic key/value row per running request.  The
scheduler is plain host logic over a block store with the methods of
`binding.Pool` (block_alloc, block_free, block_where, n_free, migrate).
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass, field
from typing import Deque, List, Optional

import numpy as np

GPU, HOST = 0, 1


@dataclass
class Request:
    rid: int
    arrival: float
    prompt_len: int
    output_len: int
    admitted: float = -1.0
    finished: float = -1.0
    generated: int = 0
    handles: List[int] = field(default_factory=list)
    row: Optional[np.ndarray] = None      # its block-table row, kept up to date as blocks are added

    @property
    def ctx(self) -> int:
        """Context length of the coming iteration, the token being decoded included."""
        return self.prompt_len + self.generated + 1


class BlockBudget:
    """Blocks the scheduler may promise: n_gpu_blocks + level * unit_blocks."""

    def __init__(self, n_gpu_blocks: int, unit_blocks: int, k_max: int):
        if n_gpu_blocks <= 0 or unit_blocks < 0 or k_max < 0:
            raise ValueError("bad budget")
        self.n_gpu, self.unit, self.k_max = n_gpu_blocks, unit_blocks, k_max
        self.level = 0

    def set_level(self, k: int):
        if not 0 <= k <= self.k_max:
            raise ValueError(f"level {k} outside [0, {self.k_max}]")
        self.level = k

    @property
    def capacity(self) -> int:
        return self.n_gpu + self.level * self.unit

    @property
    def expansion(self) -> float:
        return self.capacity / self.n_gpu


class Scheduler:
    """First come first served, one token per running request per iteration.

    A request is admitted when the blocks of its whole life (prompt + output) fit under the budget beside
    those promised to the requests already running; they are allocated as its context grows, from the GPU
    pool while that has a free slot, else from the host pool.  Nothing is ever preempted."""

    def __init__(self, store, block_tokens: int, budget: BlockBudget, max_batch: int, max_blocks_per_seq: int,
                 migrate_stream=None):
        self.store, self.T, self.budget = store, block_tokens, budget
        self.max_batch, self.max_blocks = max_batch, max_blocks_per_seq
        self.migrate_stream = migrate_stream
        self.waiting: Deque[Request] = deque()
        self.running: List[Request] = []
        self.done: List[Request] = []
        self.reserved = 0                      # blocks promised to running requests
        self.on_host = set()                   # handles in use that are homed in the host pool
        self.n_promoted = 0

    # ---- admission ---------------------------------------------------------------------------
    def lifetime_blocks(self, r: Request) -> int:
        return (r.prompt_len + r.output_len + self.T - 1) // self.T

    def submit(self, r: Request):
        if self.lifetime_blocks(r) > self.max_blocks:
            raise ValueError(f"request {r.rid} needs more blocks than a block-table row holds")
        self.waiting.append(r)

    def _alloc(self, n: int) -> List[int]:
        g = min(n, self.store.n_free(GPU))
        hs = list(self.store.block_alloc(GPU, g)) if g else []
        if n > g:
            more = list(self.store.block_alloc(HOST, n - g))
            self.on_host.update(more)
            hs += more
        return hs

    def admit(self, now: float) -> int:
        n = 0
        while self.waiting and len(self.running) < self.max_batch:
            r = self.waiting[0]
            need = self.lifetime_blocks(r)
            if r.arrival > now or self.reserved + need > self.budget.capacity:
                break
            self.waiting.popleft()
            self.reserved += need
            r.admitted = now
            r.handles = self._alloc((r.ctx + self.T - 1) // self.T)
            r.row = np.full(self.max_blocks, -1, dtype=np.int32)
            r.row[:len(r.handles)] = r.handles
            self.running.append(r)
            n += 1
        return n

    # ---- residency ----------------------------------------------------------------------------
    def promote(self, limit: Optional[int] = None) -> int:
        """Re-home host blocks in free GPU slots: what has room on the GPU is not read over the link every
        iteration.  The blocks in the highest host slots go first, and new ones take the lowest free slot, so
        the host pool stays a dense prefix with few holes and a layer's prefetch is a few long copies."""
        n = min(self.store.n_free(GPU), len(self.on_host))
        if limit is not None:
            n = min(n, limit)
        if n <= 0:
            return 0
        cand = sorted(self.on_host)
        _, slots = self.store.block_where(cand)
        hs = [h for _, h in sorted(zip(slots, cand), reverse=True)[:n]]
        if self.migrate_stream is not None:
            self.store.migrate(hs, GPU, self.migrate_stream)
        else:
            self.store.migrate(hs, GPU)
        self.on_host.difference_update(hs)
        self.n_promoted += n
        return n

    def relocate(self, src, dst):
        """The blocks src[i] now live at dst[i] (someone has moved the bytes): tables follow."""
        to = dict(zip(src, dst))
        for r in self.running:
            if any(h in to for h in r.handles):
                r.handles = [to.get(h, h) for h in r.handles]
                r.row[:len(r.handles)] = r.handles
        self.store.relocate(src, dst)

    @property
    def blocks_in_use(self) -> int:
        return sum(len(r.handles) for r in self.running)

    # ---- one iteration ---------------------------------------------------------------------------
    def tables(self):
        """Block table int32 [batch][max_blocks] (-1 = unused) and context lengths int32 [batch]."""
        if not self.running:
            return np.zeros((0, self.max_blocks), dtype=np.int32), np.zeros(0, dtype=np.int32)
        table = np.stack([r.row for r in self.running])
        ctx = np.fromiter((r.ctx for r in self.running), dtype=np.int32, count=len(self.running))
        return table, ctx

    def complete_iteration(self, now: float) -> int:
        """Every running request has decoded one token; finished ones return their blocks, the others get
        the block their next token needs.  Returns the number of tokens produced."""
        still = []
        n = len(self.running)
        for r in self.running:
            r.generated += 1
            if r.generated >= r.output_len:
                r.finished = now
                self.store.block_free(r.handles)
                self.on_host.difference_update(r.handles)
                self.reserved -= self.lifetime_blocks(r)
                r.handles, r.row = [], None
                self.done.append(r)
            else:
                still.append(r)
        self.running = still
        for r in self.running:                 # after the frees, so that a freed GPU slot is reused at once
            if (r.ctx + self.T - 1) // self.T > len(r.handles):
                r.row[len(r.handles)] = (h := self._alloc(1))[0]
                r.handles += h
        return n

    @property
    def idle(self) -> bool:
        return not self.running and not self.waiting


def summarize(done: List[Request], makespan: float) -> dict:
    """Throughput and the latency split the paper reports (queueing before admission, decoding after)."""
    if not done:
        return {"requests": 0}
    q = np.array([r.admitted - r.arrival for r in done])
    s = np.array([r.finished - r.admitted for r in done])
    tok = np.array([r.output_len for r in done])
    return {"requests": len(done), "tokens": int(tok.sum()), "makespan_s": makespan,
            "tokens_per_s": float(tok.sum() / makespan) if makespan > 0 else 0.0,
            "queue_s_mean": float(q.mean()), "queue_s_p90": float(np.percentile(q, 90)),
            "decode_s_mean": float(s.mean()), "decode_ms_per_token_mean": float((s / tok).mean() * 1e3),
            "latency_s_mean": float((q + s).mean()), "latency_s_p90": float(np.percentile(q + s, 90))}


class DeviceLoop:
    """Runs a scheduler's iterations on the library: per iteration the block table and context lengths go to
    the device, the host-homed blocks the batch touches are listed, and one `pie_step` decodes a token for
    every running request.  Queries and new key/value rows are random (there is no model); time is the
    measured wall time of the iterations, so arrivals interact with the real speed of the path."""

    def __init__(self, pool, w, max_batch: int, max_blocks: int, device: str = "cuda:0"):
        import torch
        from . import workload as WL
        self.torch, self.pool, self.w = torch, pool, w
        self.max_batch, self.max_blocks = max_batch, max_blocks
        gen = torch.Generator(device=device)
        gen.manual_seed(w.seed + 17)
        dt = WL.TORCH_DT[w.dtype]
        draw = lambda *s: (torch.randn(*s, device=device, dtype=torch.float32, generator=gen) * w.value_scale).to(dt)
        self.q = draw(w.n_layers * max_batch * w.n_q_heads * w.head_dim)
        self.k_new = draw(w.n_layers * max_batch * w.n_kv_heads * w.head_dim)
        self.v_new = draw(w.n_layers * max_batch * w.n_kv_heads * w.head_dim)
        self.out = torch.zeros_like(self.q)
        self.h_table = torch.empty((max_batch, max_blocks), dtype=torch.int32, pin_memory=True)
        self.h_ctx = torch.empty(max_batch, dtype=torch.int32, pin_memory=True)
        self.d_table = torch.empty((max_batch, max_blocks), dtype=torch.int32, device=device)
        self.d_ctx = torch.empty(max_batch, dtype=torch.int32, device=device)
        self.streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())

    def iteration(self, sched: Scheduler, step=None):
        """One decode iteration of everything running; returns (seconds, host blocks read per layer).  `step`:
        another pool's step with the argument list of pie_layer_step (no prefetch lists), instead of pie_step."""
        import time
        torch, w = self.torch, self.w
        table, ctx = sched.tables()
        B = len(ctx)
        self.h_table[:B].copy_(torch.from_numpy(table))
        self.h_ctx[:B].copy_(torch.from_numpy(ctx))
        t0 = time.perf_counter()
        with torch.cuda.stream(self.streams[0]):
            self.d_table[:B].copy_(self.h_table[:B], non_blocking=True)
            self.d_ctx[:B].copy_(self.h_ctx[:B], non_blocking=True)
        shape = lambda t, h: t[: w.n_layers * B * h * w.head_dim].view(w.n_layers, B, h, w.head_dim)
        if step is not None:
            step(shape(self.q, w.n_q_heads), shape(self.k_new, w.n_kv_heads), shape(self.v_new, w.n_kv_heads),
                 self.d_table[:B], self.d_ctx[:B], shape(self.out, w.n_q_heads), *self.streams)
            self.pool.sync()
            return time.perf_counter() - t0, 0
        pf, dirty = self.pool.prefetch_list(table, ctx)
        self.last_runs = 0
        if len(pf):                                # pieces the layer's prefetch falls into (the list is in slot order)
            slots = np.asarray(self.pool.block_where(pf)[1])
            self.last_runs = 1 + int((np.diff(slots) != 1).sum())
        self.pool.step(shape(self.q, w.n_q_heads), shape(self.k_new, w.n_kv_heads), shape(self.v_new, w.n_kv_heads),
                       self.d_table[:B], self.d_ctx[:B], pf, dirty, shape(self.out, w.n_q_heads), *self.streams)
        self.pool.sync()
        return time.perf_counter() - t0, len(pf)


def serve(pool, w, requests: List[Request], budget: BlockBudget, max_batch: int, max_blocks: int, controller=None,
          promote_limit: Optional[int] = None, progress=None) -> dict:
    """Serves a request stream to completion on the GPU.  With a controller (binding.Controller whose levels
    are the budget's) the level follows the per-layer timings of every iteration; else it stays where the
    budget was set."""
    loop = DeviceLoop(pool, w, max_batch, max_blocks)
    sched = Scheduler(pool, w.block_tokens, budget, max_batch, max_blocks, migrate_stream=loop.streams[1])
    for r in requests:
        sched.submit(r)
    pool.set_timing(2 if controller is not None else 0)        # monitoring by device clock: no gaps between kernels
    now, iters, batch_sum, host_sum, run_sum, busy, levels, recent = 0.0, 0, 0, 0, 0, 0.0, [], []
    while not sched.idle:
        sched.admit(now)
        sched.promote(promote_limit)
        if not sched.running:
            now = max(now, sched.waiting[0].arrival)
            continue
        dt, n_host = loop.iteration(sched)
        B = len(sched.running)
        now += dt
        busy += dt
        iters += 1
        batch_sum += B
        host_sum += n_host
        run_sum += loop.last_runs
        if controller is not None:
            recent.append((B, dt))                 # tokens/s over the last few iterations: single ones are noisy
            del recent[:-8]
            rate = sum(b for b, _ in recent) / sum(t for _, t in recent)
            # per promised block x the blocks the level allows: what it gives once the scheduler has filled it
            f = controller.update_from_pool(pool, rate * budget.capacity / max(sched.reserved, 1))
            budget.set_level(min(budget.k_max, int(round(f * controller.units))))
            levels.append(budget.level)
        sched.complete_iteration(now)
        if progress and iters % 500 == 0:
            progress(iters, now, len(sched.done))
    pool.set_timing(0)
    flags = pool.check_errors()
    if flags:
        raise RuntimeError(f"device error flags {flags:#x} while serving")
    res = summarize(sched.done, now)
    res.update({"iterations": iters, "mean_batch": batch_sum / max(iters, 1), "ms_per_iteration": busy / max(iters, 1) * 1e3,
                "host_blocks_per_iteration": host_sum / max(iters, 1),
                "host_runs_per_iteration": run_sum / max(iters, 1), "blocks_promoted": sched.n_promoted,
                "level_final": budget.level, "capacity_blocks": budget.capacity, "expansion": budget.expansion})
    if levels:
        res["level_mean"] = float(np.mean(levels))
        res["level_max"] = int(max(levels))
    return res


# ---- the same on layer caches that grow and shrink (the paper's own unit) ------------------------------------

class IndexStore:
    """Blocks as indices into a layer's cache (the same index in every layer), lowest free index first, below
    a limit that moves with the caches' size.  Has the block-store methods the scheduler uses; every block
    counts as GPU-homed (in this unit whole layers move, not blocks)."""

    def __init__(self, n_indices: int, limit: int):
        self.used = np.zeros(n_indices, dtype=bool)
        self.limit = limit

    def n_free(self, where: int) -> int:
        return int(self.limit - self.used[: self.limit].sum()) if where == GPU else 0

    def block_alloc(self, where: int, n: int) -> List[int]:
        if n == 0:
            return []
        idx = np.flatnonzero(~self.used[: self.limit])[:n]
        if where != GPU or len(idx) < n:
            raise MemoryError("no free block below the limit")
        self.used[idx] = True
        return idx.tolist()

    def block_free(self, handles):
        self.used[np.asarray(handles, dtype=np.int64)] = False

    def block_where(self, handles):
        return [GPU] * len(handles), list(handles)

    def plan_compaction(self, below: int):
        """Live indices at or above `below` paired with the lowest free indices under it; None if they do not
        all fit."""
        src = np.flatnonzero(self.used[below:]) + below
        dst = np.flatnonzero(~self.used[:below])[: len(src)]
        return (src.tolist(), dst.tolist()) if len(dst) == len(src) else None

    def relocate(self, src, dst):
        self.used[np.asarray(src, dtype=np.int64)] = False
        self.used[np.asarray(dst, dtype=np.int64)] = True

    def live_end(self) -> int:
        nz = np.flatnonzero(self.used)
        return int(nz[-1]) + 1 if len(nz) else 0


class VisibleBudget:
    """What the scheduler may promise = what the elastic pool shows."""

    def __init__(self, elastic, base_blocks: int):
        self.ep, self.base = elastic, base_blocks

    @property
    def capacity(self) -> int:
        return self.ep.capacity()[0]

    @property
    def expansion(self) -> float:
        return self.capacity / self.base


def serve_elastic(elastic, w, requests: List[Request], max_batch: int, max_blocks: int, controller=None,
                  layers_on_cpu: int = 0, progress=None) -> dict:
    """Serves a request stream on an elastic pool (binding.ElasticPool).  The number of layers kept in CPU memory
    is fixed (`layers_on_cpu`) or follows a controller (binding.Controller over levels = layers) that sees,
    per token, whether computation waited for a layer.  A shrink that is refused hides the blocks at once; it
    is asked for again every iteration until the blocks above the new size have been given up."""
    pool = elastic.pool
    base = pool.cfg.n_gpu_blocks
    n = elastic.n_layers
    loop = DeviceLoop(pool, w, max_batch, max_blocks)
    store = IndexStore(elastic.k_cap * elastic.C, base)
    budget = VisibleBudget(elastic, base)
    sched = Scheduler(store, w.block_tokens, budget, max_batch, max_blocks)
    for r in requests:
        sched.submit(r)
    cs = loop.streams[0]
    want = layers_on_cpu
    now, iters, batch_sum, busy, levels, sizes, recent, prev_stall, refused, moved = 0.0, 0, 0, 0.0, [], [], [], 0.0, 0, 0
    while not sched.idle:
        vis, tgt, m = elastic.capacity()
        if want != m:
            # what must fit below a smaller size: the live blocks, and the blocks promised to running requests;
            # live blocks scattered above it are moved down first if the promise already fits
            below = elastic.blocks_for(want)
            if want < m and sched.reserved <= below < store.live_end():
                plan = store.plan_compaction(below)
                if plan and plan[0]:
                    elastic.move_blocks(plan[0], plan[1], cs)
                    sched.relocate(*plan)
                    moved += len(plan[0])
            if elastic.set_layers_on_cpu(want, max(store.live_end(), sched.reserved), cs):
                vis, tgt, m = elastic.capacity()
            else:
                refused += 1
        # blocks that exist in every layer right now: while a shrink is pending the caches are still large
        store.limit = max(store.limit, vis) if want < m else vis
        sched.admit(now)
        if not sched.running:
            now = max(now, sched.waiting[0].arrival)
            continue
        elastic.set_live_blocks(store.live_end())
        dt, _ = loop.iteration(sched, step=elastic.step)
        B = len(sched.running)
        now += dt
        busy += dt
        iters += 1
        batch_sum += B
        levels.append(m)
        sizes.append(vis)
        if controller is not None:
            st = elastic.stats()
            stall, prev_stall = st.stall_ms - prev_stall, st.stall_ms
            recent.append((B, dt))
            del recent[:-8]
            tc = (dt * 1e3 - stall) / n
            # tokens/s per promised block x the blocks the level leads to: what the level will give once the
            # scheduler has filled it, without waiting for the admissions to catch up
            rate = sum(b for b, _ in recent) / sum(t for _, t in recent)
            want = controller.observe([tc] * n, [0.0] * n, [stall / n] * n, 0.0, rate * tgt / max(sched.reserved, 1))
        sched.complete_iteration(now)
        if progress and iters % 500 == 0:
            progress(iters, now, len(sched.done))
    flags = pool.check_errors()
    if flags:
        raise RuntimeError(f"device error flags {flags:#x} while serving")
    res = summarize(sched.done, now)
    st = elastic.stats()
    res.update({"iterations": iters, "mean_batch": batch_sum / max(iters, 1), "ms_per_iteration": busy / max(iters, 1) * 1e3,
                "layers_on_cpu_mean": float(np.mean(levels)) if levels else 0.0,
                "layers_on_cpu_max": int(max(levels)) if levels else 0,
                "blocks_per_layer_mean": float(np.mean(sizes)) if sizes else 0.0,
                "blocks_per_layer_max": int(max(sizes)) if sizes else 0, "blocks_per_layer_base": base,
                "shrinks_refused": refused, "blocks_moved_down": moved, "swap_ins": int(st.n_swap_in), "swap_outs": int(st.n_swap_out),
                "forced_ins": int(st.n_forced_in), "host_wait_ms": float(st.stall_ms)})
    return res
