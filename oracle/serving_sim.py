"""Iteration-level scheduling over a block budget, restated as a plain simulation.

The paper's serving layer (Section 4.1) inherits iteration-level scheduling
from the engine it extends: requests wait in arrival order, join the running
batch when the cache can hold them, produce one token per iteration and
return their blocks when they end; expanding the cache shows the scheduler
more blocks, shrinking it hides blocks first and frees them later.  The
readings this build adds (admission by whole-life reservation, hence no
preemption; a shrink only stops admissions) are the ones the product
scheduler documents.

This model knows nothing of pools, handles or residency: it only counts.  One
tick = one iteration.  It returns, per iteration, which requests ran, so that
the product scheduler can be compared with it decision by decision.

TEST INFRASTRUCTURE ONLY - never imported by the product path.
"""
from __future__ import annotations

import math


def simulate(arrival_iter, prompt_len, output_len, n_gpu_blocks, unit_blocks, level_at, block_tokens=16,
             max_batch=1 << 30):
    """arrival_iter[i]: first iteration request i may join (non-decreasing); level_at(it) -> budget level at
    iteration `it`.  Returns a list of (iteration, ids that decoded a token in it in admission order, blocks
    they held meanwhile, blocks promised to them), and the admission and last iteration of every request."""
    n = len(arrival_iter)
    life = [math.ceil((prompt_len[i] + output_len[i]) / block_tokens) for i in range(n)]
    gen = [0] * n
    admitted, finished = [-1] * n, [-1] * n
    running, nxt, promised, it, trace = [], 0, 0, 0, []
    while nxt < n or running:
        capacity = n_gpu_blocks + level_at(it) * unit_blocks
        while (nxt < n and arrival_iter[nxt] <= it and len(running) < max_batch
               and promised + life[nxt] <= capacity):
            promised += life[nxt]
            admitted[nxt] = it
            running.append(nxt)
            nxt += 1
        if not running:
            if arrival_iter[nxt] <= it:
                raise ValueError(f"request {nxt} can never be admitted")
            it = arrival_iter[nxt]           # idle until the next arrival
            continue
        held = sum(math.ceil((prompt_len[i] + gen[i] + 1) / block_tokens) for i in running)
        trace.append((it, list(running), held, promised))
        still = []
        for i in running:
            gen[i] += 1
            if gen[i] == output_len[i]:
                finished[i] = it
                promised -= life[i]
            else:
                still.append(i)
        running = still
        it += 1
    return trace, admitted, finished
