"""Endurance at the benchmark's shape, collected after the parity tests so that a long soak cannot hide them.

Four layers of the 7B workload, 1 500 decode steps.  The host-resident fraction follows a fixed schedule of
levels (nothing the box measures decides it), the monitoring mode and the swap path rotate, and the adaptive
controller is fed every timed step's measurements (its answer is not used: what it decides depends on the box's
timings and is tested elsewhere under an injected timing model).  The inputs are the same every step, so every
step's output must equal the first one's bit for bit; no device error flag may appear; the process's resident
memory must not grow; and whether a step found its first layer staged by the step before is predicted exactly
from the schedule: it must, when the step before ran with the same non-empty prefetch list and no block moved in
between, and must not otherwise.
"""
import numpy as np
import pytest
import torch

from paper_2411_09317_amd import binding as B
from paper_2411_09317_amd import inputs as I
from paper_2411_09317_amd import workload as WL

pytestmark = pytest.mark.gpu

UNITS = 8 * 32
LEVELS = (0, 3, 1, 6, 2, 10, 0, 4, 9, 5)      # level held for HOLD steps each, in turn; level / UNITS of the blocks
HOLD = 37


def test_many_steps_with_changing_residency_monitoring_and_swap_path_stay_bit_identical():
    w = I.CONFIGS["cfg3"]
    dw = WL.build(w, host_capacity_fraction=0.05, n_layers=4)
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    none = np.zeros(0, dtype=np.int32)
    ctl = B.Controller(UNITS, max(LEVELS), plateau_eps=0.5 / UNITS)
    try:
        dw.pool.set_host_fraction(0.0, dw.order, streams[1])
        dw.pool.sync()
        dw.pool.step(dw.q, dw.k_new, dw.v_new, dw.d_table, dw.d_ctx, none, none, dw.out, *streams)
        dw.pool.sync()
        ref = dw.out.clone()
        rss = lambda: int(open("/proc/self/statm").read().split()[1]) * 4096
        level, n_moves, hits, expected_hits, rss0 = 0, 0, 0, 0, None
        prev_pf = None                                   # the list the step before ran with; None after a move
        for step in range(1500):
            mode = (B.TIMING_CLOCK, B.TIMING_CLOCK, B.TIMING_EVENTS, B.TIMING_OFF)[(step // 100) % 4]
            dw.pool.set_timing(mode)
            dw.pool.set_swap_path((B.SWAP_DMA, B.SWAP_AUTO, B.SWAP_KERNEL)[(step // 250) % 3])
            new_level = LEVELS[(step // HOLD) % len(LEVELS)]
            if new_level != level:
                dw.pool.set_host_fraction(new_level / UNITS, dw.order, streams[1])
                dw.pool.sync()
                level, n_moves, prev_pf = new_level, n_moves + 1, None
            pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
            assert (len(pf) > 0) == (level > 0)
            expect = prev_pf is not None and len(pf) > 0 and np.array_equal(pf, prev_pf)
            dw.pool.step(dw.q, dw.k_new, dw.v_new, dw.d_table, dw.d_ctx, pf, dirty, dw.out, *streams)
            dw.pool.sync()
            st = dw.pool.stats()
            assert bool(st.first_layer_prestaged) == expect, (step, level, st.first_layer_prestaged, expect)
            hits += st.first_layer_prestaged
            expected_hits += int(expect)
            prev_pf = pf
            if mode != B.TIMING_OFF:                     # coverage of the monitoring -> controller path
                f = ctl.update_from_pool(dw.pool, w.batch / max(st.step_ms, 1e-3) * st.expansion_simple)
                assert 0.0 <= f <= max(LEVELS) / UNITS + 1e-6
            if step % 25 == 0:
                assert torch.equal(dw.out, ref), f"output changed at step {step}"
            if step == 300:
                rss0 = rss()
        assert torch.equal(dw.out, ref)
        assert dw.pool.check_errors() == 0
        assert n_moves == sum(1 for i in range(1, (1500 + HOLD - 1) // HOLD)
                              if LEVELS[i % len(LEVELS)] != LEVELS[(i - 1) % len(LEVELS)])
        assert hits == expected_hits and hits > 1000
        assert rss() - rss0 < 16 << 20
    finally:
        ctl.close()
        dw.pool.close()
