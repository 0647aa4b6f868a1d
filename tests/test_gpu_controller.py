"""The adaptive-expansion controller in the loop on the GPU.

Attention-only layers leave a PCIe-class link almost nothing to hide behind, so the test gives every layer
a stand-in for the rest of its compute (pie_set_layer_compute_us): the regime the paper works in, where a
layer's compute time is dominated by reading its weights.  Checked: the controller starts at f = 0 and grows
(Section 3.4.2); where it settles, every layer's swap-in is shorter than its compute and the compute stream
does not wait (the swap constraint of Section 3.1); one more level would break the rho margin or the pool's
limit; and when the compute time collapses (interference), it gives the levels back.
"""
import numpy as np
import pytest
import torch

from paper_2411_09317_amd import binding as B
from paper_2411_09317_amd import inputs as I
from paper_2411_09317_amd import workload as WL

pytestmark = pytest.mark.gpu

UNITS, K_MAX, RHO = 16, 8, 0.9


def drive(dw, ctl, streams, n_steps, level):
    trace = []
    for _ in range(n_steps):
        pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
        dw.pool.step(dw.q, dw.k_new, dw.v_new, dw.d_table, dw.d_ctx, pf, dirty, dw.out, *streams)
        dw.pool.sync()
        st = dw.pool.stats()
        lt = dw.pool.layer_times()
        f_next = ctl.update_from_pool(dw.pool, dw.w.batch / (st.step_ms * 1e-3) * st.expansion_simple)
        trace.append((level, lt, st))
        new_level = int(round(f_next * UNITS))
        if new_level != level:
            dw.pool.set_host_fraction(new_level / UNITS, dw.order, streams[1])
            dw.pool.sync()
            level = new_level
    return level, trace


def test_controller_grows_while_swaps_stay_hidden_and_gives_back_when_they_do_not():
    w = I.scaled(I.CONFIGS["cfg4"], n_layers=4, batch=32)
    dw = WL.build(w, host_capacity_fraction=K_MAX / UNITS + 0.02)
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    ctl = B.Controller(UNITS, K_MAX, rho=RHO)
    try:
        dw.pool.set_timing(B.TIMING_CLOCK)
        # The stand-in is sized from this box's own link: a step at level 1 gives the time one level's blocks
        # take to come in, and a layer is made long enough to hide about five levels' worth (rho included).
        dw.pool.set_host_fraction(1 / UNITS, dw.order, streams[1])
        dw.pool.sync()
        t_level = []
        for _ in range(4):                                  # the first passes through fresh pinned memory are slow
            pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
            dw.pool.step(dw.q, dw.k_new, dw.v_new, dw.d_table, dw.d_ctx, pf, dirty, dw.out, *streams)
            dw.pool.sync()
            t_level.append(float(dw.pool.layer_times()["swap_in"][1:].max()))
        dw.pool.set_host_fraction(0.0, dw.order, streams[1])
        dw.pool.sync()
        layer_us = 5.5 * min(t_level) * 1e3 / RHO
        assert 20.0 < layer_us < 1.0e5, t_level
        dw.pool.set_layer_compute_us(layer_us)
        level, trace = drive(dw, ctl, streams, 70, 0)
        levels = [t[0] for t in trace]
        assert levels[0] == 0 and level >= 2, levels
        assert all(b - a in (0, 1) for a, b in zip(levels, levels[1:])), levels      # one level at a time, no retreat
        assert len(set(levels[-20:])) == 1, levels                                    # settled
        # the settled level's times: the smallest of its last five steps, layer by layer (one step in which the
        # host thread lost the processor for a while would otherwise decide the asserts below)
        lt = {k: np.min(np.stack([t[1][k] for t in trace[-5:]]), axis=0) for k in trace[-1][1]}
        # the constraint holds where it settled (layer 0's prefetch has nothing to hide behind)
        assert (lt["swap_in"][1:] <= lt["attn"][1:]).all()
        assert lt["stall"][1:].sum() <= 0.01 * lt["attn"].sum()
        # and one more level was refused for a reason: the pool's limit, or the rho margin one level ahead
        if level < K_MAX:
            ahead = lt["swap_in"] * (level + 1) / level
            assert (ahead > RHO * lt["attn"]).any()
        # outputs are still the all-resident ones
        got = dw.out.clone()
        dw.pool.set_host_fraction(0.0, dw.order, streams[1])
        dw.pool.sync()
        none = np.zeros(0, dtype=np.int32)
        dw.pool.step(dw.q, dw.k_new, dw.v_new, dw.d_table, dw.d_ctx, none, none, dw.out, *streams)
        dw.pool.sync()
        assert torch.equal(got.view(torch.int16), dw.out.view(torch.int16))
        dw.pool.set_host_fraction(level / UNITS, dw.order, streams[1])
        dw.pool.sync()

        # the layer's compute shrinks to the attention alone: swap-in no longer fits, levels come back
        dw.pool.set_layer_compute_us(0.0)
        level2, trace2 = drive(dw, ctl, streams, 12 * level + 8, level)
        assert level2 <= 1, [t[0] for t in trace2]
        assert dw.pool.check_errors() == 0
    finally:
        ctl.close()
        dw.pool.close()
