"""The layer-granular swapping protocol on the GPU (pie_layer_pool).

Whole layers of KV move between GPU layer slots and pinned CPU layer slots while a token's layers are
computed in order.  Checked: every token step gives, bit for bit, the outputs of a plain pool that holds all
layers; the new token's rows written into a layer survive its trip to the CPU and back; the mapping table
stays consistent; and, with a stand-in for the rest of each layer's compute sized so that a swap takes a bit
less than two layer times, the schedule is the worked example's: no forced moves, about n / 2 swaps per
token and direction, and a FIFO of four layers away from the GPU.
"""
import numpy as np
import pytest
import torch

import gpu_helpers as GH
from oracle import attention as A
from oracle import layout as LY
from paper_2411_09317_amd import binding as B
from paper_2411_09317_amd import inputs as I

pytestmark = pytest.mark.gpu


def build(n_layers, n_gpu_slots, n_host_slots, on_host, w, seed=0):
    """A reference pool holding all layers, and a layer pool with the same content."""
    case = I.make_case(w)
    nb = int(case.n_blocks.sum())
    ref = B.Pool(n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, 16, w.dtype, nb, 0, 0, max_batch=w.batch,
                 max_blocks_per_seq=case.max_blocks, device=GH.DEV)
    inner = B.Pool(n_gpu_slots, w.n_q_heads, w.n_kv_heads, w.head_dim, 16, w.dtype, nb, 0, 0, max_batch=w.batch,
                   max_blocks_per_seq=case.max_blocks, device=GH.DEV)
    hs = np.asarray(ref.block_alloc(B.GPU, nb), dtype=np.int32)
    assert np.array_equal(hs, np.asarray(inner.block_alloc(B.GPU, nb), dtype=np.int32))
    table = np.full((w.batch, case.max_blocks), -1, dtype=np.int32)
    i = 0
    for b in range(w.batch):
        for j in range(int(case.n_blocks[b])):
            table[b, j] = hs[i]
            i += 1
    # logical images [L][nb][2][Hkv][T][d] from the dense case, stored up to ctx - 1 (the step appends the last token)
    sd = I.storage_numpy_dtype(w.dtype)
    img = np.zeros((n_layers, nb, 2, w.n_kv_heads, 16, w.head_dim), dtype=sd)
    for b in range(w.batch):
        n_tok = int(case.ctx_lens[b]) - 1
        for j in range(int(case.n_blocks[b])):
            lo, hi = j * 16, min((j + 1) * 16, n_tok)
            if hi > lo:
                img[:, table[b, j], 0, :, : hi - lo] = case.k_dense[b][:, lo:hi].transpose(0, 2, 1, 3)
                img[:, table[b, j], 1, :, : hi - lo] = case.v_dense[b][:, lo:hi].transpose(0, 2, 1, 3)
    phys = torch.from_numpy(LY.to_physical(img).view(np.uint8).copy())          # [L][nb][block_bytes]
    ref.gpu_image().copy_(phys.to(GH.DEV))
    lp = B.LayerPool(inner, n_layers, n_host_slots, on_host)
    for l in range(n_layers):
        lp.layer_image(l).copy_(phys[l])
    torch.cuda.synchronize()
    return case, ref, inner, lp, table


def new_rows(case, token):
    """The token's K / V rows per layer: the dense case's last row for token 0, seeded draws afterwards."""
    w = case.w
    if token == 0:
        k = np.stack([np.stack([case.k_dense[b][l, case.ctx_lens[b] - 1] for b in range(w.batch)]) for l in range(w.n_layers)])
        v = np.stack([np.stack([case.v_dense[b][l, case.ctx_lens[b] - 1] for b in range(w.batch)]) for l in range(w.n_layers)])
        return k, v
    k = I.to_storage(I.draw_values(w, (w.n_layers, w.batch, w.n_kv_heads, w.head_dim), 100 + token), w.dtype)
    v = I.to_storage(I.draw_values(w, (w.n_layers, w.batch, w.n_kv_heads, w.head_dim), 200 + token), w.dtype)
    return k, v


def check_table(lp, n_gpu_slots, n_host_slots):
    t = lp.table()
    g = [gs for st, gs, hs in t if gs >= 0]
    h = [hs for st, gs, hs in t if hs >= 0]
    assert len(set(g)) == len(g) <= n_gpu_slots and len(set(h)) == len(h) <= n_host_slots
    for st, gs, hs in t:
        assert (st == B.LAYER_GPU and gs >= 0 and hs < 0) or (st == B.LAYER_HOST and hs >= 0 and gs < 0) or \
               (st in (B.LAYER_MOVING_IN, B.LAYER_MOVING_OUT) and gs >= 0 and hs >= 0)
    return t


@pytest.mark.parametrize("dtype", [I.DTYPE_F16, I.DTYPE_BF16])
def test_tokens_through_swapping_layers_match_the_all_resident_pool(dtype):
    n, gpu, host, on_host = 9, 7, 4, [7, 8]
    w = I.Workload("lfifo", n, 3, 8, 2, 128, dtype, ctx_lo=40, ctx_hi=300, value_scale=0.7, seed=51)
    case, ref, inner, lp, table = build(n, gpu, host, on_host, w)
    cs, si, so = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    q = GH.to_dev(case.q, dtype)
    d_table = torch.from_numpy(table).to(GH.DEV)
    ctx = case.ctx_lens.copy()
    none = np.zeros(0, dtype=np.int32)
    try:
        for token in range(5):
            k_new, v_new = new_rows(case, token)
            dk, dv = GH.to_dev(k_new, dtype), GH.to_dev(v_new, dtype)
            d_ctx = torch.from_numpy(ctx).to(GH.DEV)
            out_ref, out = torch.empty_like(q), torch.full_like(q, float("nan"))
            ref.step(q, dk, dv, d_table, d_ctx, none, none, out_ref, cs, si, so)
            ref.sync()
            lp.step(q, dk, dv, d_table, d_ctx, out, cs, si, so)
            inner.sync()
            assert inner.check_errors() == 0 and ref.check_errors() == 0
            assert torch.equal(out.view(torch.int16), out_ref.view(torch.int16)), token
            check_table(lp, gpu, host)
            if token == 0:                                     # and the reference is the oracle's answer
                from test_gpu_attention import check
                import helpers as H
                for l in (0, 4, 8):
                    check(GH.from_dev(out[l], dtype), A.dense_attention(*H.dense_f64(case, l), case.ctx_lens), dtype)
            if int(ctx.max()) % 16 != 0 or token < 4:
                ctx = ctx + 1                                  # the next token extends every sequence
                if (I.blocks_needed(ctx, 16) > case.n_blocks).any():
                    ctx = ctx - 1                              # stay inside the allocated blocks
        st = lp.stats()
        assert st.n_steps == 5 and st.n_swap_in > 0 and st.n_swap_out > 0
        lp.settle()
        t = check_table(lp, gpu, host)
        assert all(s in (B.LAYER_GPU, B.LAYER_HOST) for s, _, _ in t)
        # every layer's image, wherever it ended up, equals the reference pool's layer
        for l in range(n):
            assert torch.equal(lp.layer_image(l).cpu(), ref.gpu_image()[l].cpu()), l
    finally:
        lp.close()
        inner.close()
        ref.close()


def test_worked_example_schedule_on_hardware():
    """Nine layers, seven GPU slots, four CPU slots, layers 8 and 9 start in CPU memory; a layer's compute is
    stretched so that one swap takes about 1.7 layer times (the example's 2, with margin for jitter)."""
    n, gpu, host, on_host = 9, 7, 4, [7, 8]
    w = I.Workload("lfifo2", n, 8, 8, 8, 128, I.DTYPE_F16, ctx_lo=1500, ctx_hi=2048, value_scale=0.5, seed=52)
    case, ref, inner, lp, table = build(n, gpu, host, on_host, w)
    cs, si, so = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    q = GH.to_dev(case.q, w.dtype)
    d_table = torch.from_numpy(table).to(GH.DEV)
    d_ctx = torch.from_numpy(case.ctx_lens).to(GH.DEV)
    out = torch.empty_like(q)
    try:
        t_swap_us = GH.copy_engine_us(lp.layer_bytes)          # measured here, with both directions busy
        print("measured swap time", round(t_swap_us, 1), "us")
        inner.set_layer_compute_us(t_swap_us / 1.7)
        tokens = 8
        for _ in range(tokens):
            lp.step(q, None, None, d_table, d_ctx, out, cs, si, so)
        inner.sync()
        assert inner.check_errors() == 0
        st = lp.stats()
        assert st.n_forced_in == 0
        # the link is busy about all the time: n * t_compute / t_swap swaps per token and direction
        per_token = st.n_swap_out / tokens
        assert n / 2 - 0.75 <= per_token <= n / 1.7 + 0.5, per_token
        assert abs(st.n_swap_in - st.n_swap_out) <= 2
        away = sum(1 for s, _, _ in lp.table() if s != B.LAYER_GPU)
        assert away in (3, 4)                                  # two in CPU memory, one or two in flight
    finally:
        lp.close()
        inner.close()
        ref.close()


def test_adaptive_expansion_in_layers_on_hardware():
    """Section 3.4.2 in the paper's own unit: every layer starts on the GPU; a controller that only sees whether
    computation waited takes GPU layer slots away one at a time and gives one back when it did.  Outputs stay
    bit-identical throughout; the run overshoots, waits, and settles where nothing waits."""
    n, host = 9, 6
    w = I.Workload("lfifo3", n, 8, 8, 8, 128, I.DTYPE_F16, ctx_lo=1500, ctx_hi=2048, value_scale=0.5, seed=53)
    case, ref, inner, lp, table = build(n, n, host, [], w)
    cs, si, so = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    q = GH.to_dev(case.q, w.dtype)
    d_table = torch.from_numpy(table).to(GH.DEV)
    d_ctx = torch.from_numpy(case.ctx_lens).to(GH.DEV)
    out_ref, out = torch.empty_like(q), torch.empty_like(q)
    none = np.zeros(0, dtype=np.int32)
    ctl = B.Controller(n, host - 2, k_up=3, k_down=2, probe_period=1000)
    try:
        ref.step(q, None, None, d_table, d_ctx, none, none, out_ref, cs, si, so)
        ref.sync()
        t_swap_us = GH.copy_engine_us(lp.layer_bytes)          # measured here, with both directions busy
        print("measured swap time", round(t_swap_us, 1), "us")
        t_layer_us = t_swap_us / 1.7
        inner.set_layer_compute_us(t_layer_us)
        levels, stalls, level, prev_stall = [], [], 0, 0.0
        for token in range(60):
            levels.append(level)
            lp.step(q, None, None, d_table, d_ctx, out, cs, si, so)
            inner.sync()
            assert torch.equal(out.view(torch.int16), out_ref.view(torch.int16)), token
            st = lp.stats()
            stall = st.stall_ms - prev_stall
            prev_stall = st.stall_ms
            stalls.append(stall)
            # the controller sees only whether computation waited: a token costs its layers' compute plus the
            # waits (what else the host adds per token differs from box to box)
            tc = t_layer_us / 1e3
            new = ctl.observe([tc] * n, [0.0] * n, [stall / n] * n, 0.0, n / (n - level) / (n * tc + stall))
            if new != level:
                lp.set_gpu_slots(n - new)
                level = new
        assert inner.check_errors() == 0
        assert levels[:3] == [0, 0, 0] and max(levels) >= 2, levels
        assert all(abs(b - a) <= 1 for a, b in zip(levels, levels[1:])), levels
        assert len(set(levels[-12:])) == 1 and levels[-1] >= 1, levels
        token_ms = n * t_layer_us / 1e3
        assert sum(stalls[-10:]) <= 0.02 * 10 * token_ms, (levels, stalls[-10:])
        lp.settle()
        away = sum(1 for s, _, _ in lp.table() if s != B.LAYER_GPU)
        assert away >= levels[-1]
    finally:
        ctl.close()
        lp.close()
        inner.close()
        ref.close()
