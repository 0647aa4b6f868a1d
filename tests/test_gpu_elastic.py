"""Layer caches that grow and shrink with the number of layers kept in CPU memory (pie_elastic_pool).

Nine layers whose caches are seven chunks each while everything is on the GPU.  Two layers are asked to stay
in CPU memory: the protocol moves layers out and in token after token, their chunks go to the layers that stay,
and once that is complete nine chunks per layer are visible - the worked example's 9/7.  A sequence that joins
then lives in blocks that did not exist before.  A shrink is refused while those blocks are in use (but hides
them at once), succeeds when they are given up, and finally every layer returns to the GPU.  At every token the
outputs are, bit for bit, those of a plain pool that holds all layers at the larger size, and at the end every
layer's bytes are the reference's.
"""
import numpy as np
import pytest
import torch

import gpu_helpers as GH
import helpers as H
from oracle import attention as A
from oracle import layout as LY
from paper_2411_09317_amd import binding as B
from paper_2411_09317_amd import inputs as I

pytestmark = pytest.mark.gpu

N_LAYERS, C, K0, K_CAP, HOST_SLOTS = 9, 4, 7, 12, 4


@pytest.mark.parametrize("dtype", [I.DTYPE_F16, I.DTYPE_BF16])
def test_capacity_follows_the_layers_on_the_cpu_and_results_never_change(dtype):
    n = N_LAYERS
    w = I.Workload("elastic", n, 3, 8, 2, 128, dtype, ctx_lo=40, ctx_hi=130, value_scale=0.7, seed=61)
    case = I.make_case(w)
    nb = int(case.n_blocks.sum())
    assert nb <= K0 * C - 1                                       # the three sequences fit the small caches
    batch, max_blocks = 4, 10
    mk = lambda blocks: B.Pool(n, w.n_q_heads, w.n_kv_heads, w.head_dim, 16, dtype, blocks, 0, 0, max_batch=batch,
                               max_blocks_per_seq=max_blocks, device=GH.DEV)
    ref, inner = mk(K_CAP * C), mk(K0 * C)
    assert ref.block_alloc(B.GPU, K_CAP * C) == list(range(K_CAP * C))          # handle = slot = block index
    table = np.full((batch, max_blocks), -1, dtype=np.int32)
    i = 0
    for b in range(3):
        for j in range(int(case.n_blocks[b])):
            table[b, j] = i
            i += 1
    late = [K0 * C + 1, K0 * C + 2]                               # blocks that exist only in the larger caches
    table[3, :2] = late
    sd = I.storage_numpy_dtype(dtype)
    img = np.zeros((n, K0 * C, 2, w.n_kv_heads, 16, w.head_dim), dtype=sd)
    for b in range(3):
        n_tok = int(case.ctx_lens[b]) - 1
        for j in range(int(case.n_blocks[b])):
            lo, hi = j * 16, min((j + 1) * 16, n_tok)
            if hi > lo:
                img[:, table[b, j], 0, :, : hi - lo] = case.k_dense[b][:, lo:hi].transpose(0, 2, 1, 3)
                img[:, table[b, j], 1, :, : hi - lo] = case.v_dense[b][:, lo:hi].transpose(0, 2, 1, 3)
    phys = torch.from_numpy(LY.to_physical(img).view(np.uint8).copy()).to(GH.DEV)   # [L][K0 C][block_bytes]
    ref.gpu_image().zero_()
    ref.gpu_image()[:, : K0 * C].copy_(phys)
    inner.gpu_image().copy_(phys)
    ep = B.ElasticPool(inner, C, K_CAP, HOST_SLOTS)
    cs, si, so = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    q_np = np.concatenate([case.q, I.to_storage(I.draw_values(w, (n, 1, w.n_q_heads, w.head_dim), 77), dtype)], axis=1)
    q = GH.to_dev(q_np, dtype)
    d_table = torch.from_numpy(table).to(GH.DEV)
    ctx = np.concatenate([case.ctx_lens, [0]]).astype(np.int32)
    none = np.zeros(0, dtype=np.int32)
    token = [0]
    # What every sequence holds, token by token, kept densely on the host: the oracle's input at every token,
    # not only the first (the fourth sequence starts empty; the others may grow to the end of their last block).
    from oracle import numfmt
    from test_gpu_attention import check
    cap = [int(case.n_blocks[b]) * 16 for b in range(3)] + [2 * 16]
    dense = []
    for d_src in (case.k_dense, case.v_dense):
        rows = [np.zeros((n, cap[b], w.n_kv_heads, w.head_dim), dtype=sd) for b in range(4)]
        for b in range(3):
            rows[b][:, : int(case.ctx_lens[b]) - 1] = d_src[b][:, : int(case.ctx_lens[b]) - 1]
        dense.append(rows)

    def oracle_check(out, layers):
        live = [b for b in range(batch) if ctx[b] > 0]
        for l in layers:
            K = [numfmt.to_f64(dense[0][b][l, : ctx[b]], dtype) for b in live]
            V = [numfmt.to_f64(dense[1][b][l, : ctx[b]], dtype) for b in live]
            ref = A.dense_attention(numfmt.to_f64(q_np[l][live], dtype), K, V, ctx[live])
            check(GH.from_dev(out[l][live], dtype), ref, dtype)

    def step():
        t = token[0]
        if t == 0:
            k3, v3 = [np.stack([np.stack([d[b][l, case.ctx_lens[b] - 1] for b in range(3)]) for l in range(n)])
                      for d in (case.k_dense, case.v_dense)]
            extra = I.to_storage(I.draw_values(w, (2, n, 1, w.n_kv_heads, w.head_dim), 78), dtype)
            k_new, v_new = np.concatenate([k3, extra[0]], axis=1), np.concatenate([v3, extra[1]], axis=1)
        else:
            k_new = I.to_storage(I.draw_values(w, (n, batch, w.n_kv_heads, w.head_dim), 100 + t), dtype)
            v_new = I.to_storage(I.draw_values(w, (n, batch, w.n_kv_heads, w.head_dim), 200 + t), dtype)
        dk, dv = GH.to_dev(k_new, dtype), GH.to_dev(v_new, dtype)
        d_ctx = torch.from_numpy(ctx).to(GH.DEV)
        for b in range(batch):
            if ctx[b] > 0:                                        # the step appends this token's rows
                dense[0][b][:, ctx[b] - 1] = k_new[:, b]
                dense[1][b][:, ctx[b] - 1] = v_new[:, b]
        out_ref, out = torch.empty_like(q), torch.full_like(q, float("nan"))
        ref.step(q, dk, dv, d_table, d_ctx, none, none, out_ref, cs, si, so)
        ref.sync()
        ep.step(q, dk, dv, d_table, d_ctx, out, cs, si, so)
        inner.sync()
        assert inner.check_errors() == 0 and ref.check_errors() == 0
        assert torch.equal(out.view(torch.int16), out_ref.view(torch.int16)), t
        # and it is the oracle's answer: three layers at the first token, two rotating ones at every later
        # token (after the appends, the join in new blocks, the moves out and in, the shrink)
        oracle_check(out, (0, 4, 8) if t == 0 else (t % n, (t + 4) % n))
        if t == 0:
            check(GH.from_dev(out[4, :3], dtype), A.dense_attention(*H.dense_f64(case, 4), case.ctx_lens), dtype)
        token[0] += 1
        return out

    def grow_context():
        for b in range(3):
            if (ctx[b] + 1 + 15) // 16 <= case.n_blocks[b]:
                ctx[b] += 1

    try:
        assert ep.capacity() == (K0 * C, K0 * C, 0)
        step()
        grow_context()
        # ---- two layers to the CPU: each cache grows to 63 // 7 = 9 chunks once they have left ----
        assert ep.set_layers_on_cpu(2, nb, cs)
        assert ep.capacity() == (K0 * C, 9 * C, 2)
        ep.set_live_blocks(nb)                                    # leaving layers take only the live chunks along
        seen = []
        for _ in range(6):
            step()
            grow_context()
            seen.append(ep.capacity()[0])
            if seen[-1] == 9 * C:
                break
        assert seen[-1] == 9 * C and all(a <= b for a, b in zip(seen, seen[1:])), seen
        st = ep.stats()
        assert st.n_swap_out >= 2 and st.n_swap_in >= 0
        assert st.bytes_out == st.n_swap_out * ((nb + C - 1) // C) * ep.chunk_bytes     # live chunks only
        # ---- a sequence joins in blocks beyond the old caches ----
        ep.set_live_blocks(late[-1] + 1)
        for t in range(20):
            ctx[3] = t + 1                                        # grows from its first token, crosses into its 2nd block
            step()
            grow_context()
        assert ctx[3] == 20 and ep.stats().n_swap_in > 0
        # ---- back to one layer on the CPU: 63 // 8 = 7 chunks; refused while the late sequence lives ----
        assert ep.set_layers_on_cpu(1, late[-1] + 1, cs) is False
        assert ep.capacity() == (K0 * C, 9 * C, 2)                # hidden at once, nothing else changed
        step()
        ctx[3] = 0                                                # the sequence ends; its blocks are given up
        ep.set_live_blocks(nb)
        assert ep.set_layers_on_cpu(1, nb, cs)
        assert ep.capacity() == (K0 * C, K0 * C, 1)
        for _ in range(3):
            step()
            grow_context()
        assert ep.set_layers_on_cpu(0, nb, cs)
        for _ in range(4):
            step()
            grow_context()
        ep.settle(cs)
        inner.sync()
        tbl = ep.table()
        assert all(s == B.LAYER_GPU for s, _, _ in tbl)           # every layer is back
        # every layer's first blocks, wherever its chunks are, hold the reference's bytes
        for l in range(n):
            where, chunks = ep.layer_chunks(l)
            assert where == B.GPU and len(chunks) == K0
            got = torch.cat([c.cpu() for c in chunks])[:nb]
            assert torch.equal(got, ref.gpu_image()[l, :nb].cpu()), l
    finally:
        ep.close()
        inner.close()
        ref.close()


def test_adaptive_expansion_grows_the_caches_on_hardware():
    """Section 3.4.2 with Section 3.1's payoff: every layer starts on the GPU; a controller that only sees
    whether computation waited asks for one more layer in CPU memory at a time, and one fewer when it did.  The
    caches of the layers that stay grow with every level (and a leaving layer carries more), outputs stay
    bit-identical, and the run settles where nothing waits with more blocks per layer than it began with."""
    import time
    n, host, C = 9, 6, 64
    w = I.Workload("elastic2", n, 8, 8, 8, 128, I.DTYPE_F16, ctx_lo=1500, ctx_hi=2048, value_scale=0.5, seed=63)
    ctx = I.draw_ctx_lens(w)
    n_blocks = I.blocks_needed(ctx, 16)
    nb, max_blocks = int(n_blocks.sum()), int(n_blocks.max())
    k0 = (nb + C - 1) // C
    k_cap = (n * k0) // (n - (host - 2))
    mk = lambda: B.Pool(n, w.n_q_heads, w.n_kv_heads, w.head_dim, 16, w.dtype, k0 * C, 0, 0, max_batch=w.batch,
                        max_blocks_per_seq=max_blocks, device=GH.DEV)
    ref, inner = mk(), mk()
    table = np.full((w.batch, max_blocks), -1, dtype=np.int32)
    i = 0
    for b in range(w.batch):
        for j in range(int(n_blocks[b])):
            table[b, j] = i
            i += 1
    assert ref.block_alloc(B.GPU, nb) == list(range(nb))
    gen = torch.Generator(device=GH.DEV)
    gen.manual_seed(5)
    fill = (torch.randn(ref.gpu_image().numel() // 2, device=GH.DEV, generator=gen) * 0.5).to(torch.float16)
    ref.gpu_image().view(-1).view(torch.float16).copy_(fill)
    inner.gpu_image().copy_(ref.gpu_image())
    q = (torch.randn(n, w.batch, w.n_q_heads, w.head_dim, device=GH.DEV, generator=gen) * 0.5).to(torch.float16)
    ep = B.ElasticPool(inner, C, k_cap, host)
    cs, si, so = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    d_table, d_ctx = torch.from_numpy(table).to(GH.DEV), torch.from_numpy(ctx).to(GH.DEV)
    out_ref, out = torch.empty_like(q), torch.empty_like(q)
    none = np.zeros(0, dtype=np.int32)
    ctl = B.Controller(n, host - 2, k_up=3, k_down=2, probe_period=1000)

    def token():
        t0 = time.perf_counter()
        ep.step(q, None, None, d_table, d_ctx, out, cs, si, so)
        inner.sync()
        dt = (time.perf_counter() - t0) * 1e3
        assert torch.equal(out.view(torch.int16), out_ref.view(torch.int16))
        return dt

    try:
        ref.step(q, None, None, d_table, d_ctx, none, none, out_ref, cs, si, so)
        ref.sync()
        t_swap_us = GH.copy_engine_us(k0 * ep.chunk_bytes, pieces=k0)   # measured here: one copy per chunk, both directions busy
        print("measured swap time", round(t_swap_us, 1), "us")
        # a layer's move takes 1.4 layer times by that measurement: the protocol hides up to two, and the chunked
        # moves it really makes (host-ordered, both directions interleaved) come out somewhat slower than measured
        t_layer_us = t_swap_us / 1.4
        inner.set_layer_compute_us(t_layer_us)
        ep.set_live_blocks(nb)                                    # a layer always travels as its k0 live chunks
        # once around before the clock counts: the first transfers through fresh pinned memory are slow
        assert ep.set_layers_on_cpu(host - 2, nb, cs)
        for _ in range(4):
            token()
        assert ep.set_layers_on_cpu(0, nb, cs)
        for _ in range(12):
            token()
        ep.settle(cs)
        assert all(s == B.LAYER_GPU for s, _, _ in ep.table()) and ep.capacity() == (k0 * C, k0 * C, 0)
        levels, stalls, visible, dts, level, prev_stall = [], [], [], [], 0, ep.stats().stall_ms
        for _ in range(70):
            levels.append(level)
            dt_ms = token()
            st = ep.stats()
            stall = st.stall_ms - prev_stall
            prev_stall = st.stall_ms
            stalls.append(stall)
            dts.append(dt_ms)
            vis, tgt, m = ep.capacity()
            visible.append(vis)
            assert m == level and vis <= tgt
            # The controller sees only whether computation waited: a token is taken to cost its layers' compute
            # plus the waits (what else the host adds per token differs from box to box and is not its business),
            # and the level is credited with the size it leads to, as soon as it is asked for.
            tc = t_layer_us / 1e3
            new = ctl.observe([tc] * n, [0.0] * n, [stall / n] * n, 0.0, tgt / (k0 * C) / (n * tc + stall))
            if new != level:
                assert ep.set_layers_on_cpu(new, nb, cs)         # the live blocks all lie below the smallest cache
                level = new
        assert inner.check_errors() == 0
        print("levels", levels, "visible blocks", visible, "ms per token", [round(x, 2) for x in dts],
              "waits", [round(x, 2) for x in stalls])
        assert levels[:3] == [0, 0, 0] and max(levels) >= 2, levels
        assert all(abs(b - a) <= 1 for a, b in zip(levels, levels[1:])), levels
        assert len(set(levels[-12:])) == 1 and levels[-1] >= 1, levels
        token_ms = n * t_layer_us / 1e3
        assert sum(stalls[-10:]) <= 0.02 * 10 * token_ms, (levels, stalls[-10:])
        m_end = levels[-1]
        assert visible[-1] == min(k_cap, (n * k0) // (n - m_end)) * C > k0 * C     # a / (n - m), in whole chunks
        assert visible[0] == k0 * C
    finally:
        ctl.close()
        ep.close()
        inner.close()
        ref.close()


def test_serving_on_growing_and_shrinking_caches_matches_an_all_resident_pool():
    """Requests come and go while the number of layers kept in CPU memory is moved up and down: admission
    follows the size the pool shows, new requests land in blocks that did not exist before, a shrink waits for
    them to end.  Every iteration's outputs are, bit for bit, those of a plain pool holding all layers at the
    largest size, fed the same tables and the same rows."""
    from paper_2411_09317_amd import serving as S
    n, C, k0, k_cap, host = 6, 4, 6, 12, 5
    dtype = I.DTYPE_F16
    w = I.Workload("eserve", n, 0, 8, 2, 128, dtype, ctx_lo=10, ctx_hi=90, value_scale=0.5, seed=71)
    max_batch, max_blocks = 12, 8
    mk = lambda blocks: B.Pool(n, w.n_q_heads, w.n_kv_heads, w.head_dim, 16, dtype, blocks, 0, 0, max_batch=max_batch,
                               max_blocks_per_seq=max_blocks, device=GH.DEV)
    ref, inner = mk(k_cap * C), mk(k0 * C)
    assert ref.block_alloc(B.GPU, k_cap * C) == list(range(k_cap * C))
    gen = torch.Generator(device=GH.DEV)
    gen.manual_seed(9)
    fill = (torch.randn(ref.gpu_image().numel() // 2, device=GH.DEV, generator=gen) * 0.5).to(torch.float16)
    ref.gpu_image().view(-1).view(torch.float16).copy_(fill)           # whatever was there before
    inner.gpu_image().copy_(ref.gpu_image()[:, : k0 * C])
    ep = B.ElasticPool(inner, C, k_cap, host)
    loop = S.DeviceLoop(inner, w, max_batch, max_blocks)
    store = S.IndexStore(k_cap * C, k0 * C)
    sched = S.Scheduler(store, 16, S.VisibleBudget(ep, k0 * C), max_batch, max_blocks)
    # every token of a request is appended by a step (empty prompts): a block's content is then defined in both
    # pools, whichever chunk it lives in (blocks that are not live are not carried when a layer moves)
    a, p, o = I.draw_requests(w, 60, 1e6, 20, 110)
    for i in range(60):
        sched.submit(S.Request(i, float(a[i]), 0, int(o[i])))
    none = np.zeros(0, dtype=np.int32)
    plan = {5: 2, 50: 3, 90: 1, 130: 0}                               # iteration -> layers asked to be on the CPU
    want, it, sizes, above, refused, moved, on_cpu_at_move = 0, 0, [], 0, 0, 0, []
    rows_of, n_oracle = {}, 0
    from test_gpu_attention import check
    cs = loop.streams[0]
    try:
        while not sched.idle:
            want = plan.get(it, want)
            vis, tgt, m = ep.capacity()
            if want != m:
                below = ep.blocks_for(want)
                if want < m and sched.reserved <= below < store.live_end():
                    mv = store.plan_compaction(below)                # live blocks above the smaller size move down
                    if mv and mv[0]:
                        ep.move_blocks(mv[0], mv[1], cs)
                        ref.sync()
                        ref.gpu_image()[:, mv[1]] = ref.gpu_image()[:, mv[0]]
                        sched.relocate(*mv)
                        moved += len(mv[0])
                if ep.set_layers_on_cpu(want, max(store.live_end(), sched.reserved), cs):
                    vis, tgt, m = ep.capacity()
                else:
                    refused += 1
            store.limit = max(store.limit, vis) if want < m else vis
            assert sched.reserved <= store.limit
            if it in (70, 75, 110):                                  # and a few times just so: the highest live
                live = np.flatnonzero(store.used)                    # blocks go to the lowest free places, with
                free = np.flatnonzero(~store.used[: store.limit])    # layers on the GPU and in CPU memory
                k = min(4, len(live), len(free))
                src, dst = live[-k:][live[-k:] > free[k - 1]].tolist(), free[:k].tolist()
                dst = dst[: len(src)]
                if src:
                    ep.move_blocks(src, dst, cs)
                    ref.sync()
                    ref.gpu_image()[:, dst] = ref.gpu_image()[:, src]
                    sched.relocate(src, dst)
                    moved += len(src)
                    on_cpu_at_move.append(sum(1 for st_, _, _ in ep.table() if st_ == B.LAYER_HOST))
            sched.admit(1.0)
            assert sched.running
            table, ctx = sched.tables()
            B_ = len(ctx)
            above += int((table >= k0 * C).sum() > 0)
            ep.set_live_blocks(store.live_end())
            dt, _ = loop.iteration(sched, step=ep.step)
            shape = lambda t, h: t[: n * B_ * h * w.head_dim].view(n, B_, h, w.head_dim)
            # the oracle's view: every request's rows, kept densely on the host as the steps append them
            k_rows, v_rows = shape(loop.k_new, w.n_kv_heads).cpu().numpy(), shape(loop.v_new, w.n_kv_heads).cpu().numpy()
            for i, r in enumerate(sched.running):
                kd, vd = rows_of.setdefault(r.rid, (np.zeros((n, max_blocks * 16, w.n_kv_heads, w.head_dim), np.float16),
                                                    np.zeros((n, max_blocks * 16, w.n_kv_heads, w.head_dim), np.float16)))
                kd[:, r.ctx - 1], vd[:, r.ctx - 1] = k_rows[:, i], v_rows[:, i]
            if it % 7 == 0 or it in plan or it - 1 in plan or it in (70, 75, 110, 71, 76, 111):
                l = it % n
                K = [rows_of[r.rid][0][l, : r.ctx].astype(np.float64) for r in sched.running]
                V = [rows_of[r.rid][1][l, : r.ctx].astype(np.float64) for r in sched.running]
                want_out = A.dense_attention(shape(loop.q, w.n_q_heads)[l].cpu().numpy().astype(np.float64), K, V, ctx)
                check(GH.from_dev(shape(loop.out, w.n_q_heads)[l], dtype), want_out, dtype)
                n_oracle += 1
            out_ref = torch.empty_like(shape(loop.out, w.n_q_heads))
            ref.step(shape(loop.q, w.n_q_heads), shape(loop.k_new, w.n_kv_heads), shape(loop.v_new, w.n_kv_heads),
                     loop.d_table[:B_], loop.d_ctx[:B_], none, none, out_ref, *loop.streams)
            ref.sync()
            assert torch.equal(shape(loop.out, w.n_q_heads).view(torch.int16), out_ref.view(torch.int16)), it
            sizes.append(vis)
            sched.complete_iteration(1.0)
            it += 1
            assert it < 3000
        assert inner.check_errors() == 0 and ref.check_errors() == 0
        assert len(sched.done) == 60 and not store.used.any() and n_oracle > 20
        assert max(sizes) >= 9 * C > k0 * C and above > 10          # requests lived in blocks the small caches lack
        assert moved > 0 and max(on_cpu_at_move) >= 1              # blocks were moved, in both kinds of memory
        assert it > 130 or want == plan[max(k for k in plan if k <= it)]
    finally:
        ep.close()
        inner.close()
        ref.close()


def test_serve_elastic_runs_to_completion_with_the_controller():
    from paper_2411_09317_amd import serving as S
    n, C, k0, host = 8, 16, 8, 5
    w = I.Workload("eserve2", n, 0, 8, 2, 128, I.DTYPE_BF16, ctx_lo=64, ctx_hi=400, value_scale=0.5, seed=72)
    max_batch, max_blocks = 32, 32
    k_cap = (n * k0) // (n - (host - 2))
    inner = B.Pool(n, w.n_q_heads, w.n_kv_heads, w.head_dim, 16, w.dtype, k0 * C, 0, 0, max_batch=max_batch,
                   max_blocks_per_seq=max_blocks, device=GH.DEV)
    inner.gpu_image().zero_()
    ep = B.ElasticPool(inner, C, k_cap, host)
    inner.set_layer_compute_us(300.0)
    a, p, o = I.draw_requests(w, 80, 1e6, 8, 48)
    reqs = [S.Request(i, float(a[i]), int(p[i]), int(o[i])) for i in range(80)]
    ctl = B.Controller(n, host - 2, k_up=3, k_down=2, probe_period=1000)
    try:
        res = S.serve_elastic(ep, w, reqs, max_batch, max_blocks, controller=ctl)
        assert res["requests"] == 80 and res["tokens"] == int(o.sum()) and res["tokens_per_s"] > 0
        assert res["blocks_per_layer_max"] >= k0 * C and res["layers_on_cpu_max"] >= 1
        reqs = [S.Request(i, float(a[i]), int(p[i]), int(o[i])) for i in range(80)]
        res2 = S.serve_elastic(ep, w, reqs, max_batch, max_blocks, layers_on_cpu=2)
        assert res2["requests"] == 80 and res2["blocks_per_layer_max"] == min(k_cap, (n * k0) // (n - 2)) * C
    finally:
        ctl.close()
        ep.close()
        inner.close()
