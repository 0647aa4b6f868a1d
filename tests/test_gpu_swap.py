"""GPU parity for the swap path, residency changes and the per-layer pipeline:
bytes and tables bit-exact against the oracle's pool model; attention outputs
against the dense float64 oracle and bit-identical across residency choices."""
import numpy as np
import pytest
import torch

import gpu_helpers as GH
import helpers as H
from oracle import attention as A
from oracle.pool_model import PoolError
from paper_2411_09317_amd import binding as B
from paper_2411_09317_amd import inputs as I

pytestmark = pytest.mark.gpu

W = I.Workload("swap", 3, 5, 8, 4, 128, I.DTYPE_F16, ctx_lo=20, ctx_hi=400, value_scale=0.5, host_fraction=0.3, seed=51)
PATHS = [B.SWAP_DMA, B.SWAP_KERNEL, B.SWAP_AUTO]


def host_tails(case, every=2):
    for b in range(0, case.w.batch, every):
        case.host_mask[b][-1] = True
    return case


def assert_images_equal(lib, mod, staging=True):
    g, h = GH.images_of(lib)
    mg, mh = GH.model_bytes(mod)
    assert np.array_equal(h, mh)
    n = mod.n_gpu + (2 * mod.n_stage if staging else 0)
    assert np.array_equal(g[:, :n], mg[:, :n])


@pytest.mark.parametrize("path", PATHS)
def test_swap_round_trip_bytes_and_staging_slots(path):
    case = host_tails(I.make_case(W))
    lib, mod, table = GH.make_pools(case, 120, 48, 64)
    lib.set_swap_path(path)
    plist = mod.prefetch_list(table, case.ctx_lens)
    assert len(plist) >= 10
    g0, h0 = GH.images_of(lib)
    s_in, s_out = torch.cuda.Stream(), torch.cuda.Stream()
    for layer in range(W.n_layers):
        lib.swap_in(layer, plist, s_in)
        mod.swap_in(layer, plist)
        lib.sync()
        slots, states = lib.block_staged(layer & 1, plist)
        assert slots == [mod.stage_slot(layer & 1, i) for i in range(len(plist))]
        assert states == [2] * len(plist)
        assert_images_equal(lib, mod)
        lib.swap_out(layer, plist[::2], s_out)
        mod.swap_out(layer, plist[::2])
    lib.sync()
    g1, h1 = GH.images_of(lib)
    assert np.array_equal(h0, h1)                                   # round trip: host bytes untouched
    assert np.array_equal(g0[:, :120], g1[:, :120])                 # resident slots untouched
    assert_images_equal(lib, mod)
    lib.close()


@pytest.mark.parametrize("path", [B.SWAP_DMA, B.SWAP_KERNEL])
def test_swap_out_carries_modified_staging_back(path):
    case = host_tails(I.make_case(W))
    lib, mod, table = GH.make_pools(case, 120, 48, 64)
    lib.set_swap_path(path)
    plist = mod.prefetch_list(table, case.ctx_lens)[::-1]           # descending host slots: many short runs
    lib.swap_in(1, plist)
    mod.swap_in(1, plist)
    lib.sync()
    for i in (0, 3):
        s = mod.stage_slot(1, i)
        lib.gpu_image()[1, s].fill_(0x5A)
        mod.gpu[1, s] = np.frombuffer(b"\x5a\x5a", dtype=np.float16)[0]
    torch.cuda.synchronize()
    lib.swap_out(1, [plist[0], plist[3]])
    mod.swap_out(1, [plist[0], plist[3]])
    lib.sync()
    assert_images_equal(lib, mod)
    lib.close()


def test_swap_errors_match_the_model():
    case = host_tails(I.make_case(W))
    lib, mod, table = GH.make_pools(case, 120, 8, 64)
    plist = mod.prefetch_list(table, case.ctx_lens)
    gpu_homed = [int(h) for h in table.ravel() if h >= 0 and mod.home[int(h)][0] == 0]

    def both(f):
        res = []
        for p in (lib, mod):
            try:
                f(p)
                res.append(0)
            except (B.PieError, PoolError) as e:
                res.append(e.code)
        assert res[0] == res[1], res
        return res[0]

    assert both(lambda p: p.swap_in(0, plist)) == B.ENOMEM           # staging region holds 8
    assert both(lambda p: p.swap_in(0, gpu_homed[:2])) == B.ESTATE
    assert both(lambda p: p.swap_in(9, plist[:2])) == B.EINVAL
    assert both(lambda p: p.swap_in(0, [plist[0], plist[0]])) == B.ESTATE
    assert both(lambda p: p.swap_in(0, plist[:4])) == 0
    assert both(lambda p: p.swap_out(2, plist[:4])) == B.ESTATE      # region 0 holds layer 0
    assert both(lambda p: p.swap_out(0, plist[4:6])) == B.ESTATE     # not staged
    assert both(lambda p: p.swap_out(0, plist[:4])) == 0
    lib.sync()
    assert_images_equal(lib, mod)
    lib.close()


def run_attn(lib, case, table, layer, stream=None):
    q = GH.to_dev(case.q[layer], case.w.dtype)
    out = torch.full_like(q, float("nan"))
    torch.cuda.synchronize()
    lib.attn_decode(layer, q, torch.from_numpy(table).to(GH.DEV), torch.from_numpy(case.ctx_lens).to(GH.DEV), out, stream)
    lib.sync()
    torch.cuda.synchronize()
    return GH.from_dev(out, case.w.dtype)


@pytest.mark.parametrize("path", [B.SWAP_DMA, B.SWAP_KERNEL])
def test_migration_and_fixed_fraction_keep_bytes_and_outputs(path):
    case = I.make_case(W, host_fraction=0.0)
    n = int(case.n_blocks.sum())
    lib, mod, table = GH.make_pools(case, n + 5, n, n)
    lib.set_swap_path(path)
    order = [int(table[b, j]) for b, j in I.draw_promotion_order(W, case.n_blocks)]
    base = [run_attn(lib, case, table, l) for l in range(W.n_layers)]
    ref = [A.dense_attention(*H.dense_f64(case, l), case.ctx_lens) for l in range(W.n_layers)]
    for l in range(W.n_layers):
        assert GH.rowwise_rel_err(base[l], ref[l]) <= 2e-3
    s_mig = torch.cuda.Stream()
    for f in (0.1, 0.5, 1.0, 0.3, 0.0):
        assert lib.set_host_fraction(f, order, s_mig) == mod.set_host_fraction(f, order)
        lib.sync()
        assert lib.block_where(order) == mod.block_where(order)
        assert_images_equal(lib, mod, staging=False)
        plist = mod.prefetch_list(table, case.ctx_lens)
        for l in range(W.n_layers):
            lib.swap_in(l, plist, s_mig)
            got = run_attn(lib, case, table, l)
            assert np.array_equal(got, base[l]), (f, l)              # residency independence, bit for bit
    assert lib.check_errors() == 0
    lib.close()


def test_attention_without_prefetch_flags_not_present():
    case = host_tails(I.make_case(W))
    lib, mod, table = GH.make_pools(case, 120, 48, 64)
    run_attn(lib, case, table, 0)
    assert lib.check_errors() & B.DEVERR_NOT_PRESENT
    plist = mod.prefetch_list(table, case.ctx_lens)
    lib.swap_in(2, plist)                                            # region 0 now holds layer 2, not layer 0
    run_attn(lib, case, table, 0)
    assert lib.check_errors() & B.DEVERR_NOT_PRESENT
    got = run_attn(lib, case, table, 2)
    assert lib.check_errors() == 0
    assert GH.rowwise_rel_err(got, A.dense_attention(*H.dense_f64(case, 2), case.ctx_lens)) <= 2e-3
    lib.close()


def new_token_rows(case):
    w = case.w
    k = np.stack([np.stack([case.k_dense[b][l, case.ctx_lens[b] - 1] for b in range(w.batch)]) for l in range(w.n_layers)])
    v = np.stack([np.stack([case.v_dense[b][l, case.ctx_lens[b] - 1] for b in range(w.batch)]) for l in range(w.n_layers)])
    return k, v


def run_step(lib, case, table, streams, timing=False):
    w = case.w
    k_new, v_new = new_token_rows(case)
    q = GH.to_dev(case.q, w.dtype)
    out = torch.full_like(q, float("nan"))
    pf, dirty = lib.prefetch_list(table, case.ctx_lens)
    torch.cuda.synchronize()
    lib.set_timing(timing)
    lib.step(q, GH.to_dev(k_new, w.dtype), GH.to_dev(v_new, w.dtype), torch.from_numpy(table).to(GH.DEV),
             torch.from_numpy(case.ctx_lens).to(GH.DEV), pf, dirty, out, *streams)
    lib.sync()
    torch.cuda.synchronize()
    return GH.from_dev(out, w.dtype), pf, dirty


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("dtype,hq,hkv,d", [(I.DTYPE_F16, 8, 4, 128), (I.DTYPE_F32, 8, 8, 64), (I.DTYPE_BF16, 8, 1, 128)])
def test_step_matches_oracle_for_any_residency(path, dtype, hq, hkv, d):
    w = I.scaled(W, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n_layers=4)
    tol = {I.DTYPE_F32: 1e-5, I.DTYPE_F16: 2e-3, I.DTYPE_BF16: 1e-2}[dtype]
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    outs = []
    for f in (0.0, 0.3, 1.0):
        case = I.make_case(w, host_fraction=f)
        if f == 0.3:
            host_tails(case)
        n = int(case.n_blocks.sum())
        lib, mod, table = GH.make_pools(case, n, n, n, upto_ctx=case.ctx_lens - 1, fill=H.nan_fill(dtype))
        lib.set_swap_path(path)
        got, pf, dirty = run_step(lib, case, table, streams)
        assert lib.check_errors() == 0
        assert np.isfinite(got).all()
        assert pf.tolist() == mod.prefetch_list(table, case.ctx_lens)
        ref_model = mod.step(case.q, *new_token_rows(case), table, case.ctx_lens)
        for l in range(w.n_layers):
            ref = A.dense_attention(*H.dense_f64(case, l), case.ctx_lens)
            assert GH.rowwise_rel_err(got[l], ref) <= tol
            assert np.abs(got[l] - ref).max() <= (1e-5 if dtype == I.DTYPE_F32 else 2e-2)
        assert GH.rowwise_rel_err(got, ref_model) <= tol
        assert_images_equal(lib, mod, staging=False)                 # both homes hold the appended token
        if f > 0:
            assert len(dirty) > 0 or f == 0.3
        outs.append(got)
        lib.close()
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


@pytest.mark.parametrize("dtype,hq,hkv,d,part", [(I.DTYPE_F16, 8, 4, 128, 256), (I.DTYPE_F16, 4, 4, 64, 512),
                                                 (I.DTYPE_BF16, 8, 1, 128, 256), (I.DTYPE_F32, 4, 2, 64, 256)])
def test_step_takes_the_newest_token_from_its_rows_at_every_edge_of_the_context(dtype, hq, hkv, d, part):
    """pie_step reads the context without its last token from the cache and that token from k_new / v_new.
    Contexts at the edges of that split: the token alone (1), alone in a fresh block (17, 257), first of a new
    partition (part + 1), last of one (part), and ordinary ones; all resident, and with every second tail block
    and a third of the others on the host.  Against the float64 oracle, and residency changes no bit."""
    ctx = [1, 2, 15, 16, 17, part - 1, part, part + 1, part + 17, 2 * part, 2 * part + 1, 3 * part - 5, 700, 33]
    w = I.scaled(W, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n_layers=3, batch=len(ctx))
    tol = {I.DTYPE_F32: 1e-5, I.DTYPE_F16: 2e-3, I.DTYPE_BF16: 1e-2}[dtype]
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    outs = []
    for f in (0.0, 0.3):
        case = I.make_case(w, host_fraction=f, ctx_lens=ctx)
        if f > 0:
            host_tails(case)
        n = int(case.n_blocks.sum())
        lib, mod, table = GH.make_pools(case, n, n, n, upto_ctx=case.ctx_lens - 1, fill=H.nan_fill(dtype))
        lib.set_attn_partition(part)
        got, pf, dirty = run_step(lib, case, table, streams)
        assert lib.check_errors() == 0
        assert np.isfinite(got).all()
        assert f == 0 or len(dirty) > 0
        for l in range(w.n_layers):
            ref = A.dense_attention(*H.dense_f64(case, l), case.ctx_lens)
            assert GH.rowwise_rel_err(got[l], ref) <= tol
            assert np.abs(got[l] - ref).max() <= (1e-5 if dtype == I.DTYPE_F32 else 2e-2)
            # a context of one token: the output is that token's value row
            v0 = H.dense_f64(case, l)[2][0][0]                         # [Hkv][d] of sequence 0's only token
            assert np.allclose(got[l][0].astype(np.float64), np.repeat(v0, hq // hkv, axis=0), rtol=tol, atol=1e-6)
        mod.step(case.q, *new_token_rows(case), table, case.ctx_lens)
        assert_images_equal(lib, mod, staging=False)
        outs.append(got)
        lib.close()
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.parametrize("path", PATHS)
def test_step_on_one_stream_and_on_the_default_stream_gives_the_same_bits_and_bytes(path):
    """The three streams may be one: a single stream for everything, or none given (the default stream).  The
    appends, copies and write-backs then simply queue up in order; outputs and both pools' bytes are those of the
    three-stream step."""
    w = I.scaled(W, n_layers=4)
    outs = []
    for streams in ("three", "one", "default"):
        case = host_tails(I.make_case(w))
        n = int(case.n_blocks.sum())
        lib, mod, table = GH.make_pools(case, n, n, n, upto_ctx=case.ctx_lens - 1, fill=H.nan_fill(w.dtype))
        lib.set_swap_path(path)
        one = torch.cuda.Stream()
        ss = {"three": (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()), "one": (one, one, one),
              "default": (None, None, None)}[streams]
        for _ in range(2):                                             # the second step finds layer 0 staged
            got, pf, dirty = run_step(lib, case, table, ss)
        assert lib.check_errors() == 0 and len(dirty) > 0
        mod.step(case.q, *new_token_rows(case), table, case.ctx_lens)
        assert_images_equal(lib, mod, staging=False)
        outs.append(got)
        lib.close()
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    ref = A.dense_attention(*H.dense_f64(case, 0), case.ctx_lens)
    assert GH.rowwise_rel_err(outs[0][0], ref) <= 2e-3


def test_two_steps_in_a_row_and_timing_stats():
    w = I.scaled(W, n_layers=4)
    case = host_tails(I.make_case(w))
    n = int(case.n_blocks.sum())
    lib, mod, table = GH.make_pools(case, n, n, n, upto_ctx=case.ctx_lens - 2)
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    full_ctx = case.ctx_lens.copy()
    for back in (1, 0):
        case.ctx_lens = full_ctx - back
        got, pf, dirty = run_step(lib, case, table, streams, timing=True)
        mod.step(case.q, *new_token_rows(case), table, case.ctx_lens)
        for l in range(w.n_layers):
            ref = A.dense_attention(*H.dense_f64(case, l), case.ctx_lens)
            assert GH.rowwise_rel_err(got[l], ref) <= 2e-3
        assert_images_equal(lib, mod, staging=False)
        st = lib.stats()
        lt = lib.layer_times()
        # every layer's blocks, and layer 0's once more for the step that follows
        assert st.bytes_in == len(pf) * lib.block_bytes * (w.n_layers + 1 - st.first_layer_prestaged)
        assert st.bytes_out == len(dirty) * lib.block_bytes * w.n_layers
        assert st.step_ms > 0 and st.attn_ms > 0 and st.swap_in_ms > 0
        assert (lt["attn"] > 0).all() and (lt["swap_in"][st.first_layer_prestaged:] > 0).all() and (lt["stall"] >= 0).all()
        assert st.step_ms >= st.attn_ms * 0.99
    assert lib.check_errors() == 0
    lib.close()


def test_step_argument_checks():
    case = host_tails(I.make_case(W))
    lib, mod, table = GH.make_pools(case, 120, 4, 64)
    q = GH.to_dev(case.q, W.dtype)
    out = torch.empty_like(q)
    tb, cl = torch.from_numpy(table).to(GH.DEV), torch.from_numpy(case.ctx_lens).to(GH.DEV)
    pf, dirty = lib.prefetch_list(table, case.ctx_lens)
    with pytest.raises(B.PieError) as e:
        lib.step(q, None, None, tb, cl, pf, dirty, out)              # more host blocks than a staging region
    assert e.value.code == B.ENOMEM
    gpu_homed = [int(h) for h in table.ravel() if h >= 0 and mod.home[int(h)][0] == 0]
    with pytest.raises(B.PieError) as e:
        lib.step(q, None, None, tb, cl, gpu_homed[:2], [], out)
    assert e.value.code == B.ESTATE
    with pytest.raises(B.PieError) as e:
        lib.step(q, None, None, tb, cl, pf[:2], pf[2:3], out)        # dirty block not among the prefetched
    assert e.value.code == B.ESTATE
    lib.close()


@pytest.mark.parametrize("path", [B.SWAP_DMA, B.SWAP_KERNEL])
def test_monitoring_by_device_clock_agrees_with_events_and_changes_no_result(path):
    """The two ways of timing a step measure the same things (loosely: the runs differ, and events add gaps),
    and neither changes an output bit."""
    w = I.Workload("clock", 4, 12, 16, 4, 128, I.DTYPE_F16, ctx_lo=1500, ctx_hi=2500, value_scale=0.5, host_fraction=0.2, seed=53)
    case = host_tails(I.make_case(w))
    n = int(case.n_blocks.sum())
    lib, mod, table = GH.make_pools(case, n, n // 3, n // 3, upto_ctx=case.ctx_lens - 1)
    lib.set_swap_path(path)
    lib.set_cross_step_prefetch(False)          # every step alike: all layers' copies inside the step
    lib.set_layer_compute_us(150.0)
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    res = {}
    # every figure is the smallest of a few steps: a host thread that loses the processor for a scheduling quantum
    # in the middle of a step (the copy-engine path is paced by the host) adds milliseconds to whatever was running
    for mode in (B.TIMING_OFF,) + (B.TIMING_EVENTS, B.TIMING_CLOCK) * 4:
        got, pf, dirty = run_step(lib, case, table, streams, timing=mode)
        if mode == B.TIMING_OFF:
            with pytest.raises(B.PieError) as e:
                lib.layer_times()
            assert e.value.code == B.ESTATE
            base = got
            continue
        assert np.array_equal(got, base)
        st = lib.stats()
        new = (lib.layer_times(), st.step_ms, st.attn_ms, st.swap_in_ms, st.stall_ms)
        if mode in res:
            old = res[mode]
            new = ({k: np.minimum(old[0][k], new[0][k]) for k in new[0]},) + tuple(min(a, b) for a, b in zip(old[1:], new[1:]))
        res[mode] = new
    assert lib.check_errors() == 0
    (le, step_e, attn_e, in_e, stall_e), (lc, step_c, attn_c, in_c, stall_c) = res[B.TIMING_EVENTS], res[B.TIMING_CLOCK]
    for key in ("attn", "kernel", "swap_in", "swap_out"):
        assert (lc[key] > 0).all() and (le[key] > 0).all(), key
        # with the gather kernel on the swap stream the decode kernel's last workgroups may have to wait for a
        # compute unit, differently from run to run: only the copy-engine path is compared closely
        if path == B.SWAP_DMA:
            assert np.allclose(lc[key], le[key], rtol=0.5, atol=0.04), (key, lc[key], le[key])
        else:
            assert (lc[key] < 5.0).all(), (key, lc[key])
    assert (lc["attn"] >= 0.150).all() and (lc["attn"] >= lc["kernel"]).all()     # the stand-in is part of a layer
    assert (lc["stall"] >= 0).all() and lc["stall"][0] > 0                        # layer 0's prefetch hides behind nothing
    assert step_c >= attn_c * 0.99
    if path == B.SWAP_DMA:
        assert step_c == pytest.approx(step_e, rel=0.5)
        assert in_c == pytest.approx(in_e, rel=0.5, abs=0.05)
    lib.close()


@pytest.mark.parametrize("path", [B.SWAP_DMA, B.SWAP_KERNEL])
def test_first_layer_staged_behind_the_previous_step(path):
    """Consecutive tokens with the same host blocks: from the second step on layer 0's blocks are already in
    their staging region (brought in behind the previous step's last layer), results and pool bytes stay those
    of the model, and anything that changes a staged block makes the next step copy again."""
    w = I.scaled(W, n_layers=4)
    case = I.make_case(w)
    c = case.ctx_lens.astype(np.int64)
    base = np.where((c - 1) % 16 >= 3, c, ((c - 1) // 16) * 16).astype(np.int32)   # base-3 .. base share a block
    for b in range(0, w.batch, 2):
        case.host_mask[b][(int(base[b]) - 1) // 16] = True                           # host-homed tails
    n = int(case.n_blocks.sum())
    case.ctx_lens = base
    lib, mod, table = GH.make_pools(case, n, n, n, upto_ctx=base - 4)
    lib.set_swap_path(path)
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    L, bb = w.n_layers, lib.block_bytes

    def one(ctx, expect_hit, timing):
        case.ctx_lens = ctx
        got, pf, dirty = run_step(lib, case, table, streams, timing=timing)
        ref = mod.step(case.q, *new_token_rows(case), table, case.ctx_lens)
        assert GH.rowwise_rel_err(got, ref) <= 2e-3
        for l in range(L):
            assert GH.rowwise_rel_err(got[l], A.dense_attention(*H.dense_f64(case, l), case.ctx_lens)) <= 2e-3
        assert_images_equal(lib, mod, staging=False)
        st = lib.stats()
        assert st.first_layer_prestaged == (1 if expect_hit else 0)
        assert len(dirty) > 0
        return st, pf

    for i, timing in enumerate((B.TIMING_OFF, B.TIMING_CLOCK, B.TIMING_CLOCK, B.TIMING_EVENTS, B.TIMING_EVENTS)):
        st, pf = one(base - 3 + min(i, 3), expect_hit=i > 0, timing=timing)
        assert st.bytes_in == len(pf) * bb * (L + (0 if i > 0 else 1))
        if timing:
            lt = lib.layer_times()
            assert lt["swap_in"][0] == 0 and (lt["swap_in"][1:] > 0).all()
            # (what is left of a copy that was started behind the step before; the bound only has to tell it from
            # garbage - a host thread that loses the processor mid-step can add milliseconds)
            assert 0 <= lt["stall"][0] < 100.0 and st.stall_ms >= lt["stall"][0]
    # a staged block moves to the GPU pool: the next step must not trust the region
    lib.migrate([int(pf[0])], B.GPU, streams[1])
    lib.sync()
    mod.migrate([int(pf[0])], B.GPU)
    st, pf2 = one(base, expect_hit=False, timing=B.TIMING_OFF)
    assert len(pf2) == len(pf) - 1
    st, _ = one(base, expect_hit=True, timing=B.TIMING_OFF)
    # a block is freed and its handle comes back in another host slot
    lib.set_cross_step_prefetch(False)
    st, _ = one(base, expect_hit=False, timing=B.TIMING_OFF)
    assert st.bytes_in == len(pf2) * bb * L
    st, _ = one(base, expect_hit=False, timing=B.TIMING_OFF)
    lib.set_cross_step_prefetch(True)
    st, _ = one(base, expect_hit=False, timing=B.TIMING_OFF)
    st, _ = one(base, expect_hit=True, timing=B.TIMING_OFF)
    lib.swap_in(0, pf2[:-1], streams[1])                              # someone else uses region 0 in between
    mod.swap_in(0, pf2[:-1].tolist())
    st, _ = one(base, expect_hit=False, timing=B.TIMING_OFF)
    assert lib.check_errors() == 0
    lib.close()


def test_device_clock_with_the_fp32_kernel():
    """The fp32 kernel has no persistent grid: its workgroups fold their times into the layer's row directly."""
    w = I.scaled(W, dtype=I.DTYPE_F32, n_q_heads=8, n_kv_heads=8, head_dim=64, n_layers=3)
    case = host_tails(I.make_case(w))
    n = int(case.n_blocks.sum())
    lib, mod, table = GH.make_pools(case, n, n, n, upto_ctx=case.ctx_lens - 1)
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    base, _, _ = run_step(lib, case, table, streams, timing=B.TIMING_OFF)
    for _ in range(2):
        got, pf, dirty = run_step(lib, case, table, streams, timing=B.TIMING_CLOCK)
        assert np.array_equal(got, base)
        lt, st = lib.layer_times(), lib.stats()
        assert (lt["kernel"] > 0).all() and (lt["kernel"] < 5.0).all() and (lt["attn"] >= lt["kernel"]).all()
        assert (lt["swap_in"][st.first_layer_prestaged:] > 0).all() and (lt["swap_out"] > 0).all()
        assert st.step_ms >= lt["attn"].sum() * 0.99 and st.step_ms < 50.0
    assert lib.check_errors() == 0
    lib.close()


def test_block_addresses_point_into_the_callers_buffers():
    """pie_block_address names the bytes of (pool, layer, slot) inside the memory the caller handed over: writing a
    block through that address and reading it through the pool's image gives the same bytes."""
    case = I.make_case(I.scaled(W, n_layers=3))
    n = int(case.n_blocks.sum())
    lib, mod, table = GH.make_pools(case, n, 4, n, upto_ctx=case.ctx_lens - 1)
    g, h = lib.gpu_image(), lib.host_image()
    for layer, slot in ((0, 0), (2, n - 1), (1, n + 3), (1, n + 2 * 4 - 1)):      # resident and staging slots
        assert lib.block_address(B.GPU, layer, slot) == g[layer, slot].data_ptr()
    for layer, slot in ((0, 0), (2, n - 1)):
        assert lib.block_address(B.HOST, layer, slot) == h[layer, slot].data_ptr()
    for where, layer, slot in ((B.GPU, 3, 0), (B.GPU, 0, n + 8), (B.HOST, 0, n), (2, 0, 0),
                               (B.GPU, -1, 0), (B.HOST, 0, -1)):
        with pytest.raises(B.PieError) as e:
            lib.block_address(where, layer, slot)
        assert e.value.code == B.EINVAL
    lib.close()


def test_gather_workgroups_and_host_presence_check_change_no_result():
    """Two knobs of the swap path that must not show in any byte: how many workgroups the gather kernel uses
    (bounds checked), and whether the host looks for a layer's swap-in itself before queuing the layer."""
    w = I.scaled(W, n_layers=4)
    case = host_tails(I.make_case(w))
    n = int(case.n_blocks.sum())
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    outs, images = [], []
    for path, wgs, check in ((B.SWAP_KERNEL, 64, True), (B.SWAP_KERNEL, 1, True), (B.SWAP_KERNEL, 7, True),
                             (B.SWAP_KERNEL, 1024, True), (B.SWAP_DMA, 64, True), (B.SWAP_DMA, 64, False)):
        lib, mod, table = GH.make_pools(case, n, n, n, upto_ctx=case.ctx_lens - 1)
        lib.set_swap_path(path)
        lib.set_swap_workgroups(wgs)
        lib.set_host_presence_check(check)
        for _ in range(2):                                                    # the second step finds layer 0 staged
            got, pf, dirty = run_step(lib, case, table, streams)
        assert lib.check_errors() == 0 and len(pf) > 0 and len(dirty) > 0
        outs.append(got)
        images.append(GH.images_of(lib)[1].copy())
        for bad in (0, -3, 1025):
            with pytest.raises(B.PieError) as e:
                lib.set_swap_workgroups(bad)
            assert e.value.code == B.EINVAL
        lib.close()
    ref = [A.dense_attention(*H.dense_f64(case, l), case.ctx_lens) for l in range(w.n_layers)]
    for l in range(w.n_layers):
        assert GH.rowwise_rel_err(outs[0][l], ref[l]) <= 2e-3
    for got, img in zip(outs[1:], images[1:]):
        assert np.array_equal(got, outs[0]) and np.array_equal(img, images[0])


@pytest.mark.parametrize("path", PATHS)
def test_asynchronous_submission_changes_no_result_and_frees_the_caller(path):
    """pie_set_async_submit: steps handed to the pool's own thread give the bytes and outputs of steps enqueued by
    the caller, in the order given; pie_step returns without waiting; argument errors are still returned by
    pie_step itself; calls that change residency cannot overtake a step."""
    import time
    w = I.scaled(W, n_layers=6, batch=6)
    case = host_tails(I.make_case(w))
    n = int(case.n_blocks.sum())
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    k_new, v_new = new_token_rows(case)
    q = GH.to_dev(case.q, w.dtype)
    dk, dv = GH.to_dev(k_new, w.dtype), GH.to_dev(v_new, w.dtype)
    d_ctx = torch.from_numpy(case.ctx_lens).to(GH.DEV)
    results = {}
    for mode in ("caller", "thread"):
        lib, mod, table = GH.make_pools(case, n, n, n, upto_ctx=case.ctx_lens - 1)
        lib.set_swap_path(path)
        lib.set_async_submit(mode == "thread")
        d_table = torch.from_numpy(table).to(GH.DEV)
        pf, dirty = lib.prefetch_list(table, case.ctx_lens)
        outs = [torch.full_like(q, float("nan")) for _ in range(4)]
        torch.cuda.synchronize()
        host = []
        for i in range(4):                                            # four steps in a row, nothing in between
            t0 = time.perf_counter()
            lib.step(q, dk, dv, d_table, d_ctx, pf, dirty, outs[i], *streams)
            host.append(time.perf_counter() - t0)
        if mode == "thread":
            with pytest.raises(B.PieError) as e:                      # checked in the caller's thread, as ever
                lib.step(q, dk, dv, d_table, d_ctx, pf[::-1].tolist() + [pf[0]], dirty, outs[0], *streams)
            assert e.value.code == B.ESTATE
            lib.step_join()                                           # everything is on the streams now
        # a residency change right behind the steps: it must wait for them, and the last step's write-back
        lib.migrate(pf[: len(pf) // 2], B.GPU, streams[1])
        lib.sync()
        torch.cuda.synchronize()
        assert lib.check_errors() == 0
        results[mode] = ([GH.from_dev(o, w.dtype) for o in outs], GH.images_of(lib), host)
        lib.set_async_submit(False)
        lib.close()
    ref = [A.dense_attention(*H.dense_f64(case, l), case.ctx_lens) for l in range(w.n_layers)]
    for l in range(w.n_layers):
        assert GH.rowwise_rel_err(results["caller"][0][0][l], ref[l]) <= 2e-3
    for a, b in zip(results["caller"][0], results["thread"][0]):
        assert np.array_equal(a, b)
    assert np.array_equal(results["caller"][1][0], results["thread"][1][0])          # device pool, staging included
    assert np.array_equal(results["caller"][1][1], results["thread"][1][1])          # host pool
    # handing a step over costs less than enqueuing it (a handful of list copies against dozens of launches)
    assert np.median(results["thread"][2]) < np.median(results["caller"][2])
