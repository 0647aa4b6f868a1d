"""Pins for oracle/pool_model.py: conservation, byte-identical round trips, error
codes, and a dictionary brute force of the allocator policy."""
import hashlib

import numpy as np
import pytest

import helpers as H
from oracle.pool_model import EINVAL, ENOMEM, ESTATE, GPU, HOST, PoolError, PoolModel
from paper_2411_09317_amd import inputs as I

W = I.Workload("pool", 3, 4, 4, 2, 8, I.DTYPE_F16, block_tokens=4, ctx_lo=5, ctx_hi=30, value_scale=1.0,
               host_fraction=0.3, seed=21)


def fresh(n_gpu=40, n_stage=16, n_host=24, w=W):
    return PoolModel(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_tokens, w.dtype, n_gpu, n_stage, n_host)


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def check_conservation(m):
    used = {GPU: set(), HOST: set()}
    for h, (w, s) in m.home.items():
        assert s not in used[w]
        used[w].add(s)
    assert len(used[GPU]) + m.n_free(GPU) == m.n_gpu
    assert len(used[HOST]) + m.n_free(HOST) == m.n_host
    assert len(m.home) + len(m.free_handles) == m.n_handles
    assert not (set(m.home) & m.free_handles)


def test_allocator_policy_matches_bruteforce_dictionary():
    """Lowest free handle, lowest free slot: replay a random alloc/free script
    against a naive list-scan implementation."""
    m = fresh()
    rng = np.random.Generator(np.random.PCG64(5))
    free_h = list(range(m.n_handles))
    free_s = {GPU: list(range(m.n_gpu)), HOST: list(range(m.n_host))}
    live = {}
    for _ in range(400):
        if live and rng.random() < 0.45:
            k = int(rng.integers(1, min(4, len(live)) + 1))
            victims = [int(x) for x in rng.choice(sorted(live), size=k, replace=False)]
            m.block_free(victims)
            for h in victims:
                w, s = live.pop(h)
                free_h.append(h)
                free_s[w].append(s)
        else:
            where = int(rng.integers(0, 2))
            n = int(rng.integers(1, 5))
            if n > len(free_s[where]):
                with pytest.raises(PoolError) as e:
                    m.block_alloc(where, n)
                assert e.value.code == ENOMEM
                continue
            got = m.block_alloc(where, n)
            exp = []
            for _i in range(n):
                h = min(free_h); free_h.remove(h)
                s = min(free_s[where]); free_s[where].remove(s)
                live[h] = (where, s)
                exp.append(h)
            assert got == exp
            wh, sl = m.block_where(got)
            assert list(zip(wh, sl)) == [live[h] for h in got]
        check_conservation(m)


def test_alloc_is_all_or_nothing_and_errors():
    m = fresh(n_gpu=3, n_stage=2, n_host=2)
    a = m.block_alloc(GPU, 2)
    with pytest.raises(PoolError) as e:
        m.block_alloc(GPU, 2)
    assert e.value.code == ENOMEM
    assert m.n_free(GPU) == 1
    with pytest.raises(PoolError) as e:
        m.block_alloc(2, 1)
    assert e.value.code == EINVAL
    m.block_free(a[:1])
    with pytest.raises(PoolError) as e:
        m.block_free(a[:1])                     # double free
    assert e.value.code == ESTATE
    with pytest.raises(PoolError) as e:
        m.block_free([a[1], a[1]])              # repeated handle: nothing is freed
    assert e.value.code == ESTATE
    assert m.block_where([a[1]]) == ([GPU], [1])
    with pytest.raises(PoolError) as e:
        m.block_free([99])
    assert e.value.code == EINVAL
    assert m.block_where([a[0]]) == ([-1], [-1])
    check_conservation(m)


def make_case_with_host_tails(w=W):
    case = I.make_case(w)
    for b in range(0, w.batch, 2):               # every other sequence's last block lives on the host
        case.host_mask[b][-1] = True
    return case


def populated(w=W, **kw):
    case = make_case_with_host_tails(w)
    m = fresh(w=w, **kw)
    table = H.allocate(m, case, H.plan_allocation(case))
    where, slot = H.home_maps(m, table)
    g, h = H.build_images(case, table, where, slot, m.n_gpu, m.n_host)
    m.gpu[:, : m.n_gpu] = g
    m.host[:] = h
    return case, m, table


def test_swap_round_trip_is_byte_identical():
    case, m, table = populated()
    plist = m.prefetch_list(table, case.ctx_lens)
    assert plist, "case must have host-homed blocks"
    before_host, before_gpu = digest(m.host), digest(m.gpu[:, : m.n_gpu])
    for layer in range(W.n_layers):
        m.swap_in(layer, plist)
        r = layer & 1
        for i, h in enumerate(plist):            # staged copy == host copy, at slot = rank
            assert np.array_equal(m.gpu[layer, m.stage_slot(r, i)], m.host[layer, m.home[h][1]])
        m.swap_out(layer, plist)
    assert digest(m.host) == before_host and digest(m.gpu[:, : m.n_gpu]) == before_gpu


def test_swap_out_writes_what_staging_holds():
    case, m, table = populated()
    plist = m.prefetch_list(table, case.ctx_lens)
    m.swap_in(1, plist)
    s = m.stage_slot(1, 0)
    m.gpu[1, s] = np.float16(7.0)
    m.swap_out(1, plist[:1])
    assert (m.host[1, m.home[plist[0]][1]] == np.float16(7.0)).all()
    # other layers of that block untouched
    assert not (m.host[0, m.home[plist[0]][1]] == np.float16(7.0)).all()


def test_swap_state_errors():
    case, m, table = populated()
    plist = m.prefetch_list(table, case.ctx_lens)
    gpu_homed = [int(h) for h in table.ravel() if h >= 0 and m.home[int(h)][0] == GPU]
    with pytest.raises(PoolError) as e:
        m.swap_in(0, gpu_homed[:1])              # not host-homed
    assert e.value.code == ESTATE
    with pytest.raises(PoolError) as e:
        m.swap_in(W.n_layers, plist)
    assert e.value.code == EINVAL
    with pytest.raises(PoolError) as e:
        m.swap_in(0, plist + plist)              # more than a staging region / repeated
    assert e.value.code in (ENOMEM, ESTATE)
    m.swap_in(0, plist)
    with pytest.raises(PoolError) as e:
        m.swap_out(2, plist)                     # region 0 holds layer 0, not layer 2
    assert e.value.code == ESTATE
    m.swap_in(0, plist[:1])
    with pytest.raises(PoolError) as e:
        m.swap_out(0, plist[1:2])                # no longer staged
    assert e.value.code == ESTATE


def test_migrate_keeps_handles_bytes_and_conservation():
    case, m, table = populated()
    out0 = m.attn_decode(0, case.q[0], table, case.ctx_lens)
    handles = sorted(m.home)
    contents = {h: m.read_block(2, h).copy() for h in handles}
    movers = handles[::3]
    m.migrate(movers, HOST)
    check_conservation(m)
    assert all(m.home[h][0] == HOST for h in movers)
    m.migrate(handles[1::3], GPU)
    check_conservation(m)
    for h in handles:
        np.testing.assert_array_equal(m.read_block(2, h), contents[h])
    np.testing.assert_array_equal(m.attn_decode(0, case.q[0], table, case.ctx_lens), out0)
    spare = m.block_alloc(HOST, m.n_free(HOST))  # fill the host pool: nothing more can be demoted
    homes = dict(m.home)
    with pytest.raises(PoolError) as e:
        m.migrate(handles, HOST)
    assert e.value.code == ENOMEM
    assert m.home == homes                       # all or nothing
    m.block_free(spare)
    check_conservation(m)


def test_set_host_fraction_nested_sets():
    case, m, table = populated(n_gpu=60, n_host=60)
    order = [int(table[b, j]) for b, j in I.draw_promotion_order(W, case.n_blocks)]
    base = m.attn_decode(1, case.q[1], table, case.ctx_lens)
    prev = set()
    for f in (0.0, 0.1, 0.3, 0.6, 1.0, 0.3, 0.0):
        k = m.set_host_fraction(f, order)
        assert k == int(np.floor(f * len(order) + 0.5))
        host_set = {h for h in order if m.home[h][0] == HOST}
        assert host_set == set(order[:k])
        assert prev <= host_set or host_set <= prev
        prev = host_set
        check_conservation(m)
        np.testing.assert_array_equal(m.attn_decode(1, case.q[1], table, case.ctx_lens), base)


def test_step_matches_dense_oracle_and_writes_back():
    """The pipeline's result is plain attention over the context including the
    appended token, whatever is host-resident; afterwards both homes hold it."""
    from oracle import attention as A
    case = make_case_with_host_tails()
    m = fresh()
    table = H.allocate(m, case, H.plan_allocation(case))
    where, slot = H.home_maps(m, table)
    g, h = H.build_images(case, table, where, slot, m.n_gpu, m.n_host, upto_ctx=case.ctx_lens - 1)
    m.gpu[:, : m.n_gpu] = g
    m.host[:] = h
    k_new = np.stack([np.stack([case.k_dense[b][l, case.ctx_lens[b] - 1] for b in range(W.batch)]) for l in range(W.n_layers)])
    v_new = np.stack([np.stack([case.v_dense[b][l, case.ctx_lens[b] - 1] for b in range(W.batch)]) for l in range(W.n_layers)])
    out = m.step(case.q, k_new, v_new, table, case.ctx_lens)
    for l in range(W.n_layers):
        q, K, V = H.dense_f64(case, l)
        np.testing.assert_allclose(out[l], A.dense_attention(q, K, V, case.ctx_lens), rtol=1e-12, atol=1e-14)
    full_g, full_h = H.build_images(case, table, where, slot, m.n_gpu, m.n_host)
    assert digest(m.gpu[:, : m.n_gpu]) == digest(full_g)
    assert digest(m.host) == digest(full_h)
    # some tail block really was host-homed, so the write-back path was exercised
    tails = [int(table[b, (case.ctx_lens[b] - 1) // W.block_tokens]) for b in range(W.batch)]
    assert any(m.home[t][0] == HOST for t in tails)


def test_append_to_unstaged_host_block_is_an_error():
    case, m, table = populated()
    tails = [int(table[b, (case.ctx_lens[b] - 1) // W.block_tokens]) for b in range(W.batch)]
    assert any(m.home[t][0] == HOST for t in tails)
    k = np.zeros((W.batch, W.n_kv_heads, W.head_dim), dtype=np.float16)
    with pytest.raises(PoolError) as e:
        m.kv_append(0, k, k, table, case.ctx_lens)
    assert e.value.code == ESTATE


def test_prefetch_list_is_the_host_homed_set_in_host_slot_order():
    case, m, table = populated()
    plist = m.prefetch_list(table, case.ctx_lens)
    want = {int(table[b, j]) for b in range(W.batch) for j in range(int(case.n_blocks[b]))
            if m.home[int(table[b, j])][0] == 1}
    assert set(plist) == want and len(plist) == len(want)
    slots = [m.home[h][1] for h in plist]
    assert slots == sorted(slots)
