"""The iteration-level scheduler and its block budget, on the CPU.

The block store is the oracle's pool model (same allocator policy as the library: lowest free handle and slot
first), time is virtual (one iteration = one tick).  What is checked is what the paper's block manager and its
grow / shrink rules fix (Section 4.1): blocks are handed out on demand and all come back, nothing is promised
beyond the visible capacity, a larger capacity means a larger batch, and a shrink hides blocks before they are
given up.
"""
import numpy as np
import pytest

from oracle import serving_sim
from oracle.pool_model import GPU, HOST, PoolModel
from paper_2411_09317_amd import inputs as I
from paper_2411_09317_amd import serving as S

T = 16


def store(n_gpu, n_host):
    return PoolModel(1, 1, 1, 8, T, I.DTYPE_F32, n_gpu, n_host, n_host)


def requests(n=200, rate=1000.0, seed=11, lo=8, hi=48):
    w = I.scaled(I.CONFIGS["cfg1"], ctx_lo=16, ctx_hi=200, seed=seed)
    a, p, o = I.draw_requests(w, n, rate, lo, hi)
    return [S.Request(i, float(a[i]), int(p[i]), int(o[i])) for i in range(n)]


def run(sched, reqs, dt=1e-3, on_iteration=None, promote=True, max_iters=100000):
    for r in reqs:
        sched.submit(r)
    now, it, batches = 0.0, 0, []
    while not sched.idle:
        sched.admit(now)
        if promote:
            sched.promote()
        if not sched.running:
            now = max(now, sched.waiting[0].arrival)
            continue
        table, ctx = sched.tables()
        for b, r in enumerate(sched.running):                      # a row holds exactly the blocks its context needs
            assert (table[b] >= 0).sum() == (ctx[b] + T - 1) // T == len(r.handles)
        assert sched.blocks_in_use <= sched.reserved
        batches.append(len(sched.running))
        if on_iteration:
            on_iteration(it, sched)
        now += dt
        sched.complete_iteration(now)
        it += 1
        assert it < max_iters
    return np.array(batches), now


def test_hand_worked_admission_first_come_first_served():
    """4 GPU blocks of 16 tokens.  A needs 2 blocks over its life, B 3, C 1: at level 0 B does not fit beside A
    and C waits behind B although it would fit; one unit of 2 host blocks admits all three at once."""
    mk = lambda: [S.Request(0, 0.0, 20, 12), S.Request(1, 0.0, 40, 8), S.Request(2, 0.0, 10, 6)]
    st = store(4, 2)
    sc = S.Scheduler(st, T, S.BlockBudget(4, 2, 1), 8, 4)
    for r in mk():
        sc.submit(r)
    assert sc.admit(0.0) == 1 and [r.rid for r in sc.running] == [0] and sc.reserved == 2
    assert [r.rid for r in sc.waiting] == [1, 2]
    st = store(4, 2)
    bud = S.BlockBudget(4, 2, 1)
    bud.set_level(1)
    assert bud.capacity == 6 and bud.expansion == 1.5
    sc = S.Scheduler(st, T, bud, 8, 4)
    for r in mk():
        sc.submit(r)
    assert sc.admit(0.0) == 3 and sc.reserved == 6
    # contexts 21, 41, 11 -> 2 + 3 + 1 blocks now; the GPU pool's 4 go first, then 2 host blocks
    assert [len(r.handles) for r in sc.running] == [2, 3, 1]
    assert st.n_free(GPU) == 0 and st.n_free(HOST) == 0 and len(sc.on_host) == 2
    where, _ = st.block_where(sc.running[0].handles + sc.running[1].handles + sc.running[2].handles)
    assert where == [GPU, GPU, GPU, GPU, HOST, HOST]


@pytest.mark.parametrize("level", [0, 1, 3])
def test_every_request_finishes_in_order_and_every_block_comes_back(level):
    st = store(96, 3 * 24)
    bud = S.BlockBudget(96, 24, 3)
    bud.set_level(level)
    sc = S.Scheduler(st, T, bud, 64, 16)
    reqs = requests()
    peak = [0]

    def watch(it, s):
        assert s.reserved <= bud.capacity
        peak[0] = max(peak[0], s.blocks_in_use)
        assert len(s.on_host) == st.n_host - st.n_free(HOST)
        assert s.blocks_in_use == (st.n_gpu - st.n_free(GPU)) + len(s.on_host)

    run(sc, reqs, on_iteration=watch)
    assert len(sc.done) == len(reqs) and all(r.generated == r.output_len for r in reqs)
    adm = [r.admitted for r in reqs]
    assert adm == sorted(adm)                                        # first come first served
    assert all(r.admitted >= r.arrival and r.finished > r.admitted for r in reqs)
    assert st.n_free(GPU) == 96 and st.n_free(HOST) == 72 and sc.reserved == 0 and not sc.on_host
    assert peak[0] <= bud.capacity
    if level == 0:
        assert st.n_free(HOST) == 72 and sc.n_promoted == 0           # the host pool is never touched


def test_a_larger_budget_is_a_larger_batch():
    """Under saturation the mean batch grows with the capacity (the premise of the method), and the same
    requests need fewer iterations."""
    means, iters = [], []
    for level in (0, 1, 2, 4):
        st = store(128, 4 * 32)
        bud = S.BlockBudget(128, 32, 4)
        bud.set_level(level)
        sc = S.Scheduler(st, T, bud, 256, 16)
        b, _ = run(sc, requests(n=400, rate=1e6))
        means.append(b[: len(b) * 3 // 4].mean())
        iters.append(len(b))
    assert all(x < y for x, y in zip(means, means[1:])) and all(x > y for x, y in zip(iters, iters[1:]))
    for level, m in zip((1, 2, 4), means[1:]):
        assert m / means[0] == pytest.approx(1 + level * 32 / 128, rel=0.12)


def test_shrink_hides_blocks_first_and_gives_them_up_later():
    st = store(64, 64)
    bud = S.BlockBudget(64, 32, 2)
    bud.set_level(2)
    sc = S.Scheduler(st, T, bud, 256, 16)
    seen = {"host_at_shrink": None, "host": [], "over": []}

    def watch(it, s):
        if it == 30:
            assert len(s.on_host) > 0 and s.reserved > 64           # the expansion is in use
            bud.set_level(0)
            seen["host_at_shrink"] = len(s.on_host)
            seen["n_running"] = len(s.running) + len(s.done)
        if it > 30:
            seen["host"].append(len(s.on_host))
            assert len(s.on_host) <= max(0, s.reserved - 64)        # never more than what was promised beyond the GPU pool
            if s.reserved > bud.capacity:                           # still over the new capacity: nothing was admitted
                assert len(s.running) + len(s.done) == seen["n_running"]
                seen["over"].append(s.reserved)
            seen["n_running"] = len(s.running) + len(s.done)

    reqs = requests(n=300, rate=1e6)
    run(sc, reqs, on_iteration=watch)
    assert seen["host_at_shrink"] > 0
    assert len(sc.done) == 300                                       # running requests kept their blocks and ended
    o = seen["over"]
    assert len(o) > 1 and all(a >= b for a, b in zip(o, o[1:]))      # the promise shrinks as requests end
    h = seen["host"]
    assert max(h[len(o):], default=0) == 0 and h[-1] == 0            # under the new capacity no host block is left
    assert sc.n_promoted > 0                                         # some by moving into freed GPU slots
    assert st.n_free(HOST) == 64


def test_host_blocks_only_when_the_gpu_pool_is_full_and_promotion_fills_it_again():
    st = store(32, 32)
    bud = S.BlockBudget(32, 32, 1)
    bud.set_level(1)
    sc = S.Scheduler(st, T, bud, 64, 16)

    def watch(it, s):
        # after admit + promote: either nothing is on the host or the GPU pool has no free slot
        assert not s.on_host or st.n_free(GPU) == 0

    run(sc, requests(n=120, rate=1e6), on_iteration=watch)
    assert sc.n_promoted > 0


def test_request_stream_is_seeded_and_poisson_shaped():
    w = I.scaled(I.CONFIGS["cfg4"])
    a1, p1, o1 = I.draw_requests(w, 4000, 50.0, 64, 256)
    a2, p2, o2 = I.draw_requests(w, 4000, 50.0, 64, 256)
    assert np.array_equal(a1, a2) and np.array_equal(p1, p2) and np.array_equal(o1, o2)
    gaps = np.diff(np.concatenate([[0.0], a1]))
    assert gaps.min() > 0 and gaps.mean() == pytest.approx(1 / 50.0, rel=0.05)
    assert gaps.std() == pytest.approx(gaps.mean(), rel=0.1)         # exponential gaps: std = mean
    assert p1.min() >= w.ctx_lo and p1.max() <= w.ctx_hi and o1.min() >= 64 and o1.max() <= 256
    assert np.median(p1) == pytest.approx(w.ctx_median, rel=0.1)


def test_summary_splits_latency_into_queueing_and_decoding():
    done = [S.Request(0, 0.0, 10, 4, admitted=1.0, finished=3.0), S.Request(1, 0.5, 10, 6, admitted=1.5, finished=4.5)]
    s = S.summarize(done, 5.0)
    assert s["tokens"] == 10 and s["tokens_per_s"] == 2.0
    assert s["queue_s_mean"] == 1.0 and s["decode_s_mean"] == 2.5 and s["latency_s_mean"] == 3.5
    assert s["decode_ms_per_token_mean"] == pytest.approx(500.0)


def test_argument_checks():
    with pytest.raises(ValueError):
        S.BlockBudget(0, 1, 1)
    bud = S.BlockBudget(8, 2, 1)
    with pytest.raises(ValueError):
        bud.set_level(2)
    sc = S.Scheduler(store(8, 2), T, bud, 4, 2)
    with pytest.raises(ValueError):
        sc.submit(S.Request(0, 0.0, 40, 8))                          # 3 blocks over its life, rows hold 2


@pytest.mark.parametrize("levels", [lambda it: 0, lambda it: 2, lambda it: 2 if it < 40 else 0,
                                    lambda it: (it // 25) % 3])
def test_scheduler_agrees_with_the_counting_model_iteration_by_iteration(levels):
    """The product scheduler over a block store against a model that only counts: same batch in every
    iteration, same blocks held and promised, same admission and last iteration for every request - also
    while the budget level moves up and down."""
    rng = np.random.Generator(np.random.PCG64(5))
    n = 150
    arrival = np.sort(rng.integers(0, 120, size=n)).tolist()
    prompt = rng.integers(10, 200, size=n).tolist()
    output = rng.integers(1, 40, size=n).tolist()
    trace, adm, fin = serving_sim.simulate(arrival, prompt, output, 64, 16, levels, T, max_batch=24)
    st = store(64, 2 * 16 + 64)
    bud = S.BlockBudget(64, 16, 2)
    sc = S.Scheduler(st, T, bud, 24, 16)
    for i in range(n):
        sc.submit(S.Request(i, float(arrival[i]), prompt[i], output[i]))
    now, got = 0, []
    while not sc.idle:
        bud.set_level(levels(now))
        sc.admit(float(now))
        sc.promote()
        if not sc.running:
            now = int(sc.waiting[0].arrival)
            continue
        got.append((now, [r.rid for r in sc.running], sc.blocks_in_use, sc.reserved))
        sc.complete_iteration(float(now))
        now += 1
    assert got == trace
    assert [int(r.admitted) for r in sorted(sc.done, key=lambda r: r.rid)] == adm
    assert [int(r.finished) for r in sorted(sc.done, key=lambda r: r.rid)] == fin


def test_counting_model_on_a_hand_worked_stream():
    """4 blocks of 16 tokens, no expansion.  A (20 + 12 tokens: 2 blocks over its life) runs iterations 0-11;
    B (40 + 8: 3 blocks) does not fit beside it and starts at 12; C (10 + 6: 1 block) arrived at 0 too but waits
    behind B, joins it at 12 (3 + 1 = 4 blocks) and ends at 17; B ends at 19."""
    trace, adm, fin = serving_sim.simulate([0, 0, 0], [20, 40, 10], [12, 8, 6], 4, 2, lambda it: 0, 16)
    assert adm == [0, 12, 12] and fin == [11, 19, 17]
    assert [t[1] for t in trace[:12]] == [[0]] * 12 and trace[12][1] == [1, 2] and trace[18][1] == [1]
    assert trace[0][2:] == (2, 2) and trace[12][2:] == (4, 4)      # 21 tokens -> 2 blocks; 41 -> 3, 11 -> 1
    # one unit of 2 host blocks more: all three at once, 6 blocks promised
    trace, adm, fin = serving_sim.simulate([0, 0, 0], [20, 40, 10], [12, 8, 6], 4, 2, lambda it: 1, 16)
    assert adm == [0, 0, 0] and fin == [11, 7, 5] and trace[0][1:] == ([0, 1, 2], 6, 6)


def test_index_store_hands_out_the_lowest_free_index_below_its_limit():
    st = S.IndexStore(16, 6)
    assert st.n_free(GPU) == 6 and st.n_free(HOST) == 0 and st.live_end() == 0
    assert st.block_alloc(GPU, 4) == [0, 1, 2, 3]
    st.block_free([1, 2])
    assert st.block_alloc(GPU, 3) == [1, 2, 4] and st.live_end() == 5 and st.n_free(GPU) == 1
    with pytest.raises(MemoryError):
        st.block_alloc(GPU, 2)
    st.limit = 10                                                    # the caches have grown
    assert st.block_alloc(GPU, 2) == [5, 6] and st.n_free(GPU) == 3
    st.block_free([6, 5, 4])
    assert st.live_end() == 4 and st.block_where([3, 0]) == ([GPU, GPU], [3, 0])


def test_scheduler_over_an_index_store_follows_a_capacity_that_moves():
    class Shown:                                                     # stands for the elastic pool's visible size
        capacity = 24
        expansion = 1.0
    bud, st = Shown(), S.IndexStore(64, 24)
    sc = S.Scheduler(st, T, bud, 64, 16)
    for r in requests(n=120, rate=1e6):
        sc.submit(r)
    it, peak = 0, []
    while not sc.idle:
        if it == 20:
            bud.capacity, st.limit = 40, 40                          # growth shows
        if it == 60:
            bud.capacity = 24                                        # a shrink hides at once; the blocks still exist
        if it > 60 and st.limit == 40 and st.live_end() <= 24:
            st.limit = 24                                            # given up: the cut can be made
        sc.admit(1.0)
        assert sc.running
        assert sc.blocks_in_use == int(st.used.sum()) <= st.limit
        peak.append(sc.blocks_in_use)
        sc.complete_iteration(1.0)
        it += 1
    assert len(sc.done) == 120 and not st.used.any()
    assert max(peak[:20]) <= 24 < max(peak[20:60]) <= 40 and st.limit == 24 and max(peak[-5:]) <= 24


def test_compaction_plan_and_relocation():
    st = S.IndexStore(32, 32)
    class Shown:
        capacity = 32
        expansion = 1.0
    sc = S.Scheduler(st, T, Shown(), 8, 8)
    for i, (p, o) in enumerate([(40, 20), (60, 30), (30, 10)]):
        sc.submit(S.Request(i, 0.0, p, o))
    sc.admit(0.0)
    assert [r.handles for r in sc.running] == [[0, 1, 2], [3, 4, 5, 6], [7, 8]]
    st.block_free([1, 2])
    sc.running[0].handles = [0, 20, 21]                              # as if two of its blocks had been given high indices
    st.used[[20, 21]] = True
    sc.running[0].row[:3] = [0, 20, 21]
    assert st.live_end() == 22 and st.plan_compaction(4) is None     # five live blocks below 4 cannot be
    src, dst = st.plan_compaction(12)
    assert (src, dst) == ([20, 21], [1, 2])
    sc.relocate(src, dst)
    assert sc.running[0].handles == [0, 1, 2] and sc.running[0].row[:4].tolist() == [0, 1, 2, -1]
    assert st.live_end() == 9 and int(st.used.sum()) == 9 and sc.blocks_in_use == 9
    table, ctx = sc.tables()
    assert table[0, :3].tolist() == [0, 1, 2] and table[1, :4].tolist() == [3, 4, 5, 6]
