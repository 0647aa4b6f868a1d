"""CPU-only checks of the native library: it loads, exports what include/pie.h
declares, and its host logic (allocator, residency, controller) matches the
oracle decision for decision.  No compute calls: there is no GPU here."""
import os
import re

import numpy as np
import pytest

from oracle.controller_sim import AdaptiveExpansion, linear_timing
from oracle.pool_model import PoolError, PoolModel
from paper_2411_09317_amd import binding as B
from paper_2411_09317_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "pie.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pie_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 30
    for n in names:
        assert hasattr(B.lib(), n), n
    assert sorted(B.SYMBOLS) == names
    assert B.lib().pie_version() >= 1
    assert B.lib().pie_strerror(-2).decode().startswith("pool")


def host_pool(n_gpu=40, n_stage=16, n_host=24, **kw):
    args = dict(n_layers=3, n_q_heads=4, n_kv_heads=2, head_dim=64, block_tokens=16, dtype=I.DTYPE_F16)
    args.update(kw)
    return B.Pool(args["n_layers"], args["n_q_heads"], args["n_kv_heads"], args["head_dim"], args["block_tokens"],
                  args["dtype"], n_gpu, n_stage, n_host, max_batch=8, max_blocks_per_seq=64, device=None)


def model_pool(n_gpu=40, n_stage=16, n_host=24):
    return PoolModel(3, 4, 2, 64, 16, I.DTYPE_F16, n_gpu, n_stage, n_host)


def both(call):
    """Run the same call on the library and on the model; both results or both error codes."""
    def run(obj):
        try:
            return ("ok", call(obj))
        except (B.PieError, PoolError) as e:
            return ("err", e.code)
    return run


def test_allocator_and_residency_match_the_model_on_a_random_script():
    lib, mod = host_pool(), model_pool()
    rng = np.random.Generator(np.random.PCG64(9))
    live = []
    for step in range(600):
        r = rng.random()
        if r < 0.40:
            where, n = int(rng.integers(0, 2)), int(rng.integers(0, 6))
            f = both(lambda p: p.block_alloc(where, n))
        elif r < 0.70 and live:
            k = int(rng.integers(1, min(5, len(live)) + 1))
            victims = [int(x) for x in rng.choice(live, size=k, replace=False)]
            if rng.random() < 0.1:
                victims.append(victims[0])                   # repeated handle -> ESTATE, nothing freed
            f = both(lambda p: p.block_free(victims))
        elif r < 0.85 and live:
            k = int(rng.integers(1, min(8, len(live)) + 1))
            movers = [int(x) for x in rng.choice(live, size=k, replace=False)]
            to = int(rng.integers(0, 2))
            f = both(lambda p: p.migrate(movers, to))
        else:
            hs = [int(x) for x in rng.integers(-2, 70, size=4)]
            f = both(lambda p: p.block_where(hs))
        a, b = f(lib), f(mod)
        assert a == b, (step, a, b)
        live = sorted(mod.home)
        assert lib.n_free(0) == mod.n_free(0) and lib.n_free(1) == mod.n_free(1)
        if live:
            assert lib.block_where(live) == mod.block_where(live)
    lib.close()


def test_set_host_fraction_matches_the_model():
    lib, mod = host_pool(n_gpu=60, n_host=60), model_pool(n_gpu=60, n_host=60)
    hs = lib.block_alloc(0, 50)
    assert hs == mod.block_alloc(0, 50)
    order = [int(x) for x in np.random.Generator(np.random.PCG64(3)).permutation(hs)]
    for f in (0.1, 0.3, 0.6, 1.0, 0.3, 0.0, 0.5):
        assert lib.set_host_fraction(f, order) == mod.set_host_fraction(f, order)
        assert lib.block_where(hs) == mod.block_where(hs)
        st = lib.stats()
        assert st.host_blocks_in_use == sum(1 for h in hs if mod.home[h][0] == 1)
        assert st.host_fraction == pytest.approx(st.host_blocks_in_use / 50)
        assert st.expansion_simple == pytest.approx(1 / (1 - st.host_fraction) if st.host_fraction < 1 else np.inf)
    with pytest.raises(B.PieError) as e:
        lib.set_host_fraction(1.5, order)
    assert e.value.code == B.EINVAL
    lib.close()


def test_stats_expansions_follow_the_closed_forms():
    # nine layers' worth: 2 of 9 blocks on the host -> 9/7 (the worked example's 1.28) and, with two staging
    # regions, L / (L (1 - f) + 2 f)
    lib = host_pool(n_gpu=20, n_host=20, n_layers=9)
    lib.block_alloc(0, 7)
    lib.block_alloc(1, 2)
    st = lib.stats()
    assert st.expansion_simple == pytest.approx(9 / 7, rel=1e-6)
    f = 2 / 9
    assert st.expansion_staged == pytest.approx(9 / (9 * (1 - f) + 2 * f), rel=1e-6)
    lib.close()


def test_prefetch_list_matches_the_model():
    w = I.Workload("pf", 3, 5, 4, 2, 64, I.DTYPE_F16, ctx_lo=1, ctx_hi=200, host_fraction=0.4, seed=5)
    case = I.make_case(I.scaled(w, n_layers=1))
    lib, mod = host_pool(n_gpu=80, n_host=80), model_pool(n_gpu=80, n_host=80)
    import helpers as H
    plan = H.plan_allocation(case)
    t1, t2 = H.allocate(lib, case, plan), H.allocate(mod, case, plan)
    assert np.array_equal(t1, t2)
    pf, dirty = lib.prefetch_list(t1, case.ctx_lens)
    assert pf.tolist() == mod.prefetch_list(t2, case.ctx_lens)
    tails = [int(t2[b, (case.ctx_lens[b] - 1) // 16]) for b in range(w.batch)]
    assert dirty.tolist() == [h for h in tails if mod.home[h][0] == 1]
    lib.close()


def test_device_calls_on_a_bookkeeping_pool_are_refused():
    lib = host_pool()
    h = lib.block_alloc(1, 2)
    with pytest.raises(B.PieError) as e:
        lib.swap_in(0, h)
    assert e.value.code == B.ESTATE
    with pytest.raises(B.PieError) as e:
        lib.swap_in(0, lib.block_alloc(0, 1))          # GPU-homed: state error comes first
    assert e.value.code == B.ESTATE
    with pytest.raises(B.PieError) as e:
        lib.swap_in(7, h)
    assert e.value.code == B.EINVAL
    lib.close()


def test_config_validation():
    with pytest.raises(B.PieError) as e:
        B.Pool(1, 3, 2, 64, 16, 0, 4, 4, 4, device=None)        # 3 query heads over 2 KV heads
    assert e.value.code == B.EINVAL
    with pytest.raises(B.PieError) as e:
        B.Pool(1, 4, 2, 64, 16, 7, 4, 4, 4, device=None)        # unknown dtype
    assert e.value.code == B.EINVAL


CASES = [
    dict(units=32, L=8, c=1.0, s=10.0),
    dict(units=32, L=4, c=1.0, s=4.0, slow_from=300, slow_until=None, slow_factor=2.0),
    dict(units=32, L=4, c=1.0, s=4.0, slow_from=300, slow_until=301, slow_factor=2.0),
    dict(units=32, L=4, c=1.0, s=2.0, tput_gain=0.0, probe_period=50),
    dict(units=9, L=9, c=1.0, s=2.0, rho=1.0),
    dict(units=100, L=32, c=0.288, s=7.7),
    dict(units=32, L=4, c=1.0, s=4.0, slow_from=200, slow_until=400, slow_factor=3.0, probe_period=32),
    dict(units=16, L=2, c=1.0, s=0.5, k_up=2, k_down=1),
]


@pytest.mark.parametrize("case", CASES)
def test_controller_matches_the_simulation_step_by_step(case):
    case = dict(case)
    units, L, c, s = case.pop("units"), case.pop("L"), case.pop("c"), case.pop("s")
    tkw = {k: case.pop(k) for k in ("tput_gain", "slow_from", "slow_until", "slow_factor") if k in case}
    timing = linear_timing(L, units, c, s, **tkw)
    sim = AdaptiveExpansion(units=units, k_max=units - 1, **case)
    ctl = B.Controller(units, units - 1, **case)
    for step in range(900):
        assert ctl.level()[0] == sim.k, step
        o = timing(sim.k, step)
        k_lib = ctl.observe(o.t_attn, o.t_in, o.t_stall, o.link_util, o.throughput)
        k_sim = sim.observe(o)
        assert k_lib == k_sim, step
        assert ctl.level()[1] == (sim.ceiling if sim.ceiling is not None else -1)
    ctl.close()


def test_controller_with_noisy_timings_matches_the_simulation():
    rng = np.random.Generator(np.random.PCG64(17))
    sim = AdaptiveExpansion(units=40, k_max=30, probe_period=40)
    ctl = B.Controller(40, 30, probe_period=40)
    L = 6
    for step in range(1500):
        k = sim.k
        t_attn = 1.0 + 0.05 * rng.standard_normal(L)
        t_in = (k / 40) * 5.0 * (1.0 + 0.1 * rng.standard_normal(L)) * (3.0 if 600 <= step < 800 else 1.0)
        t_stall = np.maximum(0.0, t_in - t_attn) * (rng.random(L) < 0.8)
        util = float(min(1.0, t_in.sum() / (t_attn.sum() + t_stall.sum())))
        tput = float((1.0 / (1.0 - k / 40)) / (t_attn.sum() + t_stall.sum()) * (1 + 0.002 * rng.standard_normal()))
        from oracle.controller_sim import Observation
        a = ctl.observe(t_attn, t_in, t_stall, util, tput)
        b = sim.observe(Observation(t_attn.tolist(), t_in.tolist(), t_stall.tolist(), util, tput))
        assert a == b, step
    ctl.close()


def test_controller_argument_checks():
    with pytest.raises(B.PieError):
        B.Controller(0, 0)
    with pytest.raises(B.PieError):
        B.Controller(8, 9)
    with pytest.raises(B.PieError):
        B.Controller(8, 7, k_up=0)
