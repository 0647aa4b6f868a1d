"""GPU parity under a changing batch: the scheduler serves a request stream on the library while the
oracle's pool model is driven by the very same decisions (one block store that forwards every call to both
and insists they answer alike).  Every iteration's outputs are checked against the model's float64 attention,
and at the end both pools' bytes must be identical: requests join and leave, contexts cross block boundaries,
new tail blocks land in the host pool when the GPU pool is full (staged append, dirty write-back), and host
blocks move into freed GPU slots between iterations.
"""
import numpy as np
import pytest
import torch

import gpu_helpers as GH
from oracle.pool_model import PoolModel
from paper_2411_09317_amd import binding as B
from paper_2411_09317_amd import inputs as I
from paper_2411_09317_amd import serving as S

pytestmark = pytest.mark.gpu


class Both:
    """A block store that keeps the library pool and the pool model in lockstep."""

    def __init__(self, lib, mod):
        self.lib, self.mod = lib, mod

    def n_free(self, where):
        n = self.lib.n_free(where)
        assert n == self.mod.n_free(where)
        return n

    def block_alloc(self, where, n):
        hs = list(self.lib.block_alloc(where, n))
        assert hs == list(self.mod.block_alloc(where, n))
        return hs

    def block_where(self, hs):
        w = self.lib.block_where(hs)
        assert (list(w[0]), list(w[1])) == tuple(map(list, self.mod.block_where(hs)))
        return w

    def block_free(self, hs):
        self.lib.block_free(hs)
        self.mod.block_free(hs)

    def migrate(self, hs, where, stream=None):
        self.lib.migrate(hs, where, stream)
        self.lib.sync()
        self.mod.migrate(hs, where)


def filled_pools(w, n_gpu, n_host, max_batch, max_blocks):
    lib = B.Pool(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_tokens, w.dtype, n_gpu, n_host, n_host,
                 max_batch=max_batch, max_blocks_per_seq=max_blocks, device=GH.DEV)
    mod = PoolModel(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_tokens, w.dtype, n_gpu, n_host, n_host)
    mod.gpu[:] = I.to_storage(I.draw_values(w, mod.gpu.shape, 20), w.dtype)      # "prompts already in the cache"
    mod.host[:] = I.to_storage(I.draw_values(w, mod.host.shape, 21), w.dtype)
    GH.load_images(lib, mod)
    return lib, mod


@pytest.mark.parametrize("dtype,hq,hkv,d,tol", [(I.DTYPE_F16, 8, 2, 128, 2e-3), (I.DTYPE_BF16, 16, 2, 128, 1e-2),
                                                (I.DTYPE_F32, 4, 4, 64, 1e-5)])
def test_serving_iterations_match_the_model_step_by_step(dtype, hq, hkv, d, tol):
    w = I.Workload("serve", 2, 0, hq, hkv, d, dtype, ctx_lo=10, ctx_hi=150, value_scale=0.5, seed=77)
    n_gpu, unit, k_max, max_batch, max_blocks = 40, 10, 2, 12, 12
    lib, mod = filled_pools(w, n_gpu, unit * k_max, max_batch, max_blocks)
    bud = S.BlockBudget(n_gpu, unit, k_max)
    bud.set_level(2)
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    sched = S.Scheduler(Both(lib, mod), w.block_tokens, bud, max_batch, max_blocks, migrate_stream=streams[1])
    a, p, o = I.draw_requests(w, 40, 1e6, 5, 40)
    for i in range(40):
        sched.submit(S.Request(i, float(a[i]), int(p[i]), int(o[i])))
    it, batches, host_reads, dirty_total, shrunk = 0, set(), 0, 0, False
    while not sched.idle:
        sched.admit(1.0)
        sched.promote()
        assert sched.running
        if it == 25:
            bud.set_level(0)                                          # hide the expansion mid-run
            shrunk = True
        table, ctx = sched.tables()
        nb = len(ctx)
        wi = I.scaled(w, seed=1000 + it)
        q = I.to_storage(I.draw_values(wi, (w.n_layers, nb, hq, d), 1), dtype)
        k_new = I.to_storage(I.draw_values(wi, (w.n_layers, nb, hkv, d), 2), dtype)
        v_new = I.to_storage(I.draw_values(wi, (w.n_layers, nb, hkv, d), 3), dtype)
        pf, dirty = lib.prefetch_list(table, ctx)
        assert pf.tolist() == mod.prefetch_list(table, ctx)
        assert set(pf.tolist()) <= sched.on_host
        out = torch.full((w.n_layers, nb, hq, d), float("nan"), dtype=GH.TORCH_DT[dtype], device=GH.DEV)
        lib.step(GH.to_dev(q, dtype), GH.to_dev(k_new, dtype), GH.to_dev(v_new, dtype), torch.from_numpy(table).to(GH.DEV),
                 torch.from_numpy(ctx).to(GH.DEV), pf, dirty, out, *streams)
        lib.sync()
        ref = mod.step(q, k_new, v_new, table, ctx)
        got = GH.from_dev(out, dtype)
        assert np.isfinite(got).all()
        assert GH.rowwise_rel_err(got, ref) <= tol, it
        batches.add(nb)
        host_reads += len(pf)
        dirty_total += len(dirty)
        sched.complete_iteration(1.0)
        it += 1
        assert it < 2000
    assert lib.check_errors() == 0
    assert len(sched.done) == 40 and shrunk
    assert len(batches) > 3 and host_reads > 0 and dirty_total > 0 and sched.n_promoted > 0
    g, h = GH.images_of(lib)
    mg, mh = GH.model_bytes(mod)
    assert np.array_equal(h, mh) and np.array_equal(g[:, :n_gpu], mg[:, :n_gpu])
    assert lib.n_free(B.GPU) == n_gpu and lib.n_free(B.HOST) == unit * k_max
    lib.close()


def test_serve_runs_a_request_stream_to_completion_with_the_controller():
    """The product loop end to end (random device inputs, measured time, controller in the loop): every
    request ends, every block comes back, no device error flag."""
    w = I.Workload("serve", 4, 0, 8, 2, 128, I.DTYPE_BF16, ctx_lo=64, ctx_hi=600, value_scale=0.5, seed=78)
    n_gpu, unit, k_max, max_batch, max_blocks = 512, 16, 8, 64, 48
    lib = B.Pool(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_tokens, w.dtype, n_gpu, unit * k_max,
                 unit * k_max, max_batch=max_batch, max_blocks_per_seq=max_blocks, device=GH.DEV)
    lib.gpu_image().zero_()
    lib.host_image().zero_()
    a, p, o = I.draw_requests(w, 120, 2000.0, 8, 64)
    reqs = [S.Request(i, float(a[i]), int(p[i]), int(o[i])) for i in range(120)]
    bud = S.BlockBudget(n_gpu, unit, k_max)
    ctl = B.Controller(n_gpu // unit, k_max)
    res = S.serve(lib, w, reqs, bud, max_batch, max_blocks, controller=ctl)
    ctl.close()
    assert res["requests"] == 120 and res["tokens"] == int(o.sum())
    assert res["tokens_per_s"] > 0 and res["mean_batch"] > 1
    assert lib.n_free(B.GPU) == n_gpu and lib.n_free(B.HOST) == unit * k_max
    bud2 = S.BlockBudget(n_gpu, unit, k_max)
    bud2.set_level(4)
    reqs = [S.Request(i, float(a[i]), int(p[i]), int(o[i])) for i in range(120)]
    res2 = S.serve(lib, w, reqs, bud2, max_batch, max_blocks)
    assert res2["requests"] == 120 and res2["expansion"] == 1.125
    lib.close()
