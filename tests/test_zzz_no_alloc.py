"""pie_attn_decode_static: the attention call whose scratch lives in the library's static device array.

Through the C ABI, against pie_attn_decode on the same pool and inputs (same kernels: bit for bit) and against
the float64 oracle, on two calls in a row, the second with a smaller input (the array keeps the first call's
contents); a call that needs more than the array holds is refused before anything is enqueued; and the call
works on a pool whose own workspace was sized for nothing.
"""
import numpy as np
import pytest
import torch

import gpu_helpers as GH
import helpers as H
from oracle import attention as A
from paper_2411_09317_amd import binding as B
from paper_2411_09317_amd import inputs as I

pytestmark = pytest.mark.gpu

REL = {I.DTYPE_F16: 2e-3, I.DTYPE_BF16: 1e-2}
ABS = 2e-2


def both_ways(lib, case, table, layer, stream=None):
    w = case.w
    q = GH.to_dev(case.q[layer], w.dtype)
    tb = torch.from_numpy(table).to(GH.DEV)
    cl = torch.from_numpy(case.ctx_lens).to(GH.DEV)
    out_pool, out_static = torch.full_like(q, float("nan")), torch.full_like(q, float("nan"))
    lib.attn_decode(layer, q, tb, cl, out_pool, stream)
    lib.attn_decode_static(layer, q, tb, cl, out_static, stream)
    assert lib.check_errors() == 0
    assert torch.equal(out_pool.view(torch.int16), out_static.view(torch.int16))
    got = GH.from_dev(out_static, w.dtype)
    ref = A.dense_attention(*H.dense_f64(case, layer), case.ctx_lens)
    assert np.isfinite(got).all()
    assert GH.rowwise_rel_err(got, ref) <= REL[w.dtype] and np.abs(got - ref).max() <= ABS
    return out_static


@pytest.mark.parametrize("dtype,hq,hkv", [(I.DTYPE_F16, 8, 8), (I.DTYPE_BF16, 8, 2)])
def test_two_calls_in_a_row_the_second_smaller_match_the_pool_workspace_call_and_the_oracle(dtype, hq, hkv):
    big = I.make_case(I.Workload("static_big", 2, 6, hq, hkv, 128, dtype, ctx_lo=300, ctx_hi=1900, value_scale=0.7, seed=81))
    small = I.make_case(I.Workload("static_small", 2, 2, hq, hkv, 128, dtype, ctx_lo=5, ctx_hi=600, value_scale=0.7, seed=82))
    lib_big, _, table_big = GH.make_pools(big, int(big.n_blocks.sum()) + 3, 2, 2, fill=H.nan_fill(dtype))
    lib_small, _, table_small = GH.make_pools(small, int(small.n_blocks.sum()) + 3, 2, 2, fill=H.nan_fill(dtype))
    try:
        first = both_ways(lib_big, big, table_big, 1)
        both_ways(lib_small, small, table_small, 0)                 # smaller batch, shorter contexts, another pool
        again = both_ways(lib_big, big, table_big, 1)               # and the large one once more
        assert torch.equal(first.view(torch.int16), again.view(torch.int16))
        s = torch.cuda.Stream()
        both_ways(lib_small, small, table_small, 1, s)              # on a stream of the caller's
    finally:
        lib_big.close()
        lib_small.close()


def test_a_call_beyond_the_static_array_is_refused_and_a_pool_without_workspace_still_decodes():
    w = I.Workload("static_tiny", 1, 3, 8, 8, 128, I.DTYPE_F16, ctx_lo=40, ctx_hi=500, value_scale=0.7, seed=83)
    case = I.make_case(w)
    lib, _, table = GH.make_pools(case, int(case.n_blocks.sum()), 2, 2)
    # a pool whose workspace holds one sequence of one block: the pool-workspace call is refused, the static one runs
    n = int(case.n_blocks.sum())
    bare = B.Pool(1, 8, 8, 128, 16, I.DTYPE_F16, n, 0, 0, max_batch=1, max_blocks_per_seq=1, device=GH.DEV)
    try:
        assert bare.block_alloc(B.GPU, n) == list(range(n))      # handle = slot, as in the other pool
        bare.gpu_image()[:, :n].copy_(lib.gpu_image()[:, :n])
        q = GH.to_dev(case.q[0], w.dtype)
        tb = torch.from_numpy(table).to(GH.DEV)
        cl = torch.from_numpy(case.ctx_lens).to(GH.DEV)
        out_ref, out = torch.empty_like(q), torch.full_like(q, float("nan"))
        lib.attn_decode(0, q, tb, cl, out_ref)
        with pytest.raises(B.PieError) as e:
            bare.attn_decode(0, q, tb, cl, out)
        assert e.value.code == B.EINVAL
        bare.attn_decode_static(0, q, tb, cl, out)
        assert bare.check_errors() == 0 and lib.check_errors() == 0
        assert torch.equal(out.view(torch.int16), out_ref.view(torch.int16))
        # 4096 sequences x 4096 blocks of partials is far more than 40 MiB: refused on the host, nothing enqueued
        wide = torch.full((4096, 4096), -1, dtype=torch.int32, device=GH.DEV)
        ctx0 = torch.zeros(4096, dtype=torch.int32, device=GH.DEV)
        qq = torch.zeros(4096, 8, 128, dtype=torch.float16, device=GH.DEV)
        with pytest.raises(B.PieError) as e:
            lib.attn_decode_static(0, qq, wide, ctx0, torch.empty_like(qq))
        assert e.value.code == B.ENOMEM
        with pytest.raises(B.PieError) as e:
            lib.attn_decode_static(0, torch.zeros(4097, 8, 128, dtype=torch.float16, device=GH.DEV),
                                   torch.full((4097, 1), -1, dtype=torch.int32, device=GH.DEV),
                                   torch.zeros(4097, dtype=torch.int32, device=GH.DEV),
                                   torch.empty(4097, 8, 128, dtype=torch.float16, device=GH.DEV))
        assert e.value.code == B.EINVAL
        assert lib.check_errors() == 0
    finally:
        bare.close()
        lib.close()
