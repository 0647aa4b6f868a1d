"""GPU parity: pie_attn_decode / pie_kv_append against the float64 oracle.

Tolerances: fp32 row-wise inf-norm relative 1e-5; fp16 / bf16 2e-2 absolute (the
contract) and, because that is loose for these inputs, also row-wise relative
2e-3 (fp16) / 1e-2 (bf16)."""
import numpy as np
import pytest
import torch

import gpu_helpers as GH
import helpers as H
from oracle import attention as A
from paper_2411_09317_amd import binding as B
from paper_2411_09317_amd import inputs as I

pytestmark = pytest.mark.gpu

REL = {I.DTYPE_F32: 1e-5, I.DTYPE_F16: 2e-3, I.DTYPE_BF16: 1e-2}
ABS = {I.DTYPE_F32: 1e-5, I.DTYPE_F16: 2e-2, I.DTYPE_BF16: 2e-2}


def run_attn(lib, case, table, layer=0):
    w = case.w
    q = GH.to_dev(case.q[layer], w.dtype)
    out = torch.full_like(q, float("nan"))
    tb = torch.from_numpy(table).to(GH.DEV)
    cl = torch.from_numpy(case.ctx_lens).to(GH.DEV)
    lib.attn_decode(layer, q, tb, cl, out)
    assert lib.check_errors() == 0
    return GH.from_dev(out, w.dtype)


def check(got, ref, dtype):
    assert np.isfinite(got).all()
    assert GH.rowwise_rel_err(got, ref) <= REL[dtype]
    assert np.abs(got - ref).max() <= ABS[dtype]


def test_cfg1_all_resident_fp32():
    w = I.scaled(I.CONFIGS["cfg1"], host_fraction=0.0)
    case = I.make_case(w)
    lib, mod, table = GH.make_pools(case, 512, 8, 8)
    got = run_attn(lib, case, table)
    q, K, V = H.dense_f64(case, 0)
    check(got, A.dense_attention(q, K, V, case.ctx_lens), w.dtype)
    check(got, mod.attn_decode(0, case.q[0], table, case.ctx_lens), w.dtype)
    lib.close()


SHAPES = [
    # name, dtype, Hq, Hkv, d, batch, ctx range, partition
    ("mha_f16_d128", I.DTYPE_F16, 8, 8, 128, 5, (1, 700), 256),
    ("mha_bf16_d128", I.DTYPE_BF16, 4, 4, 128, 4, (300, 1400), 512),
    ("gqa4_bf16_d128", I.DTYPE_BF16, 8, 2, 128, 3, (17, 900), 256),
    ("gqa8_bf16_d128", I.DTYPE_BF16, 16, 2, 128, 3, (1, 1100), 512),
    ("gqa2_f16_d64", I.DTYPE_F16, 4, 2, 64, 4, (1, 600), 256),
    ("gqa16_f16_d128", I.DTYPE_F16, 16, 1, 128, 2, (33, 1500), 512),
    ("gqa3_bf16_d64", I.DTYPE_BF16, 6, 2, 64, 3, (2, 777), 256),
    ("mha_bf16_d64", I.DTYPE_BF16, 3, 3, 64, 4, (15, 300), 256),
    ("mha_f32_d128", I.DTYPE_F32, 4, 4, 128, 3, (5, 530), 256),
    ("gqa4_f32_d64", I.DTYPE_F32, 8, 2, 64, 3, (60, 800), 512),
]


@pytest.mark.parametrize("name,dtype,hq,hkv,d,batch,ctx,part", SHAPES, ids=[s[0] for s in SHAPES])
def test_shapes_dtypes_and_splits(name, dtype, hq, hkv, d, batch, ctx, part):
    """Several tiles, several partitions, ragged tails, poisoned unused rows and slots."""
    w = I.Workload(name, 2, batch, hq, hkv, d, dtype, ctx_lo=ctx[0], ctx_hi=ctx[1], value_scale=1.0, seed=31)
    case = I.make_case(w)
    case.ctx_lens[0] = ctx[0]
    case = _recase(case)
    n = int(case.n_blocks.sum())
    lib, mod, table = GH.make_pools(case, n + 7, 4, 4, fill=H.nan_fill(dtype))
    lib.set_attn_partition(part)
    for layer in (0, 1):
        got = run_attn(lib, case, table, layer)
        q, K, V = H.dense_f64(case, layer)
        check(got, A.dense_attention(q, K, V, case.ctx_lens), dtype)
    lib.close()


def _recase(case):
    """Re-derive block counts / masks after ctx_lens was edited (dense K/V are simply truncated by ctx)."""
    w = case.w
    case.n_blocks = I.blocks_needed(case.ctx_lens, w.block_tokens)
    case.host_mask = [np.zeros(int(nb), dtype=bool) for nb in case.n_blocks]
    for b in range(w.batch):
        need = int(case.ctx_lens[b])
        if case.k_dense[b].shape[1] < need:
            raise AssertionError("ctx grew beyond the drawn data")
    return case


def test_partition_size_does_not_change_the_result_beyond_rounding():
    w = I.Workload("parts", 1, 3, 8, 8, 128, I.DTYPE_F16, ctx_lo=900, ctx_hi=2048, value_scale=0.5, seed=33)
    case = I.make_case(w)
    lib, mod, table = GH.make_pools(case, int(case.n_blocks.sum()), 4, 4)
    ref = A.dense_attention(*H.dense_f64(case, 0), case.ctx_lens)
    outs = []
    for part in (256, 512, 1000, 4096, 0):
        lib.set_attn_partition(part)
        outs.append(run_attn(lib, case, table))
        check(outs[-1], ref, w.dtype)
        # what the kernels used: the size set, rounded up to a multiple of 64; left to the library (0), a batch
        # this small gets the smallest of the sizes it chooses from
        assert lib.attn_partition() == {256: 256, 512: 512, 1000: 1024, 4096: 4096, 0: 512}[part]
    lib.close()


def test_ctx_one_is_bit_exact_and_ctx_zero_gives_zeros():
    w = I.Workload("one", 1, 4, 8, 2, 128, I.DTYPE_BF16, ctx_lo=1, ctx_hi=1, value_scale=1.0, seed=35)
    case = I.make_case(w)
    lib, mod, table = GH.make_pools(case, 8, 2, 2, fill=H.nan_fill(w.dtype))
    got = run_attn(lib, case, table)
    from oracle import numfmt
    G = w.n_q_heads // w.n_kv_heads
    for b in range(w.batch):
        v0 = numfmt.to_f64(case.v_dense[b][0, 0], w.dtype)
        for h in range(w.n_q_heads):
            assert np.array_equal(got[b, h], v0[h // G])
    case.ctx_lens[1] = 0
    got = run_attn(lib, case, table)
    assert (got[1] == 0).all() and np.isfinite(got).all()
    lib.close()


def test_peaked_softmax_and_constant_values():
    w = I.Workload("peak", 1, 3, 4, 4, 128, I.DTYPE_F16, ctx_lo=200, ctx_hi=900, value_scale=1.0, seed=37)
    case = I.make_case(w)
    target = 123
    for b in range(w.batch):
        for g in range(w.n_kv_heads):
            qv = case.q[0, b, g].astype(np.float64)
            case.k_dense[b][0, target, g] = (40.0 * qv / np.linalg.norm(qv)).astype(np.float16)
    lib, mod, table = GH.make_pools(case, int(case.n_blocks.sum()), 2, 2)
    got = run_attn(lib, case, table)
    ref = A.dense_attention(*H.dense_f64(case, 0), case.ctx_lens)
    check(got, ref, w.dtype)
    for b in range(w.batch):       # the oracle itself says the peak dominates: output ~ that token's value row
        assert np.abs(ref[b] - case.v_dense[b][0, target].astype(np.float64)).max() < 1e-2
        assert np.abs(got[b] - case.v_dense[b][0, target].astype(np.float64)).max() < 2e-2
    lib.close()
    # constant V
    case2 = I.make_case(w)
    for b in range(w.batch):
        case2.v_dense[b][:] = np.float16(0.375)
    lib, mod, table = GH.make_pools(case2, int(case2.n_blocks.sum()), 2, 2)
    got = run_attn(lib, case2, table)
    assert np.abs(got - 0.375).max() < 1e-3
    lib.close()


def test_physical_placement_does_not_matter_bit_exact():
    w = I.Workload("perm", 1, 3, 4, 4, 128, I.DTYPE_F16, ctx_lo=100, ctx_hi=700, value_scale=0.5, seed=39)
    case = I.make_case(w)
    outs = []
    for seed in (0, 1, 2):
        lib, mod, table = GH.make_pools(case, int(case.n_blocks.sum()) + 11 * seed, 2, 2, order_seed=seed)
        outs.append(run_attn(lib, case, table))
        lib.close()
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_softmax_scale_argument():
    w = I.Workload("scale", 1, 2, 4, 4, 64, I.DTYPE_F32, ctx_lo=50, ctx_hi=300, value_scale=1.0, seed=41)
    case = I.make_case(w)
    lib, mod, table = GH.make_pools(case, int(case.n_blocks.sum()), 2, 2, scale=0.3)
    got = run_attn(lib, case, table)
    check(got, A.dense_attention(*H.dense_f64(case, 0), case.ctx_lens, scale=0.3), w.dtype)
    lib.close()


def test_kv_append_is_bit_exact_and_then_attention_sees_the_token():
    w = I.Workload("append", 2, 6, 8, 2, 128, I.DTYPE_BF16, ctx_lo=17, ctx_hi=300, value_scale=1.0, seed=43)
    case = I.make_case(w)
    case.ctx_lens[0], case.ctx_lens[1], case.ctx_lens[2] = 1, 16, 17        # first row, last row, first row of block 2
    case = _recase(case)
    lib, mod, table = GH.make_pools(case, int(case.n_blocks.sum()), 2, 2, upto_ctx=case.ctx_lens - 1)
    tb = torch.from_numpy(table).to(GH.DEV)
    cl = torch.from_numpy(case.ctx_lens).to(GH.DEV)
    for layer in range(w.n_layers):
        k_new = np.stack([case.k_dense[b][layer, case.ctx_lens[b] - 1] for b in range(w.batch)])
        v_new = np.stack([case.v_dense[b][layer, case.ctx_lens[b] - 1] for b in range(w.batch)])
        lib.kv_append(layer, GH.to_dev(k_new, w.dtype), GH.to_dev(v_new, w.dtype), tb, cl)
        mod.kv_append(layer, k_new, v_new, table, case.ctx_lens)
    g, _ = GH.images_of(lib)
    mg, _ = GH.model_bytes(mod)
    assert np.array_equal(g, mg)
    for layer in range(w.n_layers):
        got = run_attn(lib, case, table, layer)
        check(got, A.dense_attention(*H.dense_f64(case, layer), case.ctx_lens), w.dtype)
    lib.close()


def test_bad_tables_are_flagged_not_dereferenced():
    w = I.Workload("bad", 1, 2, 4, 4, 128, I.DTYPE_F16, ctx_lo=40, ctx_hi=80, value_scale=1.0, seed=45)
    case = I.make_case(w)
    lib, mod, table = GH.make_pools(case, 16, 2, 2)
    q = GH.to_dev(case.q[0], w.dtype)
    out = torch.empty_like(q)
    cl = torch.from_numpy(case.ctx_lens).to(GH.DEV)
    bad = table.copy()
    bad[0, 1] = 10 ** 6                               # outside the handle range
    lib.attn_decode(0, q, torch.from_numpy(bad).to(GH.DEV), cl, out)
    assert lib.check_errors() & B.DEVERR_BAD_HANDLE
    bad = table.copy()
    free_handle = max(int(table.max()) + 1, 0)
    bad[1, 0] = free_handle                           # a handle that is not allocated: no slot
    lib.attn_decode(0, q, torch.from_numpy(bad).to(GH.DEV), cl, out)
    assert lib.check_errors() & B.DEVERR_NOT_PRESENT
    assert lib.check_errors() == 0
    assert torch.isfinite(out.float()).all()
    lib.close()


def test_argument_checks():
    w = I.Workload("args", 1, 2, 4, 4, 128, I.DTYPE_F16, ctx_lo=40, ctx_hi=80, seed=47)
    case = I.make_case(w)
    lib, mod, table = GH.make_pools(case, 16, 2, 2)
    q = GH.to_dev(case.q[0], w.dtype)
    out = torch.empty_like(q)
    tb = torch.from_numpy(table).to(GH.DEV)
    cl = torch.from_numpy(case.ctx_lens).to(GH.DEV)
    with pytest.raises(B.PieError) as e:
        lib.attn_decode(3, q, tb, cl, out)
    assert e.value.code == B.EINVAL
    wide = torch.full((2, 4096), -1, dtype=torch.int32, device=GH.DEV)
    with pytest.raises(B.PieError) as e:
        lib.attn_decode(0, q, wide, cl, out)          # wider than max_blocks_per_seq
    assert e.value.code == B.EINVAL
    lib.close()
    with pytest.raises(B.PieError) as e:
        B.Pool(1, 4, 4, 96, 16, I.DTYPE_F16, 4, 2, 2, device=GH.DEV)     # unsupported head_dim
    assert e.value.code == B.EINVAL


def test_batch_at_the_planning_limit_and_contexts_on_partition_edges():
    """4096 sequences (the most the planning kernel lists), contexts that sit exactly on, one under and one over
    block and partition boundaries."""
    w = I.Workload("wide", 1, 4096, 2, 1, 64, I.DTYPE_F16, ctx_lo=1, ctx_hi=40, value_scale=1.0, seed=37)
    case = I.make_case(w)
    edges = [1, 15, 16, 17, 31, 32, 33, 40]
    for b in range(w.batch):
        case.ctx_lens[b] = min(edges[b % len(edges)], case.k_dense[b].shape[1])
    case = _recase(case)
    lib, mod, table = GH.make_pools(case, int(case.n_blocks.sum()) + 3, 2, 2, fill=H.nan_fill(w.dtype))
    got = run_attn(lib, case, table)
    check(got, A.dense_attention(*H.dense_f64(case, 0), case.ctx_lens), w.dtype)
    lib.close()
    w = I.Workload("edges", 1, 9, 4, 2, 128, I.DTYPE_BF16, ctx_lo=1100, ctx_hi=1100, value_scale=0.5, seed=38)
    case = I.make_case(w)
    for b, c in enumerate([255, 256, 257, 511, 512, 513, 1023, 1024, 1025]):
        case.ctx_lens[b] = c
    case = _recase(case)
    lib, mod, table = GH.make_pools(case, int(case.n_blocks.sum()), 2, 2, fill=H.nan_fill(w.dtype))
    for part in (256, 512):
        lib.set_attn_partition(part)
        check(run_attn(lib, case, table), A.dense_attention(*H.dense_f64(case, 0), case.ctx_lens), w.dtype)
    lib.close()


def test_stream_probe_runs_on_the_same_plan_and_leaves_no_trace():
    w = I.Workload("probe", 2, 4, 8, 2, 128, I.DTYPE_BF16, ctx_lo=100, ctx_hi=900, value_scale=0.5, seed=39)
    case = I.make_case(w)
    lib, mod, table = GH.make_pools(case, int(case.n_blocks.sum()), 2, 2, fill=H.nan_fill(w.dtype))
    before = run_attn(lib, case, table, 1)
    tb = torch.from_numpy(table).to(GH.DEV)
    cl = torch.from_numpy(case.ctx_lens).to(GH.DEV)
    ms = lib.attn_stream_probe(1, tb, cl)
    assert ms > 0.0 and lib.check_errors() == 0
    assert np.array_equal(run_attn(lib, case, table, 1), before)
    lib.close()


@pytest.mark.parametrize("dtype,d", [(I.DTYPE_F16, 128), (I.DTYPE_BF16, 128), (I.DTYPE_F16, 64), (I.DTYPE_BF16, 64)])
def test_mha_on_the_vector_alu_matches_the_oracle_and_the_matrix_core_kernel(dtype, d):
    """pie_set_attn_vector_alu: the same attention with both products as two-element dot products on the vector
    ALU.  Several partitions, ragged tails, poisoned unused rows and slots, a context of one token and an empty one;
    refused for grouped queries and fp32."""
    w = I.Workload("valu", 2, 6, 4, 4, d, dtype, ctx_lo=1, ctx_hi=1300, value_scale=1.0, seed=37)
    case = I.make_case(w)
    case.ctx_lens[0], case.ctx_lens[1] = 1, min(529, int(case.ctx_lens[1]))
    case = _recase(case)
    n = int(case.n_blocks.sum())
    lib, mod, table = GH.make_pools(case, n + 5, 4, 4, fill=H.nan_fill(dtype))
    lib.set_attn_partition(256)
    for layer in (0, 1):
        lib.set_attn_vector_alu(False)
        on_matrix_cores = run_attn(lib, case, table, layer)
        lib.set_attn_vector_alu(True)
        got = run_attn(lib, case, table, layer)
        ref = A.dense_attention(*H.dense_f64(case, layer), case.ctx_lens)
        check(got, ref, dtype)
        check(on_matrix_cores, ref, dtype)
        assert GH.rowwise_rel_err(got, on_matrix_cores) <= REL[dtype]             # and with each other
    from oracle import numfmt
    assert np.array_equal(got[0], numfmt.to_f64(case.v_dense[0][1, 0], dtype))    # one token: exactly its value row
    case.ctx_lens[2] = 0
    got = run_attn(lib, case, table, 1)
    assert (got[2] == 0).all() and np.isfinite(got).all()
    lib.close()
    gqa = B.Pool(1, 8, 2, 128, 16, I.DTYPE_F16, 4, 0, 0, device=GH.DEV)
    f32 = B.Pool(1, 4, 4, 64, 16, I.DTYPE_F32, 4, 0, 0, device=GH.DEV)
    for pool in (gqa, f32):
        with pytest.raises(B.PieError) as e:
            pool.set_attn_vector_alu(True)
        assert e.value.code == B.ESTATE
        pool.close()
