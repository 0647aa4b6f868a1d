"""Pins for oracle/attention.py and the attention side of oracle/pool_model.py.

None of these re-types the oracle's formula with the same library calls: they
are a loop-only brute force, closed forms, invariances and a library routine.
"""
import math

import numpy as np
import pytest
import torch

import helpers as H
from oracle import attention as A
from oracle import numfmt
from oracle.pool_model import PoolModel
from paper_2411_09317_amd import inputs as I

TINY = I.Workload("tiny", 2, 3, 4, 2, 8, I.DTYPE_F32, block_tokens=4, ctx_dist="uniform", ctx_lo=1, ctx_hi=19,
                  value_scale=1.0, host_fraction=0.4, seed=11)


def model_for(case, n_gpu=64, n_stage=32, n_host=64, order_seed=0, fill=None, scale=0.0):
    w = case.w
    m = PoolModel(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_tokens, w.dtype, n_gpu, n_stage, n_host,
                  softmax_scale=scale)
    table = H.allocate(m, case, H.plan_allocation(case, order_seed))
    where, slot = H.home_maps(m, table)
    g, h = H.build_images(case, table, where, slot, n_gpu, n_host, fill=fill)
    m.gpu[:, :n_gpu] = g
    m.host[:] = h
    if fill is not None:
        m.gpu[:, n_gpu:] = fill
    return m, table


def paged_out(case, layer=0, **kw):
    m, table = model_for(case, **kw)
    return m.attn_decode(layer, case.q[layer], table, case.ctx_lens)


def test_paged_vs_bruteforce_loops_tiny():
    case = I.make_case(TINY)
    for layer in range(TINY.n_layers):
        q, K, V = H.dense_f64(case, layer)
        brute = np.array(A.dense_attention_bruteforce(q.tolist(), [k.tolist() for k in K], [v.tolist() for v in V],
                                                      case.ctx_lens))
        np.testing.assert_allclose(paged_out(case, layer), brute, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(A.dense_attention(q, K, V, case.ctx_lens), brute, rtol=1e-12, atol=1e-14)


def test_cfg1_paged_vs_dense_and_library():
    w = I.CONFIGS["cfg1"]
    case = I.make_case(w)
    q, K, V = H.dense_f64(case, 0)
    out = paged_out(case, 0, n_gpu=512, n_stage=64, n_host=64)
    np.testing.assert_allclose(out, A.dense_attention(q, K, V, case.ctx_lens), rtol=1e-12, atol=1e-14)
    # library routine on de-paged inputs, one sequence at a time
    for b in range(w.batch):
        ctx = int(case.ctx_lens[b])
        tq = torch.from_numpy(q[b]).unsqueeze(1)                         # [H][1][d]
        tk = torch.from_numpy(K[b][:ctx]).permute(1, 0, 2)               # [H][ctx][d]
        tv = torch.from_numpy(V[b][:ctx]).permute(1, 0, 2)
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).squeeze(1).numpy()
        np.testing.assert_allclose(out[b], ref, rtol=1e-10, atol=1e-12)


def test_ctx_one_returns_first_value_exactly():
    w = I.scaled(TINY, ctx_lo=1, ctx_hi=1, host_fraction=0.0)
    case = I.make_case(w)
    out = paged_out(case)
    G = w.n_q_heads // w.n_kv_heads
    for b in range(w.batch):
        for h in range(w.n_q_heads):
            assert np.array_equal(out[b, h], case.v_dense[b][0, 0, h // G].astype(np.float64))


def test_constant_values_are_returned():
    case = I.make_case(TINY)
    for b in range(TINY.batch):
        case.v_dense[b][:] = np.float32(0.375)
    np.testing.assert_allclose(paged_out(case), 0.375, rtol=1e-14)


def test_equal_keys_give_the_mean_value():
    case = I.make_case(TINY)
    for b in range(TINY.batch):
        case.k_dense[b][:] = case.k_dense[b][:, :1]
    out = paged_out(case)
    G = TINY.n_q_heads // TINY.n_kv_heads
    for b in range(TINY.batch):
        mean = case.v_dense[b][0, : case.ctx_lens[b]].astype(np.float64).mean(axis=0)   # [Hkv][d]
        for h in range(TINY.n_q_heads):
            np.testing.assert_allclose(out[b, h], mean[h // G], rtol=1e-12, atol=1e-14)


def test_peaked_softmax_selects_one_row():
    w = I.scaled(TINY, n_q_heads=2, n_kv_heads=2, ctx_lo=9, ctx_hi=19)
    case = I.make_case(w)
    target = 5
    for b in range(w.batch):
        for g in range(w.n_kv_heads):
            qv = case.q[0, b, g].astype(np.float64)
            case.k_dense[b][0, target, g] = (200.0 * qv / np.linalg.norm(qv)).astype(np.float32)
    out = paged_out(case)
    for b in range(w.batch):
        np.testing.assert_allclose(out[b], case.v_dense[b][0, target].astype(np.float64), rtol=0, atol=1e-9)


def test_key_shift_invariance():
    case = I.make_case(TINY)
    base = paged_out(case)
    c = np.linspace(-1, 1, TINY.head_dim, dtype=np.float32) * 0.5          # exactly representable steps are not needed:
    for b in range(TINY.batch):                                            # compare against the shifted dense oracle too
        case.k_dense[b][:] = case.k_dense[b] + c
    shifted = paged_out(case)
    np.testing.assert_allclose(shifted, base, rtol=1e-5, atol=1e-6)        # fp32 rounding of K + c only
    # and exactly (to float64 rounding) on the de-paged float64 inputs, where the shift is not re-rounded
    case = I.make_case(TINY)
    q, K, V = H.dense_f64(case, 0)
    K2 = [k + np.linspace(-3, 3, TINY.head_dim) for k in K]
    np.testing.assert_allclose(A.dense_attention(q, K2, V, case.ctx_lens), A.dense_attention(q, K, V, case.ctx_lens),
                               rtol=1e-11, atol=1e-13)


def test_gqa_equals_mha_with_repeated_heads():
    case = I.make_case(TINY)
    out = paged_out(case)
    G = TINY.n_q_heads // TINY.n_kv_heads
    w2 = I.scaled(TINY, n_kv_heads=TINY.n_q_heads)
    case2 = I.make_case(w2)
    case2.q = case.q
    case2.ctx_lens, case2.n_blocks, case2.host_mask = case.ctx_lens, case.n_blocks, case.host_mask
    case2.k_dense = [np.repeat(k, G, axis=2) for k in case.k_dense]
    case2.v_dense = [np.repeat(v, G, axis=2) for v in case.v_dense]
    np.testing.assert_array_equal(paged_out(case2), out)


def test_independent_of_physical_placement_and_residency():
    case = I.make_case(TINY)
    base = paged_out(case, order_seed=0)
    np.testing.assert_array_equal(paged_out(case, order_seed=5), base)
    for f in (0.0, 1.0):
        c2 = I.make_case(TINY, host_fraction=f)
        np.testing.assert_array_equal(paged_out(c2, order_seed=3), base)


def test_poisoned_unused_slots_do_not_leak():
    case = I.make_case(TINY)
    base = paged_out(case)
    poisoned = paged_out(case, fill=np.nan)
    assert np.isfinite(poisoned).all()
    np.testing.assert_array_equal(poisoned, base)


def test_scale_argument_and_default():
    case = I.make_case(TINY)
    q, K, V = H.dense_f64(case, 0)
    d = TINY.head_dim
    np.testing.assert_array_equal(paged_out(case, scale=0.0), paged_out(case, scale=1.0 / math.sqrt(d)))
    out2 = paged_out(case, scale=0.25)
    np.testing.assert_allclose(out2, A.dense_attention(q, K, V, case.ctx_lens, scale=0.25), rtol=1e-12, atol=1e-14)
    assert not np.allclose(out2, paged_out(case))


@pytest.mark.parametrize("dtype", [I.DTYPE_F16, I.DTYPE_BF16])
def test_storage_decoding_16bit(dtype):
    # decoding pins: values exactly representable in both 16-bit formats survive a round trip through storage
    vals = np.array([0.0, 1.0, -2.0, 0.5, 0.15625, -3.5, 96.0], dtype=np.float32)
    st = I.to_storage(vals, dtype)
    np.testing.assert_array_equal(numfmt.to_f64(st, dtype), vals.astype(np.float64))
    if dtype == I.DTYPE_BF16:
        # 1 + 2^-8 is a tie between two bfloat16 neighbours: nearest-even keeps 1.0; 1 + 3*2^-8 rounds up to 1 + 2^-6
        x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], dtype=np.float32)
        np.testing.assert_array_equal(numfmt.to_f64(I.to_storage(x, dtype), dtype), [1.0, 1.0 + 2.0 ** -6])
    w = I.scaled(TINY, dtype=dtype)
    case = I.make_case(w)
    q, K, V = H.dense_f64(case, 0)
    np.testing.assert_allclose(paged_out(case), A.dense_attention(q, K, V, case.ctx_lens), rtol=1e-12, atol=1e-14)
