"""GPU parity at the benchmark's sizes, in the launch configuration bench.py times.

The full workloads hold tens of GB, so the float64 oracle checks sampled outputs:
for sampled (layer, sequence) pairs the sequence's blocks are read back from the
library's pool, de-paged with the oracle's own statement of the block layout, and
the dense definition is evaluated for all of that sequence's query heads.  On top
of that, properties that hold at any size: every output finite, the swap leg's
outputs bit-identical to the all-resident ones (residency independence), no device
error flags.

The 70B-shaped workload needs more memory than one GPU has; its test keeps the real
per-layer shape (batch 32 x 32768 tokens, 64 / 8 heads) on fewer layers.
"""
import numpy as np
import pytest
import torch

import gpu_helpers as GH
from oracle import attention as A
from oracle import layout as LY
from oracle import numfmt
from paper_2411_09317_amd import binding as B
from paper_2411_09317_amd import inputs as I
from paper_2411_09317_amd import workload as WL

pytestmark = pytest.mark.gpu

REL = {I.DTYPE_F16: 2e-3, I.DTYPE_BF16: 1e-2}
ABS = 2e-2


def oracle_rows(dw, layer, b):
    """float64 oracle output [Hq][d] of sequence b in `layer`, from the bytes the pool holds."""
    w = dw.w
    nb = int(dw.n_blocks[b])
    where, slots = dw.pool.block_where(dw.table[b, :nb])
    sd = I.storage_numpy_dtype(w.dtype)
    raw = []
    for wh, sl in zip(where, slots):
        img = dw.pool.gpu_image() if wh == B.GPU else dw.pool.host_image()
        raw.append(img[layer, sl].cpu().numpy())
    blocks = LY.from_physical(np.stack(raw).view(sd), w.n_kv_heads, w.block_tokens, w.head_dim)   # [nb][2][Hkv][T][d]
    blocks = numfmt.to_f64(blocks, w.dtype)
    ctx = int(dw.ctx_lens[b])
    K = blocks[:, 0].transpose(0, 2, 1, 3).reshape(nb * w.block_tokens, w.n_kv_heads, w.head_dim)[:ctx]
    V = blocks[:, 1].transpose(0, 2, 1, 3).reshape(nb * w.block_tokens, w.n_kv_heads, w.head_dim)[:ctx]
    qd = dw.q[layer, b]
    q = (qd.view(torch.int16).cpu().numpy().view(np.uint16) if w.dtype == I.DTYPE_BF16 else qd.cpu().numpy())
    q = numfmt.to_f64(q, w.dtype)
    return A.dense_attention(q[None], [K], [V], np.array([ctx]))[0]


def expected_partition(dw, new_token=True):
    """The item size the planning kernel is documented to choose: the largest of its candidates that leaves more
    than 17 x (compute units) (partition, kv head) units, the smallest candidate if none does."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    ctx = dw.ctx_lens.astype(np.int64) - (1 if new_token else 0)
    pick = 512
    for p in (768, 1024, 1536, 2048, 3072, 4096):
        units = int(np.maximum(1, -(-ctx // p)).sum()) * dw.w.n_kv_heads
        if units > 17 * cus:
            pick = p
    return pick


def run_steps(dw, pf, dirty, n=1):
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    for _ in range(n):
        dw.pool.step(dw.q, dw.k_new, dw.v_new, dw.d_table, dw.d_ctx, pf, dirty, dw.out, *streams)
    dw.pool.sync()
    assert dw.pool.check_errors() == 0


def check_samples(dw, samples):
    w = dw.w
    got_all = dw.out
    assert bool(torch.isfinite(got_all.float()).all())
    worst = 0.0
    for layer, b in samples:
        ref = oracle_rows(dw, layer, b)
        got = got_all[layer, b].to(torch.float64).cpu().numpy()
        worst = max(worst, GH.rowwise_rel_err(got, ref))
        assert np.abs(got - ref).max() <= ABS
    assert worst <= REL[w.dtype], worst
    return worst


def sample_pairs(dw, n, seed):
    """Seeded (layer, sequence) pairs that always include the shortest and the longest sequence."""
    rng = np.random.Generator(np.random.PCG64([dw.w.seed, 901, seed]))
    pairs = [(int(rng.integers(dw.w.n_layers)), int(np.argmin(dw.ctx_lens))),
             (int(rng.integers(dw.w.n_layers)), int(np.argmax(dw.ctx_lens)))]
    while len(pairs) < n:
        pairs.append((int(rng.integers(dw.w.n_layers)), int(rng.integers(dw.w.batch))))
    return pairs


def fresh_rows(dw, seed):
    """New K / V rows for this step's token (the same distribution as the workload's), in place."""
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(seed)
    for t in (dw.k_new, dw.v_new):
        t.copy_((torch.randn(t.shape, device="cuda:0", dtype=torch.float32, generator=gen) * dw.w.value_scale).to(t.dtype))
    torch.cuda.synchronize()


def rows_np(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16 if t.dtype == torch.bfloat16 else np.float16)


def step_and_check_tail_blocks(dw, pf, dirty, seed, layers, n_each=5):
    """One step with fresh rows.  Afterwards the home image of sampled tail blocks - host-homed ones in the pinned
    pool (they were staged, appended to and written back), GPU-homed ones in the device pool - must be what the
    oracle's layout says: the image before the step with row (ctx - 1) % T of every kv head's K and V replaced
    by the new rows, every other byte unchanged.  Sampled host blocks that are not tails (staged, read, dropped)
    must not have changed at all."""
    w = dw.w
    T = w.block_tokens
    fresh_rows(dw, seed)
    k_new, v_new = rows_np(dw.k_new), rows_np(dw.v_new)
    sd = I.storage_numpy_dtype(w.dtype)
    tail_of = {int(dw.table[b, (int(dw.ctx_lens[b]) - 1) // T]): b for b in range(w.batch)}
    dirty_set = set(int(h) for h in dirty)
    assert dirty_set <= set(tail_of)
    rng = np.random.Generator(np.random.PCG64([w.seed, 902, seed]))
    pick = lambda xs, n: [xs[i] for i in rng.permutation(len(xs))[:n]]
    host_tails = pick(sorted(dirty_set), n_each)
    gpu_tails = pick(sorted(set(tail_of) - dirty_set), n_each)
    clean = pick(sorted(set(int(h) for h in pf) - dirty_set), n_each)
    assert host_tails and gpu_tails and clean
    handles = host_tails + gpu_tails + clean
    where, slots = dw.pool.block_where(handles)
    assert where == [B.HOST] * len(host_tails) + [B.GPU] * len(gpu_tails) + [B.HOST] * len(clean)
    image = lambda wh: dw.pool.host_image() if wh == B.HOST else dw.pool.gpu_image()
    before = {(l, h): image(wh)[l, sl].cpu().numpy().copy() for h, wh, sl in zip(handles, where, slots) for l in layers}
    run_steps(dw, pf, dirty, n=1)
    for h, wh, sl in zip(handles, where, slots):
        for l in layers:
            after = image(wh)[l, sl].cpu().numpy()
            if h not in tail_of:
                assert np.array_equal(after, before[(l, h)]), (l, h)
                continue
            b, t = tail_of[h], (int(dw.ctx_lens[tail_of[h]]) - 1) % T
            logical = LY.from_physical(before[(l, h)].view(sd), w.n_kv_heads, T, w.head_dim).copy()   # [2][Hkv][T][d]
            logical[0, :, t, :] = k_new[l, b]
            logical[1, :, t, :] = v_new[l, b]
            expect = LY.to_physical(logical).view(np.uint8)
            assert np.array_equal(after, expect), (l, h, wh)
            assert not np.array_equal(after, before[(l, h)])          # the row really is new


def test_llama2_7b_shape_all_resident_then_thirty_percent_on_the_host():
    """The benchmark's workload: all resident, then the 30 % leg; sampled outputs against the oracle, and the
    swap leg's outputs bit-identical to the resident ones."""
    none = np.zeros(0, dtype=np.int32)
    dw = WL.build(I.CONFIGS["cfg2"], host_capacity_fraction=0.32)
    try:
        run_steps(dw, none, none, n=2)
        assert dw.pool.attn_partition() == expected_partition(dw)
        samples = sample_pairs(dw, 6, 0)
        check_samples(dw, samples)
        resident = dw.out.clone()
        streams = torch.cuda.Stream()
        hs = WL.per_sequence_host_order(dw, 0.30, I.CONFIGS["cfg3"])
        dw.pool.migrate(hs, B.HOST, streams)
        dw.pool.sync()
        pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
        assert len(pf) == len(hs) and len(dirty) > 0
        dw.out.zero_()
        run_steps(dw, pf, dirty, n=1)
        assert torch.equal(dw.out.view(torch.int16), resident.view(torch.int16))
        check_samples(dw, samples[:3])          # the oracle now reads 30 % of the blocks from the host pool
        st = dw.pool.stats()
        assert abs(st.host_fraction - 0.30) < 0.01
        # the write-back at this size, through the copy engine and through the gather / scatter kernel
        for path, seed in ((B.SWAP_DMA, 11), (B.SWAP_KERNEL, 12), (B.SWAP_AUTO, 13)):
            dw.pool.set_swap_path(path)
            step_and_check_tail_blocks(dw, pf, dirty, seed, layers=(0, 17, 31))
            check_samples(dw, samples[3:5])     # and the attention saw the new rows (the oracle reads the pools' bytes)
    finally:
        dw.pool.close()


def test_llama3_8b_shape_gqa_bf16_all_resident_then_ten_percent_on_the_host():
    """The 8B-shaped workload at full size (bf16, four query heads per kv head, 64 KiB blocks, skewed contexts):
    sampled outputs against the oracle, the leg with a tenth of the blocks on the host bit-identical to the
    resident one, and the write-back checked in the home images on all three swap paths."""
    none = np.zeros(0, dtype=np.int32)
    dw = WL.build(I.CONFIGS["cfg4"], host_capacity_fraction=0.12)
    try:
        run_steps(dw, none, none, n=2)
        assert dw.pool.attn_partition() == expected_partition(dw)
        samples = sample_pairs(dw, 6, 1)
        check_samples(dw, samples)
        resident = dw.out.clone()
        dw.pool.set_host_fraction(0.10, dw.order, torch.cuda.Stream())
        dw.pool.sync()
        pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
        assert len(pf) == round(0.10 * dw.total_blocks) and len(dirty) > 0
        dw.out.zero_()
        run_steps(dw, pf, dirty, n=1)
        assert torch.equal(dw.out.view(torch.int16), resident.view(torch.int16))
        check_samples(dw, samples[:3])
        for path, seed in ((B.SWAP_DMA, 21), (B.SWAP_KERNEL, 22), (B.SWAP_AUTO, 23)):
            dw.pool.set_swap_path(path)
            step_and_check_tail_blocks(dw, pf, dirty, seed, layers=(0, 13, 31))
            check_samples(dw, samples[3:5])
    finally:
        dw.pool.close()


def test_70b_shape_long_context_per_layer_shape_on_four_layers():
    """The 70B shape's real per-layer size (batch 32 x 32768 tokens, 64 / 8 heads) on four layers: sampled outputs
    against the oracle; then the share of the cache that cannot fit one GPU (21.5 %) on the host: outputs
    bit-identical, the oracle reading the host pool, and the write-back in the home images."""
    none = np.zeros(0, dtype=np.int32)
    dw = WL.build(I.CONFIGS["cfg5"], n_layers=4, host_capacity_fraction=0.225)
    try:
        run_steps(dw, none, none, n=1)
        assert dw.pool.attn_partition() == expected_partition(dw) > 512
        check_samples(dw, [(0, 0), (3, 17), (2, 31)])
        resident = dw.out.clone()
        hs = WL.per_sequence_host_order(dw, 0.215)
        dw.pool.migrate(hs, B.HOST, torch.cuda.Stream())
        dw.pool.sync()
        pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
        assert len(pf) == len(hs) and abs(len(hs) / dw.total_blocks - 0.215) < 0.002
        dw.out.zero_()
        run_steps(dw, pf, dirty, n=1)
        assert torch.equal(dw.out.view(torch.int16), resident.view(torch.int16))
        check_samples(dw, [(1, 5), (3, 30)])
        if len(dirty):
            step_and_check_tail_blocks(dw, pf, dirty, 31, layers=(0, 3))
    finally:
        dw.pool.close()
