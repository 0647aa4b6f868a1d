"""Shared test plumbing: lay a synthetic decode case out into pool images.

Works against anything exposing block_alloc(where, n) -> handles and
block_where(handles) -> (where[], slot[]): the oracle's PoolModel and the HIP
library's Python binding both do.
"""
import numpy as np

from paper_2411_09317_amd import inputs as I


def plan_allocation(case, order_seed=0, shuffle=True):
    """Order in which the (sequence, block) pairs ask for a block, and in which pool."""
    pairs = [(b, j) for b in range(case.w.batch) for j in range(int(case.n_blocks[b]))]
    if shuffle:
        perm = np.random.Generator(np.random.PCG64([case.w.seed, 77, order_seed])).permutation(len(pairs))
        pairs = [pairs[i] for i in perm]
    return [(b, j, 1 if case.host_mask[b][j] else 0) for (b, j) in pairs]


def allocate(pool, case, plan):
    """Run the plan through an allocator; returns the block table int32[B][max_blocks]."""
    table = np.full((case.w.batch, max(1, case.max_blocks)), -1, dtype=np.int32)
    for (b, j, where) in plan:
        table[b, j] = pool.block_alloc(where, 1)[0]
    return table


def build_images(case, table, where, slot, n_gpu, n_host, upto_ctx=None, fill=None):
    """Pool images holding the case's dense K/V.

    where/slot: dicts handle -> pool / slot.  upto_ctx[b]: number of tokens of
    sequence b to store (default ctx_b).  Slots and token rows not written hold
    `fill` (default zero; pass NaN patterns to poison)."""
    w = case.w
    sd = I.storage_numpy_dtype(w.dtype)
    blk = (2, w.n_kv_heads, w.block_tokens, w.head_dim)
    gpu = np.zeros((w.n_layers, n_gpu) + blk, dtype=sd)
    host = np.zeros((w.n_layers, n_host) + blk, dtype=sd)
    if fill is not None:
        gpu[...] = fill
        host[...] = fill
    T = w.block_tokens
    for b in range(w.batch):
        n_tok = int(case.ctx_lens[b]) if upto_ctx is None else int(upto_ctx[b])
        for j in range(int(case.n_blocks[b])):
            h = int(table[b, j])
            img = gpu if where[h] == 0 else host
            lo, hi = j * T, min((j + 1) * T, n_tok)
            if hi <= lo:
                continue
            # dense [L][ctx][Hkv][d] -> block [L][Hkv][T][d]
            img[:, slot[h], 0, :, : hi - lo, :] = case.k_dense[b][:, lo:hi].transpose(0, 2, 1, 3)
            img[:, slot[h], 1, :, : hi - lo, :] = case.v_dense[b][:, lo:hi].transpose(0, 2, 1, 3)
    return gpu, host


def nan_fill(dtype):
    if dtype == I.DTYPE_BF16:
        return np.uint16(0x7FC0)
    return np.nan


def home_maps(pool, table):
    hs = sorted({int(h) for h in table.ravel() if h >= 0})
    wh, sl = pool.block_where(hs)
    return dict(zip(hs, wh)), dict(zip(hs, sl))


def dense_f64(case, layer):
    """De-paged float64 K, V lists and q for one layer (for the dense oracle)."""
    from oracle import numfmt
    K = [numfmt.to_f64(k[layer], case.w.dtype) for k in case.k_dense]
    V = [numfmt.to_f64(v[layer], case.w.dtype) for v in case.v_dense]
    q = numfmt.to_f64(case.q[layer], case.w.dtype)
    return q, K, V
