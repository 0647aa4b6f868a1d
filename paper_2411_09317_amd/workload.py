"""Builds a full-size synthetic decode workload directly in a library pool.

Lengths, tables and residency come from the seeded host generators in `inputs`;
the bulk K/V fill is drawn on the device (torch generator) because the full
configurations hold tens of GB.  Plumbing only: no arithmetic of the method.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from . import binding as B
from . import inputs as I

TORCH_DT = {I.DTYPE_F32: torch.float32, I.DTYPE_F16: torch.float16, I.DTYPE_BF16: torch.bfloat16}


@dataclass
class DeviceWorkload:
    w: I.Workload
    pool: B.Pool
    ctx_lens: np.ndarray
    n_blocks: np.ndarray
    table: np.ndarray            # int32 [B][max_blocks] handles
    d_table: torch.Tensor
    d_ctx: torch.Tensor
    q: torch.Tensor              # [L][B][Hq][d]
    k_new: torch.Tensor          # [L][B][Hkv][d]
    v_new: torch.Tensor
    out: torch.Tensor
    order: np.ndarray            # handles in demotion order (seeded permutation of all blocks)

    @property
    def kv_bytes_per_layer(self) -> int:
        """Algorithmic bytes one layer's attention must read: every context token's keys and values."""
        return int(self.ctx_lens.astype(np.int64).sum()) * self.w.kv_bytes_per_token_layer

    @property
    def total_blocks(self) -> int:
        return int(self.n_blocks.sum())


def build(w: I.Workload, host_capacity_fraction: float = 0.0, device: str = "cuda:0", spare_blocks: int = 64,
          n_layers: Optional[int] = None) -> DeviceWorkload:
    """All blocks start GPU-resident, placed in a seeded random permutation of the
    pool's slots.  host_capacity_fraction sizes the pinned host pool and the two
    staging regions (as a fraction of the blocks in use)."""
    if n_layers is not None:
        w = I.scaled(w, n_layers=n_layers)
    ctx = I.draw_ctx_lens(w)
    nb = I.blocks_needed(ctx, w.block_tokens)
    total = int(nb.sum())
    max_blocks = int(nb.max())
    n_host = int(np.ceil(total * host_capacity_fraction)) + (8 if host_capacity_fraction > 0 else 0)
    pool = B.Pool(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_tokens, w.dtype, total + spare_blocks,
                  n_host, n_host, max_batch=w.batch, max_blocks_per_seq=max_blocks, device=device)
    # handles are handed out lowest-first, so allocating in a shuffled (sequence, block) order scatters every
    # sequence over the pool
    pairs = np.array([(b, j) for b in range(w.batch) for j in range(int(nb[b]))], dtype=np.int32)
    perm = I.rng_for(w, 3).permutation(len(pairs))
    handles = np.asarray(pool.block_alloc(B.GPU, total), dtype=np.int32)
    table = np.full((w.batch, max_blocks), -1, dtype=np.int32)
    table[pairs[perm, 0], pairs[perm, 1]] = handles
    order_pairs = I.draw_promotion_order(w, nb)
    order = table[order_pairs[:, 0], order_pairs[:, 1]].astype(np.int32)

    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed)
    dt = TORCH_DT[w.dtype]
    img = pool.gpu_image()
    for l in range(w.n_layers):
        layer = img[l].view(-1).view(dt)
        chunk = 1 << 28
        for off in range(0, layer.numel(), chunk):
            n = min(chunk, layer.numel() - off)
            layer[off:off + n] = (torch.randn(n, device=device, dtype=torch.float32, generator=gen) * w.value_scale).to(dt)

    def draw(*shape):
        return (torch.randn(*shape, device=device, dtype=torch.float32, generator=gen) * w.value_scale).to(dt)

    q = draw(w.n_layers, w.batch, w.n_q_heads, w.head_dim)
    k_new = draw(w.n_layers, w.batch, w.n_kv_heads, w.head_dim)
    v_new = draw(w.n_layers, w.batch, w.n_kv_heads, w.head_dim)
    out = torch.zeros_like(q)
    torch.cuda.synchronize()
    return DeviceWorkload(w, pool, ctx, nb, table, torch.from_numpy(table).to(device), torch.from_numpy(ctx).to(device),
                          q, k_new, v_new, out, order)


def per_sequence_host_order(dw: DeviceWorkload, fraction: float, seed_workload: Optional[I.Workload] = None) -> np.ndarray:
    """Handles of round(fraction * blocks) blocks of every sequence, chosen from a
    seed: the 'X % of each sequence's blocks in pinned host memory' residency."""
    w = seed_workload or dw.w
    mask = I.draw_host_mask(I.scaled(w, batch=dw.w.batch), dw.n_blocks, fraction)
    hs = [dw.table[b, j] for b in range(dw.w.batch) for j in np.nonzero(mask[b])[0]]
    return np.asarray(hs, dtype=np.int32)
