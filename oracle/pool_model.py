"""Bookkeeping model of the split KV cache: a GPU block pool, a pinned-host block
pool, per-handle residency, two staging regions and the swaps between them.

Follows the paper's mapping table (Section 3.2: logical unit -> CPU pointer,
GPU pointer, updated in two phases around a background copy; presence is
checked before a layer is computed) and block manager (Section 4.1: a free
list, blocks handed out on demand and returned on completion; blocks are
addressed as base pointer + unchanged offset).  The unit of residency here is
a block rather than a whole layer: a logical block is homed either in the GPU
pool or in the host pool, in the same slot of every layer.

The model is synchronous: a swap has completed when the call returns, so the
two-phase states collapse.  It keeps images of both pools, blocks in the logical
order [K|V][head][token][dim]; gpu_bytes / host_bytes give them in the physical
order the C ABI documents (oracle.layout), so that the GPU library's pool
contents can be compared bit for bit.

TEST INFRASTRUCTURE ONLY - never imported by the product path.
"""
from __future__ import annotations

import numpy as np

from . import layout, numfmt
from .attention import paged_attention_decode

EINVAL, ENOMEM, ESTATE = -1, -2, -3
GPU, HOST = 0, 1


class PoolError(Exception):
    def __init__(self, code: int, msg: str = ""):
        super().__init__(f"{code}: {msg}")
        self.code = code


class PoolModel:
    def __init__(self, n_layers, n_q_heads, n_kv_heads, head_dim, block_tokens, dtype,
                 n_gpu_blocks, n_stage_blocks, n_host_blocks, softmax_scale=0.0):
        if min(n_layers, n_q_heads, n_kv_heads, head_dim, block_tokens) <= 0:
            raise PoolError(EINVAL, "non-positive dimension")
        if n_q_heads % n_kv_heads or min(n_gpu_blocks, n_stage_blocks, n_host_blocks) < 0:
            raise PoolError(EINVAL, "bad head counts or pool sizes")
        self.L, self.Hq, self.Hkv, self.d, self.T = n_layers, n_q_heads, n_kv_heads, head_dim, block_tokens
        self.dtype = dtype
        self.n_gpu, self.n_stage, self.n_host = n_gpu_blocks, n_stage_blocks, n_host_blocks
        self.scale = float(softmax_scale) if softmax_scale else 1.0 / np.sqrt(head_dim)
        sd = numfmt.storage_dtype(dtype)
        blk = (2, self.Hkv, self.T, self.d)
        # image of the GPU pool: resident slots first, then staging region 0, then region 1
        self.gpu = np.zeros((self.L, self.n_gpu + 2 * self.n_stage) + blk, dtype=sd)
        self.host = np.zeros((self.L, self.n_host) + blk, dtype=sd)
        self.n_handles = self.n_gpu + self.n_host
        self.free_handles = set(range(self.n_handles))
        self.free_slots = {GPU: set(range(self.n_gpu)), HOST: set(range(self.n_host))}
        self.home = {}                       # handle -> (where, slot)
        self.stage_of = [dict(), dict()]     # region -> {handle: rank}
        self.region_layer = [-1, -1]         # which layer's data a region holds
        self.dirty = [set(), set()]          # staged handles written since they were brought in

    # ---- byte images in the ABI's physical block order ---------------------
    def gpu_bytes(self):
        """uint8 [L][n_gpu + 2 n_stage][block_bytes]."""
        return layout.to_physical(self.gpu).view(np.uint8)

    def host_bytes(self):
        """uint8 [L][n_host][block_bytes]."""
        return layout.to_physical(self.host).view(np.uint8)

    def blocks_from_bytes(self, raw):
        """uint8 [..., block_bytes] in physical order -> storage dtype [..., 2, Hkv, T, d]."""
        return layout.from_physical(np.ascontiguousarray(raw).view(self.gpu.dtype), self.Hkv, self.T, self.d)

    # ---- allocator -------------------------------------------------------
    def block_alloc(self, where, n):
        if where not in (GPU, HOST) or n < 0:
            raise PoolError(EINVAL)
        if n > len(self.free_slots[where]) or n > len(self.free_handles):
            raise PoolError(ENOMEM)
        handles = sorted(self.free_handles)[:n]
        slots = sorted(self.free_slots[where])[:n]
        for h, s in zip(handles, slots):
            self.free_handles.discard(h)
            self.free_slots[where].discard(s)
            self.home[h] = (where, s)
        return handles

    def _check_handles(self, handles, need_where=None):
        seen = set()
        for h in handles:
            h = int(h)
            if h < 0 or h >= self.n_handles:
                raise PoolError(EINVAL, f"handle {h} out of range")
            if h not in self.home or h in seen:
                raise PoolError(ESTATE, f"handle {h} not allocated or repeated")
            if need_where is not None and self.home[h][0] != need_where:
                raise PoolError(ESTATE, f"handle {h} not homed in pool {need_where}")
            seen.add(h)

    def block_free(self, handles):
        self._check_handles(handles)
        for h in handles:
            h = int(h)
            where, slot = self.home.pop(h)
            self.free_slots[where].add(slot)
            self.free_handles.add(h)
            for r in (0, 1):
                self.stage_of[r].pop(h, None)
                self.dirty[r].discard(h)

    def block_where(self, handles):
        where, slot = [], []
        for h in handles:
            h = int(h)
            if h < 0 or h >= self.n_handles:
                raise PoolError(EINVAL)
            w, s = self.home.get(h, (-1, -1))
            where.append(w)
            slot.append(s)
        return where, slot

    def n_free(self, where):
        return len(self.free_slots[where])

    # ---- swaps -------------------------------------------------------------
    def stage_slot(self, region, rank):
        return self.n_gpu + region * self.n_stage + rank

    def swap_in(self, layer, handles):
        """host slot -> staging region (layer & 1); the staging slot of
        handles[i] is i.  Replaces whatever the region held."""
        if layer < 0 or layer >= self.L:
            raise PoolError(EINVAL)
        if len(handles) > self.n_stage:
            raise PoolError(ENOMEM)
        self._check_handles(handles, need_where=HOST)
        r = layer & 1
        self.stage_of[r] = {}
        self.dirty[r] = set()
        self.region_layer[r] = layer
        for i, h in enumerate(handles):
            h = int(h)
            self.stage_of[r][h] = i
            self.gpu[layer, self.stage_slot(r, i)] = self.host[layer, self.home[h][1]]

    def swap_out(self, layer, handles):
        """staged copy of `layer` -> its host slot."""
        if layer < 0 or layer >= self.L:
            raise PoolError(EINVAL)
        self._check_handles(handles, need_where=HOST)
        r = layer & 1
        if self.region_layer[r] != layer and len(handles):
            raise PoolError(ESTATE, "staging region holds another layer")
        for h in handles:
            if int(h) not in self.stage_of[r]:
                raise PoolError(ESTATE, f"handle {h} not staged")
        for h in handles:
            h = int(h)
            self.host[layer, self.home[h][1]] = self.gpu[layer, self.stage_slot(r, self.stage_of[r][h])]
            self.dirty[r].discard(h)

    def migrate(self, handles, to_where):
        """Re-home blocks (all layers) in the other pool; the handle is kept."""
        if to_where not in (GPU, HOST):
            raise PoolError(EINVAL)
        self._check_handles(handles)
        movers = [int(h) for h in handles if self.home[int(h)][0] != to_where]
        if len(movers) > len(self.free_slots[to_where]):
            raise PoolError(ENOMEM)
        src_img, dst_img = (self.gpu, self.host) if to_where == HOST else (self.host, self.gpu)
        for h in movers:
            w, s = self.home[h]
            t = min(self.free_slots[to_where])
            self.free_slots[to_where].discard(t)
            dst_img[:, t] = src_img[:, s]
            self.free_slots[w].add(s)
            self.home[h] = (to_where, t)
            for r in (0, 1):
                self.stage_of[r].pop(h, None)
                self.dirty[r].discard(h)

    def set_host_fraction(self, f, order):
        """Fixed-fraction mode: of the handles in `order`, the first
        round(f * len(order)) are homed on the host, the rest on the GPU."""
        if not (0.0 <= f <= 1.0):
            raise PoolError(EINVAL)
        self._check_handles(order)
        k = int(np.floor(f * len(order) + 0.5))
        to_host, to_gpu = [int(h) for h in order[:k]], [int(h) for h in order[k:]]
        # bring blocks back first so that their GPU slots are known free before demotions
        self.migrate(to_gpu, GPU)
        self.migrate(to_host, HOST)
        return k

    # ---- where a logical block's bytes currently are ------------------------
    def _locate(self, layer, h, for_write=False):
        if h not in self.home:
            raise PoolError(ESTATE, f"handle {h} not allocated")
        w, s = self.home[h]
        if w == GPU:
            return self.gpu, s
        r = layer & 1
        if self.region_layer[r] == layer and h in self.stage_of[r]:
            return self.gpu, self.stage_slot(r, self.stage_of[r][h])
        if for_write:
            raise PoolError(ESTATE, f"host-homed handle {h} written while not staged")
        return self.host, s

    def read_block(self, layer, h):
        img, s = self._locate(layer, int(h))
        return numfmt.to_f64(img[layer, s], self.dtype)

    # ---- the per-layer operations --------------------------------------------
    def kv_append(self, layer, k_new, v_new, block_table, ctx_lens):
        """Write this step's key/value rows [B][Hkv][d] (storage dtype) at token
        position ctx_b - 1 of every sequence."""
        for b in range(len(ctx_lens)):
            ctx = int(ctx_lens[b])
            if ctx <= 0:
                continue
            pos = ctx - 1
            h = int(block_table[b, pos // self.T])
            img, s = self._locate(layer, h, for_write=True)
            img[layer, s, 0, :, pos % self.T, :] = k_new[b]
            img[layer, s, 1, :, pos % self.T, :] = v_new[b]
            if self.home[h][0] == HOST:
                self.dirty[layer & 1].add(h)

    def attn_decode(self, layer, q, block_table, ctx_lens):
        qf = numfmt.to_f64(q, self.dtype)
        return paged_attention_decode(qf, block_table, ctx_lens,
                                      lambda h: self.read_block(layer, h), self.T, self.scale)

    def prefetch_list(self, block_table, ctx_lens):
        """Host-homed handles a batch touches, each once, in ascending order of
        their host slot (so that a densely used host pool is read as one
        contiguous piece and lands, in the same order, in the staging region)."""
        seen = set()
        for b in range(len(ctx_lens)):
            nb = (int(ctx_lens[b]) + self.T - 1) // self.T
            for j in range(nb):
                h = int(block_table[b, j])
                if h in self.home and self.home[h][0] == HOST:
                    seen.add(h)
        return sorted(seen, key=lambda h: self.home[h][1])

    def step(self, q_all, k_new, v_new, block_table, ctx_lens):
        """One decode step over all layers: bring layer l's host-homed blocks
        into staging, append the new token, attend, write dirty blocks back."""
        plist = self.prefetch_list(block_table, ctx_lens)
        outs = []
        for l in range(self.L):
            self.swap_in(l, plist)
            self.kv_append(l, k_new[l], v_new[l], block_table, ctx_lens)
            outs.append(self.attn_decode(l, q_all[l], block_table, ctx_lens))
            dirty = [h for h in plist if h in self.dirty[l & 1]]
            self.swap_out(l, dirty)
        return np.stack(outs)
