"""Decode attention over a paged KV cache, written out as its definition.

What is computed (paper Section 2.3: attention keys and values live in
non-contiguous fixed-size blocks; Section 3.2: one layer's cache is read per
layer per generated token).  The paper inherits the attention arithmetic from
the serving engine it builds on and does not restate it; the reading taken
here is the textbook one:

    for sequence b, query head h, KV head g = h // (Hq // Hkv):
        s_t  = scale * <q[b,h], K[b,g,t]>          for t < ctx_b
        p    = softmax_t(s)
        out  = sum_t p_t V[b,g,t]

scale defaults to 1/sqrt(head_dim); ctx_b counts the token being decoded; no
mask other than t < ctx_b; no positional term (q and K are taken as already
position-encoded).

Everything here is float64 on the *stored* (already rounded) inputs.
TEST INFRASTRUCTURE ONLY - never imported by the product path.
"""
from __future__ import annotations

import math
from typing import Callable, Sequence

import numpy as np


def softmax_attention_row(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """One query vector against ctx keys/values.  q [d], K [ctx,d], V [ctx,d] (float64)."""
    s = (K @ q) * scale
    s = s - s.max()
    p = np.exp(s)
    p = p / p.sum()
    return p @ V


def dense_attention(q: np.ndarray, K: Sequence[np.ndarray], V: Sequence[np.ndarray],
                    ctx_lens: np.ndarray, scale: float | None = None) -> np.ndarray:
    """Decode attention on de-paged inputs.

    q [B][Hq][d]; K[b], V[b]: [>=ctx_b][Hkv][d]; all float64.  Returns [B][Hq][d].
    """
    B, Hq, d = q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros((B, Hq, d), dtype=np.float64)
    for b in range(B):
        ctx = int(ctx_lens[b])
        Hkv = K[b].shape[1]
        G = Hq // Hkv
        for h in range(Hq):
            g = h // G
            out[b, h] = softmax_attention_row(q[b, h], K[b][:ctx, g, :], V[b][:ctx, g, :], scale)
    return out


def dense_attention_bruteforce(q, K, V, ctx_lens, scale=None):
    """The same quantity with nothing but Python float loops: no numpy
    arithmetic, no tables, no pools.  For tiny inputs only; it exists to pin
    `dense_attention` and `paged_attention_decode`."""
    B = len(q)
    Hq = len(q[0])
    d = len(q[0][0])
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = [[[0.0] * d for _ in range(Hq)] for _ in range(B)]
    for b in range(B):
        ctx = int(ctx_lens[b])
        Hkv = len(K[b][0])
        G = Hq // Hkv
        for h in range(Hq):
            g = h // G
            scores = []
            for t in range(ctx):
                acc = 0.0
                for i in range(d):
                    acc += float(q[b][h][i]) * float(K[b][t][g][i])
                scores.append(acc * scale)
            top = max(scores)
            weights = [math.exp(s - top) for s in scores]
            z = math.fsum(weights)
            for i in range(d):
                out[b][h][i] = math.fsum(weights[t] * float(V[b][t][g][i]) for t in range(ctx)) / z
    return out


def paged_attention_decode(q: np.ndarray, block_table: np.ndarray, ctx_lens: np.ndarray,
                           read_block: Callable[[int], np.ndarray], block_tokens: int,
                           scale: float | None = None) -> np.ndarray:
    """Decode attention through a block table.

    q            float64 [B][Hq][d]
    block_table  int32 [B][max_blocks] of logical block handles (-1 = unused)
    ctx_lens     int32 [B]
    read_block   handle -> float64 array [2][Hkv][T][d] (index 0 = keys, 1 =
                 values) of that logical block, wherever it currently lives
    Returns float64 [B][Hq][d].
    """
    B, Hq, d = q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    T = block_tokens
    out = np.zeros((B, Hq, d), dtype=np.float64)
    for b in range(B):
        ctx = int(ctx_lens[b])
        if ctx <= 0:
            continue
        nb = (ctx + T - 1) // T
        blocks = [read_block(int(block_table[b, j])) for j in range(nb)]
        Hkv = blocks[0].shape[1]
        G = Hq // Hkv
        # [nb*T][Hkv][d], logical token order, truncated to ctx rows
        Kb = np.concatenate([blk[0].transpose(1, 0, 2) for blk in blocks], axis=0)[:ctx]
        Vb = np.concatenate([blk[1].transpose(1, 0, 2) for blk in blocks], axis=0)[:ctx]
        for h in range(Hq):
            g = h // G
            out[b, h] = softmax_attention_row(q[b, h], Kb[:, g, :], Vb[:, g, :], scale)
    return out
