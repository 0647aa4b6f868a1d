"""Physical order of the elements inside one KV block, as the C ABI documents it.

The paper leaves the layout of a block open (its Section 2.3 only says that the
KV cache is kept in non-contiguous pages); the library fixes one, and this
module states it a second time, independently, so that pool images can be
compared byte for byte:

  block  = K tile of kv head 0, ..., K tile of head Hkv-1, V tile of head 0, ...
  v      = 16 / elem_bytes            (elements in a 16-byte vector)
  K tile : element (token t, dim c) sits at   (c // v) * (T * v) + t * v + c % v
  V tile : with w = v // 4,
           element (t, c) sits at   (((c // (16 w)) * (T // 4) + t // 4) * 16 + c % 16) * v
                                     + ((c // 16) % w) * 4 + t % 4

The oracle's pool model keeps blocks in the logical order [K|V][head][token][dim];
to_physical / from_physical convert whole images.

TEST INFRASTRUCTURE ONLY - never imported by the product path.
"""
from __future__ import annotations

from functools import lru_cache

import numpy as np


@lru_cache(maxsize=32)
def element_index(n_kv_heads: int, block_tokens: int, head_dim: int, elem_bytes: int) -> np.ndarray:
    """int64 [2][Hkv][T][d]: position (in elements) of each logical element inside the physical block."""
    T, d = block_tokens, head_dim
    v = 16 // elem_bytes
    w = v // 4
    if v * elem_bytes != 16 or w < 1 or T % 4 or d % (16 * w) or d % v:
        raise ValueError("layout undefined for these sizes")
    t = np.arange(T, dtype=np.int64)[:, None]
    c = np.arange(d, dtype=np.int64)[None, :]
    k_tile = (c // v) * (T * v) + t * v + c % v
    v_tile = (((c // (16 * w)) * (T // 4) + t // 4) * 16 + c % 16) * v + ((c // 16) % w) * 4 + t % 4
    tile = T * d
    idx = np.empty((2, n_kv_heads, T, d), dtype=np.int64)
    for g in range(n_kv_heads):
        idx[0, g] = g * tile + k_tile
        idx[1, g] = (n_kv_heads + g) * tile + v_tile
    return idx


def to_physical(logical: np.ndarray) -> np.ndarray:
    """[..., 2, Hkv, T, d] in logical order -> [..., 2*Hkv*T*d] in the block's physical order."""
    two, hkv, T, d = logical.shape[-4:]
    assert two == 2
    idx = element_index(hkv, T, d, logical.dtype.itemsize).ravel()
    inverse = np.empty_like(idx)
    inverse[idx] = np.arange(idx.size)
    flat = logical.reshape(logical.shape[:-4] + (-1,))
    return np.take(flat, inverse, axis=-1)          # out[..., idx[i]] = flat[..., i]


def from_physical(physical: np.ndarray, n_kv_heads: int, block_tokens: int, head_dim: int) -> np.ndarray:
    """Inverse of to_physical."""
    idx = element_index(n_kv_heads, block_tokens, head_dim, physical.dtype.itemsize).ravel()
    return np.take(physical, idx, axis=-1).reshape(physical.shape[:-1] + (2, n_kv_heads, block_tokens, head_dim))
