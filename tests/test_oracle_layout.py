"""Pins of the oracle's statement of the block layout (no GPU).

The layout is a convention, so what can be pinned is that it is a bijection, that it
has the properties the C header promises (which elements share a 16-byte vector, which
vectors are adjacent), and a handful of positions worked out by hand from the text.
"""
import numpy as np
import pytest

from oracle import layout as LY


@pytest.mark.parametrize("hkv,d,eb", [(1, 64, 2), (8, 128, 2), (2, 64, 4), (3, 128, 4)])
def test_is_a_permutation_and_round_trips(hkv, d, eb):
    idx = LY.element_index(hkv, 16, d, eb)
    n = 2 * hkv * 16 * d
    assert idx.shape == (2, hkv, 16, d)
    assert np.array_equal(np.sort(idx.ravel()), np.arange(n))
    dt = {2: np.uint16, 4: np.float32}[eb]
    rng = np.random.Generator(np.random.PCG64(5))
    logical = rng.integers(0, 60000, size=(3, 2, 2, hkv, 16, d)).astype(dt)
    phys = LY.to_physical(logical)
    assert phys.shape == (3, 2, n)
    assert np.array_equal(LY.from_physical(phys, hkv, 16, d), logical)


@pytest.mark.parametrize("d,eb", [(64, 2), (128, 2), (64, 4), (128, 4)])
def test_vectors_hold_what_the_header_says(d, eb):
    hkv = 2
    v = 16 // eb
    idx = LY.element_index(hkv, 16, d, eb)
    tile = 16 * d
    # tiles: K of head 0, K of head 1, V of head 0, V of head 1
    for kv in range(2):
        for g in range(hkv):
            lo = (kv * hkv + g) * tile
            assert idx[kv, g].min() == lo and idx[kv, g].max() == lo + tile - 1
    k = idx[0, 1] - tile
    # a K vector: v consecutive dims of one token; the 16 tokens of the same dims follow each other
    for t in range(16):
        for c0 in range(0, d, v):
            vec = k[t, c0:c0 + v]
            assert vec[0] % v == 0 and np.array_equal(vec, vec[0] + np.arange(v))
            assert vec[0] // v == (c0 // v) * 16 + t
    vt = idx[1, 0] - hkv * tile
    # a V vector: 4 consecutive tokens of one dim (and, 16-bit, of the dim 16 further) ...
    for t0 in range(0, 16, 4):
        for c in range(d):
            quad = vt[t0:t0 + 4, c]
            assert np.array_equal(quad, quad[0] + np.arange(4)) and quad[0] % 4 == 0
            if eb == 2 and (c // 16) % 2 == 0:
                assert vt[t0, c + 16] == quad[0] + 4 and quad[0] % 8 == 0
    # ... and the vectors of dims c0..c0+15 (same token quad) are 16 adjacent vectors
    for c0 in range(0, d, 16):
        first = vt[0, c0] // v
        if eb == 2 and (c0 // 16) % 2 == 1:
            continue
        assert np.array_equal(vt[0, c0:c0 + 16] // v, first + np.arange(16))


def test_positions_worked_out_by_hand():
    # fp16, d = 128, T = 16, one head: v = 8, w = 2
    idx = LY.element_index(1, 16, 128, 2)
    K, V = idx[0, 0], idx[1, 0] - 2048
    assert K[0, 0] == 0 and K[1, 0] == 8 and K[0, 8] == 128 and K[5, 77] == 9 * 128 + 5 * 8 + 5
    # V (t=6, c=50): c//32 = 1, t//4 = 1, c%16 = 2, (c//16)%2 = 1, t%4 = 2
    assert V[6, 50] == ((1 * 4 + 1) * 16 + 2) * 8 + 1 * 4 + 2
    assert V[0, 0] == 0 and V[0, 16] == 4 and V[0, 1] == 8 and V[4, 0] == 128 and V[0, 32] == 512
    # fp32, d = 64: v = 4, w = 1
    idx = LY.element_index(1, 16, 64, 4)
    K, V = idx[0, 0], idx[1, 0] - 1024
    assert K[3, 9] == 2 * 64 + 3 * 4 + 1
    assert V[9, 37] == ((2 * 4 + 2) * 16 + 5) * 4 + 1
