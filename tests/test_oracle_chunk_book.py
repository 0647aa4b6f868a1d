"""Pins for oracle/chunk_book.py: the redistribution the paper states (a / (n - m) per layer; its example's
1.28), the two visibility rules, and conservation under arbitrary histories."""
import os

import numpy as np
import pytest

from oracle.chunk_book import BookError, ChunkBook, ESTATE

G = {}
for line in open(os.path.join(os.path.dirname(__file__), "golden", "worked_example.txt")):
    line = line.split("#")[0].strip()
    if line:
        k, v = line.split("=")
        G[k.strip()] = float(v)


def test_worked_example_two_of_nine_layers_on_the_cpu_give_each_cache_nine_sevenths():
    n, m = int(G["n_layers"]), int(G["layers_on_cpu"])
    b = ChunkBook(n, 7 * n, 16)                      # seven chunks per layer when everything is on the GPU
    assert b.k_target == b.visible == 7
    assert b.set_layers_on_cpu(m, 7)
    assert b.k_target == 9 and b.target_for(m) == (7 * n) // (n - m)
    assert b.visible == 7                            # nothing has moved yet: nothing more to show
    b.left_gpu(8)
    assert b.visible == 7 and len(b.free) == 0       # the first layer's seven chunks went to layers 0-3 ...
    assert [len(c) for c in b.chunks] == [9, 9, 9, 8, 7, 7, 7, 7, 0]
    b.left_gpu(7)
    assert b.visible == 9                            # ... the second layer's complete it: now it shows
    assert [len(c) for c in b.chunks] == [9] * 7 + [0, 0] and not b.free
    assert int(b.visible / 7 * 100) / 100 == G["expansion_printed"]          # 9/7 = 1.2857 -> "1.28"
    b.check()
    # rotation as in the protocol: a layer leaves, one of the CPU's comes back with the new size, carrying 7
    b.left_gpu(0)
    assert b.visible == 9 and len(b.free) == 9
    got, n_data = b.enters_gpu(8)
    assert len(got) == 9 and n_data == 7 and b.visible == 9 and not b.free
    b.check()


def test_a_shrink_hides_at_once_and_waits_for_the_blocks_above_to_be_given_up():
    b = ChunkBook(9, 63, 16)
    b.set_layers_on_cpu(2, 7)
    b.left_gpu(8)
    b.left_gpu(7)
    assert b.visible == 9
    assert not b.set_layers_on_cpu(1, 9)             # chunks 8 and 9 of the caches still hold live blocks
    assert b.visible == 7 and b.k_target == 9 and b.m == 2        # hidden; nothing else has changed
    assert [len(c) for c in b.chunks][:7] == [9] * 7
    assert b.set_layers_on_cpu(1, 7)                 # the scheduler has drained them
    assert b.m == 1 and b.k_target == 7 and b.visible == 7
    assert [len(c) for c in b.chunks][:7] == [7] * 7 and len(b.free) == 14 and b.image == [7] * 9
    got, n_data = b.enters_gpu(7)
    assert len(got) == 7 and n_data == 7 and len(b.free) == 7
    b.check()
    # a refused shrink followed by growth shows everything again
    b2 = ChunkBook(4, 16, 8)
    b2.set_layers_on_cpu(2, 4)
    b2.left_gpu(3), b2.left_gpu(2)
    assert b2.visible == 8
    assert not b2.set_layers_on_cpu(1, 8) and b2.visible == 5
    assert b2.set_layers_on_cpu(2, 8) and b2.visible == 8


def test_a_leaving_layer_carries_only_what_it_is_told_is_live():
    b = ChunkBook(4, 16, 8)
    b.set_layers_on_cpu(2, 4)
    b.left_gpu(3, 3)                                 # three of its four chunks hold live blocks
    b.left_gpu(2)
    assert b.image == [4, 4, 4, 3] and b.visible == 8
    b.left_gpu(0, 5)                                 # grown to eight, five of them live
    got, n_data = b.enters_gpu(3)
    assert len(got) == 8 and n_data == 3
    with pytest.raises(BookError):
        b.left_gpu(1, 9)
    b.check()


def test_the_cap_per_layer_bounds_the_target():
    b = ChunkBook(4, 16, 6)
    assert [b.target_for(m) for m in range(4)] == [4, 5, 6, 6]


def test_errors():
    with pytest.raises(BookError):
        ChunkBook(4, 18, 8)                          # chunks must divide evenly at the start
    with pytest.raises(BookError):
        ChunkBook(4, 16, 3)
    b = ChunkBook(4, 16, 8)
    with pytest.raises(BookError) as e:
        b.enters_gpu(0)
    assert e.value.code == ESTATE
    b.left_gpu(0)
    with pytest.raises(BookError) as e:
        b.left_gpu(0)
    assert e.value.code == ESTATE
    with pytest.raises(BookError):
        b.set_layers_on_cpu(4, 0)


@pytest.mark.parametrize("seed", range(6))
def test_conservation_and_visibility_under_random_histories(seed):
    """Random requests and moves that respect the slot count: every chunk is always held once or free, every
    resident layer holds at least what is visible, and what is visible only falls by a shrink request."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n, k0, cap = 8, 6, 14
    b = ChunkBook(n, n * k0, cap)
    in_use = k0
    for _ in range(400):
        before = b.visible
        r = rng.random()
        n_res = sum(b.resident)
        if r < 0.15:
            m = int(rng.integers(0, n - 1))
            ok = b.set_layers_on_cpu(m, in_use)
            if not ok or b.target_for(m) < before:
                assert b.visible <= before
            else:
                assert b.visible >= min(before, b.k_target)
        elif r < 0.55 and n_res > max(1, n - b.m - 1):
            b.left_gpu(int(rng.choice([j for j in range(n) if b.resident[j]])))
            assert b.visible >= before
        elif n_res < n - b.m:
            cpu = [j for j in range(n) if not b.resident[j]]
            if cpu:
                j = int(rng.choice(cpu))
                got, n_data = b.enters_gpu(j)
                assert len(got) >= n_data and len(got) >= b.visible and b.visible >= before
        in_use = int(rng.integers(1, b.visible + 1))                  # the scheduler only uses what it is shown
        b.check()
