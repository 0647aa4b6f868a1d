"""The library's chunk book (host logic behind the C ABI) against the oracle's, call by call, on the worked
example and on random histories: same chunk lists, same data sizes, same visible / target / free counts, same
refusals."""
import numpy as np
import pytest

from oracle.chunk_book import BookError, ChunkBook as Model
from paper_2411_09317_amd import binding as B


def same(lib, mod):
    v, t, f, m = lib.capacity()
    assert (v, t, f, m) == (mod.visible, mod.k_target, len(mod.free), mod.m)
    for j in range(mod.n):
        res, n_data, chunks = lib.layer(j)
        assert res == mod.resident[j] and chunks == mod.chunks[j]
        assert n_data == mod.image[j]


def test_worked_example_step_by_step():
    lib, mod = B.ChunkBook(9, 63, 16), Model(9, 63, 16)
    same(lib, mod)
    assert lib.set_layers_on_cpu(2, 7) and mod.set_layers_on_cpu(2, 7)
    same(lib, mod)
    for j in (8, 7, 0):
        lib.left_gpu(j), mod.left_gpu(j)
        same(lib, mod)
    assert lib.enters_gpu(8) == mod.enters_gpu(8)
    same(lib, mod)
    assert lib.capacity()[0] == 9
    assert lib.set_layers_on_cpu(1, 9) is False and mod.set_layers_on_cpu(1, 9) is False
    same(lib, mod)
    assert lib.capacity()[0] == 7
    assert lib.set_layers_on_cpu(1, 7) and mod.set_layers_on_cpu(1, 7)
    same(lib, mod)
    lib.close()


@pytest.mark.parametrize("seed", range(8))
def test_random_histories(seed):
    rng = np.random.Generator(np.random.PCG64(100 + seed))
    n = int(rng.integers(3, 10))
    k0 = int(rng.integers(2, 8))
    cap = k0 + int(rng.integers(0, 10))
    lib, mod = B.ChunkBook(n, n * k0, cap), Model(n, n * k0, cap)
    in_use = k0
    for _ in range(300):
        r = rng.random()
        n_res = sum(mod.resident)
        if r < 0.2:
            m = int(rng.integers(0, n))
            assert lib.set_layers_on_cpu(m, in_use) == mod.set_layers_on_cpu(m, in_use)
        elif r < 0.6 and n_res > 1:
            j = int(rng.choice([j for j in range(n) if mod.resident[j]]))
            if rng.random() < 0.5:
                lib.left_gpu(j), mod.left_gpu(j)
            else:                                                      # it takes along only the live chunks
                carried = int(rng.integers(0, min(in_use, len(mod.chunks[j])) + 1))
                lib.left_gpu(j, carried), mod.left_gpu(j, carried)
        else:
            cpu = [j for j in range(n) if not mod.resident[j]]
            if cpu:
                j = int(rng.choice(cpu))
                try:
                    want = mod.enters_gpu(j)
                except BookError as e:
                    with pytest.raises(B.PieError) as got:
                        lib.enters_gpu(j)
                    assert got.value.code == e.code
                else:
                    assert lib.enters_gpu(j) == want
        same(lib, mod)
        mod.check()
        in_use = int(rng.integers(0, mod.visible + 1))
    lib.close()


def test_argument_checks():
    with pytest.raises(B.PieError) as e:
        B.ChunkBook(4, 18, 8)
    assert e.value.code == B.EINVAL
    with pytest.raises(B.PieError):
        B.ChunkBook(4, 16, 3)
    with pytest.raises(B.PieError):
        B.ChunkBook(4, 16, 100000)
    b = B.ChunkBook(4, 16, 8)
    with pytest.raises(B.PieError) as e:
        b.enters_gpu(0)
    assert e.value.code == B.ESTATE
    with pytest.raises(B.PieError) as e:
        b.left_gpu(7)
    assert e.value.code == B.EINVAL
    with pytest.raises(B.PieError):
        b.set_layers_on_cpu(4, 0)
    b.close()
