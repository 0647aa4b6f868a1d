"""Pins of the oracle's layer-granular swapping protocol against the paper's worked example
(Section 3.3, the nine-layer figure and the paragraphs around it) and the swap constraint of Section 3.1."""
import os

import pytest

from oracle import layer_fifo as LF

GOLD = {}
for line in open(os.path.join(os.path.dirname(__file__), "golden", "worked_example.txt")):
    line = line.split("#")[0].strip()
    if "=" in line:
        k, v = [x.strip() for x in line.split("=")]
        GOLD[k] = float(v)

N = int(GOLD["n_layers"])
M = int(GOLD["layers_on_cpu"])
RATIO = GOLD["t_swap_over_t_compute"]


def example(n_tokens=6, t_swap=RATIO):
    # layers 8 and 9 (here 7 and 8) start in CPU memory; the GPU holds n - m layer slots; the CPU holds the
    # m layers plus the two buffers the text gives each device
    return LF.simulate(N, N - M, M + 2, [N - 2, N - 1], n_tokens, t_compute=1.0, t_in=t_swap, t_out=t_swap)


def test_first_four_layers_of_the_worked_example():
    r = example()
    l1, l2, l3, l4 = r.records[:4]
    # layer 1: no swap-out, the CPU layers (8 and 9) are colder than any GPU layer
    assert l1.out_started is None and l1.out_skipped == "colder_on_host" and l1.in_started is None
    # layer 2: layer 1 is the coldest, its swap-out starts; no space for a swap-in
    assert l2.out_started == 0 and l2.in_started is None and l2.in_skipped == "no_slot"
    # layer 3: layer 1's swap-out still in progress: both skipped
    assert l3.out_started is None and l3.out_skipped == "busy" and l3.in_started is None
    # layer 4: layer 3 goes out; layer 1's space takes layer 8, the hottest layer in CPU memory
    assert l4.out_started == 2 and l4.in_started == N - 2


def test_fifo_is_four_long_and_every_layer_stays_eight_compute_times():
    r = example(n_tokens=8)
    assert r.max_away == int(GOLD["fifo_length"])
    # after the warm-up every record sees exactly that many layers away from the GPU
    later = [x for x in r.residences if x[1] is not None and x[1] >= 2 * N]
    assert len(later) >= 10
    assert all(abs((t_in_done - t_out_start) - GOLD["residence_compute_times"]) < 1e-9 for _, t_out_start, t_in_done in later)
    assert r.stall == 0.0                                     # performance-transparent
    assert abs(N / (N - M) - GOLD["expansion_printed"]) < 0.01


def test_swap_constraint_is_tight_at_two_compute_times_per_swap():
    """Section 3.1: transparent while t_swap * m <= t_compute * n.  In the example the link is busy all the
    time: n * t_compute / t_swap = 4.5 layers cross per token and direction."""
    r = example(n_tokens=12)
    steady = [x for x in r.records if x.token >= 2]
    tokens = len({x.token for x in steady})
    assert sum(x.out_started is not None for x in steady) / tokens == pytest.approx(N / RATIO)
    assert sum(x.in_started is not None for x in steady) / tokens == pytest.approx(N / RATIO)
    assert example(t_swap=RATIO * 1.1).stall > 0.0            # a slower link cannot hide it
    assert example(t_swap=RATIO * 0.5).stall == 0.0           # a faster one can


def test_nothing_moves_when_nothing_is_in_cpu_memory():
    r = LF.simulate(6, 6, 2, [], 3)
    assert all(x.out_started is None and x.in_started is None for x in r.records) and r.stall == 0.0


@pytest.mark.parametrize("n,gpu,host,on_host,t", [(9, 7, 4, [7, 8], 2.0), (12, 8, 6, [8, 9, 10, 11], 1.5),
                                                 (5, 3, 4, [0, 4], 0.7), (16, 10, 8, [1, 5, 9, 12, 13, 15], 3.3)])
def test_table_invariants(n, gpu, host, on_host, t):
    r = LF.simulate(n, gpu, host, on_host, 7, t_in=t, t_out=1.3 * t)
    # every layer is somewhere; slots are not shared; computations happen in order and never overlap
    g = [e.gpu_slot for e in r.table.values() if e.gpu_slot is not None]
    h = [e.host_slot for e in r.table.values() if e.host_slot is not None]
    assert len(set(g)) == len(g) <= gpu and len(set(h)) == len(h) <= host
    assert all(e.gpu_slot is not None or e.host_slot is not None for e in r.table.values())
    starts = [x.t_start for x in r.records]
    assert all(b - a >= 1.0 - 1e-12 for a, b in zip(starts, starts[1:]))
    assert [x.layer for x in r.records] == [k for _ in range(7) for k in range(n)]
    assert r.stall == pytest.approx(sum(x.t_start - x.t_begin for x in r.records))


def test_two_layers_in_cpu_memory_is_the_most_the_example_hides():
    """The example's choice of two CPU layers is the optimum for its timing: with t_swap = 2 t_compute the
    protocol runs without any wait for 0, 1 and 2 layers in CPU memory, and waits from 3 on."""
    def stall(m):
        return LF.simulate(N, N - m, m + 2, list(range(N - m, N)), 10, t_compute=1.0, t_in=RATIO, t_out=RATIO).stall
    assert [stall(m) == 0.0 for m in range(0, 6)] == [True, True, True, False, False, False]


def test_adaptive_expansion_finds_the_examples_two_layers_from_all_on_gpu():
    """Section 3.4.2 on the example's timing: start with every layer on the GPU, add a layer to swapping after
    k_up tokens without a wait, take one back after k_down tokens with waits.  The run overshoots to three
    layers, waits, and settles on two - the example's own choice and the most its timing hides."""
    levels, res = LF.simulate_adaptive(N, 6, 80, t_compute=1.0, t_in=RATIO, t_out=RATIO, k_up=4, k_down=2,
                                       probe_period=1000)
    assert levels[:4] == [0, 0, 0, 0]
    assert all(abs(b - a) <= 1 for a, b in zip(levels, levels[1:]))
    assert max(levels) == M + 1 and levels[-40:] == [M] * 40
    # the waits all belong to the tokens spent at three layers (and the one that drains the third)
    waits = {}
    for r in res.records:
        waits[r.token] = waits.get(r.token, 0.0) + (r.t_start - r.t_begin)
    assert all(w == 0.0 for t, w in waits.items() if levels[t] <= M and (t == 0 or levels[t - 1] <= M))
    # a faster link carries more: with t_swap = t_compute the same rule goes to the limit of the CPU slots
    levels, res = LF.simulate_adaptive(N, 6, 80, t_compute=1.0, t_in=1.0, t_out=1.0)
    assert levels[-1] == 4 and res.stall == 0.0


def test_layers_drain_back_when_every_gpu_slot_is_available():
    """With a GPU slot for every layer, the layers in CPU memory come back one by one and nothing leaves any
    more: a swap-out is only there to make room."""
    r = LF.simulate(N, N, 6, [N - 2, N - 1], 4)
    assert [x.in_started for x in r.records if x.in_started is not None] == [N - 2, N - 1]
    assert all(x.out_started is None for x in r.records)
    assert all(e.state == LF.GPU for e in r.table.values()) and r.stall == 0.0
