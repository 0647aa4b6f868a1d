"""Pins for oracle/expansion.py: values the paper prints and closed forms."""
from fractions import Fraction

import pytest

from conftest import load_golden
from oracle import expansion as ex

G = load_golden("worked_example.txt")


def test_worked_example_expansion_is_the_simple_form():
    n, m = int(G["n_layers"]), int(G["layers_on_cpu"])
    e = ex.expansion_simple(n, m)
    assert e == Fraction(9, 7)
    # the paper prints 1.28: 9/7 = 1.2857 cut to two decimals
    assert int(float(e) * 100) / 100 == G["expansion_printed"]


def test_buffered_form_on_the_same_example():
    # (n+4)/(n-m+2) = 13/9: not what the example prints, so the example uses the simple form
    e = ex.expansion_buffered(9, 2)
    assert e == Fraction(13, 9)
    assert abs(float(e) - G["expansion_printed"]) > 0.1


def test_transparency_bound_worked_example():
    # t_swap = 2 t_compute, n = 9: the queue holds 4 layers; 4*2 = 8 <= 9 but 5*2 = 10 > 9
    n = int(G["n_layers"])
    r = G["t_swap_over_t_compute"]
    assert ex.max_transparent_layers(n, r, 1.0) == int(G["fifo_length"])
    assert r * 4 <= n < r * 5


@pytest.mark.parametrize("n,ts,tc", [(9, 2.0, 1.0), (32, 7.7, 0.288), (80, 1.0, 1.0), (10, 3.0, 0.9), (6, 0.5, 1.0)])
def test_transparency_bound_bruteforce(n, ts, tc):
    brute = max(m for m in range(0, n) if ts * m <= tc * n)
    assert ex.max_transparent_layers(n, ts, tc) == brute


def test_kv_bytes_per_token_opt13b():
    b = ex.kv_bytes_per_token(int(G["opt13b_layers"]), int(G["opt13b_heads"]), int(G["opt13b_head_dim"]),
                              int(G["opt13b_elem_bytes"]))
    assert b == 819200                              # = 800 KiB, printed as "800 KB"
    assert b / 1024 == G["opt13b_kv_kb_per_token"]
    gb = b * G["opt13b_request_tokens"] / 2 ** 30   # 1.5625 GiB; 1.68e9 bytes; the paper rounds to 1.6
    assert abs(gb - G["opt13b_request_gb"]) < 0.1


def test_block_forms_agree_with_layer_forms():
    for n in (9, 32, 80):
        for m in range(0, n):
            f = m / n
            assert ex.expansion_from_host_fraction(f) == pytest.approx(float(ex.expansion_simple(n, m)), rel=1e-12)
    # staging form: f = 0 -> 1; and it is below the simple form whenever f > 0
    assert ex.expansion_with_staging(0.0, 32) == 1.0
    for f in (0.1, 0.3, 0.6):
        assert 1.0 < ex.expansion_with_staging(f, 32) < ex.expansion_from_host_fraction(f)
    # closed form: L / (L(1-f) + 2f)
    assert ex.expansion_with_staging(0.5, 4) == pytest.approx(4 / (2 + 1))


def test_effective_extended_memory_bound():
    # bandwidth x interval x efficiency; on the paper's machine a 20 ms token at 419 GB/s hides 8.38 GB
    assert ex.effective_extended_bytes(G["gh200_h2d_gbs"] * 1e9, 0.020) == pytest.approx(8.38e9)
    assert ex.effective_extended_bytes(100.0, 2.0, 0.5) == 100.0
    # per-layer form: fraction = link / achieved attention bandwidth
    assert ex.transparent_host_fraction(419e9, 0.7 * 4e12) == pytest.approx(0.1496, abs=1e-3)
    assert ex.transparent_host_fraction(10.0, 5.0) == 1.0


def test_argument_checks():
    with pytest.raises(ValueError):
        ex.expansion_simple(9, 9)
    with pytest.raises(ValueError):
        ex.expansion_from_host_fraction(1.0)
