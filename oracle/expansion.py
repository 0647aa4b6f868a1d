"""Closed forms of the paper's capacity model.

Section 3.1: with n layers of KV cache, m of them on the CPU and a GB on the
GPU, each layer gets a/(n-m) GB and the effective cache is n*a/(n-m):
expansion = n/(n-m).  Swapping is performance-transparent while
t_swap*m <= t_compute*n.  Section 3.3 refines the ratio for the swap buffers
every device reserves (four buffers in the effective space, two on the
physical GPU): (n+4)/(n-m+2).  Section 1 bounds the effective extended memory
by prefetch bandwidth x prefetch interval x prefetch efficiency.

TEST INFRASTRUCTURE ONLY - never imported by the product path.
"""
from __future__ import annotations

from fractions import Fraction


def expansion_simple(n: int, m: int) -> Fraction:
    """Section 3.1: logical layers over layers physically on the GPU."""
    if not 0 <= m < n:
        raise ValueError("need 0 <= m < n")
    return Fraction(n, n - m)


def expansion_buffered(n: int, m: int) -> Fraction:
    """Section 3.3: the same ratio once swap buffers are counted."""
    if not 0 <= m < n:
        raise ValueError("need 0 <= m < n")
    return Fraction(n + 4, n - m + 2)


def max_transparent_layers(n: int, t_swap: float, t_compute: float) -> int:
    """Largest m with t_swap*m <= t_compute*n (Section 3.1), at most n - 1."""
    if t_swap <= 0:
        return n - 1
    m = int((t_compute * n) // t_swap)
    while t_swap * (m + 1) <= t_compute * n:
        m += 1
    while m > 0 and t_swap * m > t_compute * n:
        m -= 1
    return min(m, n - 1)


def expansion_from_host_fraction(f: float) -> float:
    """Block-granular form of n/(n-m) with f = m/n of the blocks on the host."""
    if not 0.0 <= f < 1.0:
        raise ValueError("need 0 <= f < 1")
    return 1.0 / (1.0 - f)


def expansion_with_staging(f: float, n_layers: int) -> float:
    """Block-granular ratio when two staging regions, each able to hold one
    layer's host-homed blocks, are carved out of the GPU's memory: per layer the
    GPU holds (1-f) of the blocks, plus 2f of one layer for staging in total."""
    if not 0.0 <= f < 1.0:
        raise ValueError("need 0 <= f < 1")
    return n_layers / (n_layers * (1.0 - f) + 2.0 * f)


def kv_bytes_per_token(n_layers: int, n_kv_heads: int, head_dim: int, elem_bytes: int) -> int:
    """Keys and values of one token over all layers."""
    return 2 * n_layers * n_kv_heads * head_dim * elem_bytes


def effective_extended_bytes(prefetch_bw: float, interval_s: float, efficiency: float = 1.0) -> float:
    """Section 1: bandwidth x interval x efficiency."""
    return prefetch_bw * interval_s * efficiency


def transparent_host_fraction(link_bw: float, attn_bw: float) -> float:
    """The bound above applied per layer to an attention-only step: a layer of
    S bytes is read in S/attn_bw seconds, in which link_bw*S/attn_bw bytes can be
    prefetched, so at most link_bw/attn_bw of it can live on the host."""
    return min(1.0, link_bw / attn_bw)
