"""Seeded synthetic inputs for the paged-attention decode + KV swapping path.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic (no attention, no allocator policy, no controller rule) so
that both the CPU oracle's tests and the HIP path's tests can be fed the same
data without sharing any code of the method itself.

The workloads stand in for the ShareGPT / Alpaca request mixes the paper
evaluates on (Evaluation Setup, "Workloads"): only their shape is kept, i.e.
variable, skewed context lengths; every value is i.i.d. Gaussian.

All host-side draws use numpy's PCG64 so they are reproducible across machines.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Tuple

import numpy as np

DTYPE_F32, DTYPE_F16, DTYPE_BF16 = 0, 1, 2
DTYPE_NAMES = {DTYPE_F32: "f32", DTYPE_F16: "f16", DTYPE_BF16: "bf16"}
DTYPE_BYTES = {DTYPE_F32: 4, DTYPE_F16: 2, DTYPE_BF16: 2}


@dataclass(frozen=True)
class Workload:
    """Shape of one synthetic decode workload (one of the five named configs)."""
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: int
    block_tokens: int = 16
    ctx_dist: str = "uniform"          # "uniform" | "lognormal" | "fixed"
    ctx_lo: int = 64
    ctx_hi: int = 256
    ctx_median: int = 1024
    ctx_sigma: float = 0.7
    value_scale: float = 1.0
    host_fraction: float = 0.0
    seed: int = 0
    ffn_dim: int = 0                   # MLP width of the public architecture the shape is taken from (0: none)

    @property
    def elem_bytes(self) -> int:
        return DTYPE_BYTES[self.dtype]

    @property
    def block_bytes(self) -> int:
        return 2 * self.n_kv_heads * self.block_tokens * self.head_dim * self.elem_bytes

    @property
    def kv_bytes_per_token_layer(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * self.elem_bytes

    @property
    def layer_weight_bytes(self) -> int:
        """Bytes of one transformer layer's weights for this shape at the cache's element size: query and
        output projections (hidden x hidden), key and value projections (hidden x kv width), and a gated MLP
        of three hidden x ffn_dim matrices."""
        hidden, kv = self.n_q_heads * self.head_dim, self.n_kv_heads * self.head_dim
        return (2 * hidden * hidden + 2 * hidden * kv + 3 * hidden * self.ffn_dim) * self.elem_bytes


# The five workloads the build is measured and parity-tested on.
CONFIGS: Dict[str, Workload] = {
    "cfg1": Workload("cfg1", 1, 4, 8, 8, 64, DTYPE_F32, ctx_dist="uniform", ctx_lo=64, ctx_hi=256,
                     value_scale=1.0, host_fraction=0.25, seed=0),
    "cfg2": Workload("cfg2", 32, 64, 32, 32, 128, DTYPE_F16, ctx_dist="uniform", ctx_lo=1024, ctx_hi=2048,
                     value_scale=0.5, host_fraction=0.0, seed=1, ffn_dim=11008),
    "cfg3": Workload("cfg3", 32, 64, 32, 32, 128, DTYPE_F16, ctx_dist="uniform", ctx_lo=1024, ctx_hi=2048,
                     value_scale=0.5, host_fraction=0.30, seed=2, ffn_dim=11008),
    "cfg4": Workload("cfg4", 32, 256, 32, 8, 128, DTYPE_BF16, ctx_dist="lognormal", ctx_lo=128, ctx_hi=4096,
                     ctx_median=1024, ctx_sigma=0.7, value_scale=0.5, host_fraction=0.0, seed=3, ffn_dim=14336),
    "cfg5": Workload("cfg5", 80, 32, 64, 8, 128, DTYPE_BF16, ctx_dist="fixed", ctx_lo=32768, ctx_hi=32768,
                     value_scale=0.5, host_fraction=0.0, seed=4, ffn_dim=28672),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller batch, fewer layers...)."""
    return replace(w, **kw)


def rng_for(w: Workload, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([w.seed, stream]))


def draw_ctx_lens(w: Workload) -> np.ndarray:
    """Context lengths, each including the token being decoded. int32[batch]."""
    g = rng_for(w, 1)
    if w.ctx_dist == "uniform":
        ctx = g.integers(w.ctx_lo, w.ctx_hi + 1, size=w.batch)
    elif w.ctx_dist == "lognormal":
        ctx = np.rint(g.lognormal(np.log(w.ctx_median), w.ctx_sigma, size=w.batch))
        ctx = np.clip(ctx, w.ctx_lo, w.ctx_hi)
    elif w.ctx_dist == "fixed":
        ctx = np.full(w.batch, w.ctx_hi)
    else:
        raise ValueError(w.ctx_dist)
    return ctx.astype(np.int32)


def draw_requests(w: Workload, n: int, rate_per_s: float, out_lo: int, out_hi: int):
    """A seeded request stream: Poisson arrivals (exponential gaps, `rate_per_s` requests per second), prompt
    lengths from the workload's context-length distribution, output lengths uniform in [out_lo, out_hi].
    Returns (arrival seconds float64[n], prompt_len int32[n], output_len int32[n])."""
    g = rng_for(w, 5)
    arrival = np.cumsum(g.exponential(1.0 / rate_per_s, size=n))
    prompt = draw_ctx_lens(scaled(w, batch=n, seed=w.seed + 7919))
    output = g.integers(out_lo, out_hi + 1, size=n).astype(np.int32)
    return arrival, prompt, output


def blocks_needed(ctx_lens: np.ndarray, block_tokens: int) -> np.ndarray:
    return (ctx_lens.astype(np.int64) + block_tokens - 1) // block_tokens


def draw_host_mask(w: Workload, n_blocks: np.ndarray, fraction: float | None = None) -> List[np.ndarray]:
    """For each sequence a boolean array over its logical blocks: True = homed in
    the pinned host pool.  round(fraction * n) blocks of each sequence, at least
    one when fraction > 0, chosen uniformly at random."""
    f = w.host_fraction if fraction is None else fraction
    g = rng_for(w, 2)
    out = []
    for nb in n_blocks:
        nb = int(nb)
        m = np.zeros(nb, dtype=bool)
        if f > 0:
            k = min(nb, max(1, int(np.rint(f * nb))))
            m[g.choice(nb, size=k, replace=False)] = True
        out.append(m)
    return out


def draw_slot_permutation(w: Workload, n_slots: int) -> np.ndarray:
    """A random permutation of a pool's slot ids (physical placement of blocks)."""
    return rng_for(w, 3).permutation(n_slots).astype(np.int32)


def draw_promotion_order(w: Workload, n_blocks: np.ndarray) -> np.ndarray:
    """A seeded permutation of all (sequence, logical block) pairs.  Taking a
    prefix of it as the host set makes host sets nested as the fraction grows.
    int32[total, 2]."""
    pairs = np.array([(b, j) for b, nb in enumerate(n_blocks) for j in range(int(nb))], dtype=np.int32)
    return pairs[rng_for(w, 4).permutation(len(pairs))]


# ---------------------------------------------------------------------------
# value draws and storage rounding (input preparation only)
# ---------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def to_storage(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round float values to the storage type.  fp32 -> float32 array, fp16 ->
    float16 array, bf16 -> uint16 array of bit patterns."""
    if dtype == DTYPE_F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == DTYPE_F16:
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16)
    if dtype == DTYPE_BF16:
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def storage_numpy_dtype(dtype: int):
    return {DTYPE_F32: np.float32, DTYPE_F16: np.float16, DTYPE_BF16: np.uint16}[dtype]


def draw_values(w: Workload, shape: Tuple[int, ...], stream: int) -> np.ndarray:
    """i.i.d. N(0,1) * value_scale as float32 (not yet rounded to storage)."""
    return (rng_for(w, stream).standard_normal(size=shape, dtype=np.float32) * np.float32(w.value_scale))


@dataclass
class DecodeCase:
    """Everything one decode step over a workload needs, as host arrays."""
    w: Workload
    ctx_lens: np.ndarray                 # int32[B], includes the token being decoded
    n_blocks: np.ndarray                 # int64[B]
    host_mask: List[np.ndarray]          # per sequence, bool[nb_b]
    q: np.ndarray                        # storage [L][B][Hq][d]
    k_dense: List[np.ndarray]            # per sequence, storage [L][ctx_b][Hkv][d]
    v_dense: List[np.ndarray]
    extra: dict = field(default_factory=dict)

    @property
    def max_blocks(self) -> int:
        return int(self.n_blocks.max()) if len(self.n_blocks) else 0


def make_case(w: Workload, host_fraction: float | None = None, ctx_lens=None) -> DecodeCase:
    """Draw a whole decode case on the host (use only for sizes that fit RAM).  ctx_lens: given context
    lengths (one per sequence of the workload's batch) instead of drawn ones."""
    ctx = draw_ctx_lens(w) if ctx_lens is None else np.asarray(ctx_lens, dtype=np.int32)
    assert ctx.shape == (w.batch,)
    nb = blocks_needed(ctx, w.block_tokens)
    mask = draw_host_mask(w, nb, host_fraction)
    q = to_storage(draw_values(w, (w.n_layers, w.batch, w.n_q_heads, w.head_dim), 10), w.dtype)
    kd, vd = [], []
    for b in range(w.batch):
        kd.append(to_storage(draw_values(w, (w.n_layers, int(ctx[b]), w.n_kv_heads, w.head_dim), 100 + 2 * b), w.dtype))
        vd.append(to_storage(draw_values(w, (w.n_layers, int(ctx[b]), w.n_kv_heads, w.head_dim), 101 + 2 * b), w.dtype))
    return DecodeCase(w, ctx, nb, mask, q, kd, vd)
