"""MI355X-native paged-attention decode over a KV cache split between a GPU
block pool and a pinned-host pool, with per-layer prefetch of host-resident
blocks (performance-transparent swapping) and an adaptive-expansion controller.

`inputs` (seeded synthetic workloads) is importable without the native library;
`binding` loads the HIP library and fails loudly if it has not been built.
"""
__all__ = ["inputs", "binding"]
