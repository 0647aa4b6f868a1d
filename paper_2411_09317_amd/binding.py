"""ctypes binding of libpie.so: argument marshalling only.

Every step of the path (allocator, residency, swaps, attention, pipeline,
controller) runs inside the native library; this module converts Python
arguments to C ones, owns the torch tensors that back the pools, and raises
`PieError` for negative return codes.  There is no fallback: if the library has
not been built (`python -m paper_2411_09317_amd.build`) importing fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpie.so")

OK, EINVAL, ENOMEM, ESTATE, EHIP = 0, -1, -2, -3, -4
GPU, HOST = 0, 1
SWAP_AUTO, SWAP_DMA, SWAP_KERNEL = 0, 1, 2
DEVERR_BAD_HANDLE, DEVERR_NOT_PRESENT = 1, 2
TIMING_OFF, TIMING_EVENTS, TIMING_CLOCK = 0, 1, 2

# every symbol include/pie.h declares
SYMBOLS = [
    "pie_pool_bytes_required", "pie_pool_init", "pie_pool_destroy", "pie_block_alloc", "pie_block_free",
    "pie_block_where", "pie_block_staged", "pie_pool_free_count", "pie_block_address", "pie_swap_in", "pie_swap_out",
    "pie_migrate", "pie_set_host_fraction", "pie_set_swap_path", "pie_set_attn_partition", "pie_get_attn_partition_sync", "pie_set_swap_workgroups",
    "pie_set_layer_compute_us", "pie_set_attn_vector_alu",
    "pie_kv_append", "pie_attn_decode", "pie_attn_decode_static", "pie_attn_stream_probe_sync",
    "pie_step", "pie_set_async_submit", "pie_step_join_sync", "pie_prefetch_list", "pie_set_timing", "pie_set_cross_step_prefetch", "pie_set_host_presence_check", "pie_pool_sync", "pie_get_stats", "pie_get_layer_times",
    "pie_check_errors_sync", "pie_controller_create", "pie_controller_destroy", "pie_controller_config",
    "pie_controller_observe", "pie_controller_level", "pie_controller_update", "pie_last_hip_error", "pie_strerror",
    "pie_version",
    "pie_layer_sched_create", "pie_layer_sched_destroy", "pie_layer_sched_complete", "pie_layer_sched_present",
    "pie_layer_sched_policy", "pie_layer_sched_table", "pie_layer_sched_set_gpu_slots", "pie_layer_pool_set_gpu_slots", "pie_layer_pool_bytes_required", "pie_layer_pool_create",
    "pie_layer_pool_destroy", "pie_layer_step", "pie_layer_pool_settle_sync", "pie_layer_pool_address",
    "pie_layer_pool_table", "pie_layer_pool_stats",
    "pie_chunk_book_create", "pie_chunk_book_destroy", "pie_chunk_book_set_layers_on_cpu", "pie_chunk_book_left_gpu",
    "pie_chunk_book_enters_gpu", "pie_chunk_book_layer", "pie_chunk_book_capacity",
    "pie_elastic_bytes_required", "pie_elastic_create", "pie_elastic_destroy", "pie_elastic_set_layers_on_cpu",
    "pie_elastic_capacity", "pie_elastic_blocks_for", "pie_elastic_set_live_blocks", "pie_elastic_move_blocks", "pie_elastic_step", "pie_elastic_settle_sync", "pie_elastic_layer", "pie_elastic_table",
    "pie_elastic_stats",
]


class PieError(RuntimeError):
    def __init__(self, code: int, what: str = ""):
        self.code = code
        msg = _lib.pie_strerror(code).decode() if _lib is not None else str(code)
        if code == EHIP and _lib is not None:
            msg += f" (hipError {_lib.pie_last_hip_error()})"
        super().__init__(f"{what}: {msg} [{code}]")


class PieConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "n_q_heads", "n_kv_heads", "head_dim", "block_tokens", "dtype", "n_gpu_blocks", "n_stage_blocks",
        "n_host_blocks", "max_batch", "max_blocks_per_seq")] + [("softmax_scale", C.c_float)]


class PieStats(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("host_blocks_in_use", C.c_int32), ("gpu_blocks_in_use", C.c_int32),
                ("host_fraction", C.c_float), ("expansion_simple", C.c_float), ("expansion_staged", C.c_float),
                ("step_ms", C.c_float), ("attn_ms", C.c_float), ("swap_in_ms", C.c_float), ("swap_out_ms", C.c_float),
                ("stall_ms", C.c_float), ("bytes_in", C.c_uint64), ("bytes_out", C.c_uint64),
                ("device_error_flags", C.c_uint32), ("first_layer_prestaged", C.c_uint32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2411_09317_amd.build` "
                           "(there is no fallback path)")
    # PyTorch owns the device memory and the streams handed to the library, so both must talk to the same
    # HIP runtime: torch's wheel carries its own libamdhip64 (same soname as the system one); importing torch
    # first makes the dynamic loader resolve the library's dependency to that already-loaded copy.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    lib.pie_strerror.restype = C.c_char_p
    lib.pie_strerror.argtypes = [C.c_int]
    return lib


_lib = None
_lib = _load()


def lib():
    return _lib


def _i32(seq) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(seq, dtype=np.int32).ravel())


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _check(code: int, what: str):
    if code != OK:
        raise PieError(code, what)


def _stream_ptr(stream) -> C.c_void_p:
    if stream is None:
        return C.c_void_p(0)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def _dptr(t) -> C.c_void_p:
    if t is None:
        return C.c_void_p(0)
    return C.c_void_p(t.data_ptr())


class Pool:
    """A KV pool over torch-owned memory.  device=None makes a bookkeeping-only pool (no GPU needed)."""

    def __init__(self, n_layers, n_q_heads, n_kv_heads, head_dim, block_tokens, dtype, n_gpu_blocks, n_stage_blocks,
                 n_host_blocks, max_batch=1, max_blocks_per_seq=1, softmax_scale=0.0, device: Optional[str] = "cuda:0",
                 host_ptr: int = 0, host_bytes: int = 0):
        """host_ptr / host_bytes: page-locked host memory of the caller's own (e.g. hipHostMalloc with particular
        flags) for the host pool instead of a torch pinned tensor; the caller keeps it alive and frees it."""
        self.cfg = PieConfig(n_layers, n_q_heads, n_kv_heads, head_dim, block_tokens, dtype, n_gpu_blocks,
                             n_stage_blocks, n_host_blocks, max_batch, max_blocks_per_seq, softmax_scale)
        self._h = C.c_void_p(0)
        self.device = device
        d_bytes, h_bytes = C.c_size_t(0), C.c_size_t(0)
        _check(_lib.pie_pool_bytes_required(C.byref(self.cfg), C.byref(d_bytes), C.byref(h_bytes)), "bytes_required")
        self.d_bytes, self.h_bytes = d_bytes.value, h_bytes.value
        self.elem_bytes = 4 if dtype == 0 else 2
        self.block_bytes = 2 * n_kv_heads * block_tokens * head_dim * self.elem_bytes
        self.n_slots = n_gpu_blocks + 2 * n_stage_blocks
        self.d_buf = self.h_buf = None
        if device is not None:
            import torch
            self.d_buf = torch.empty(self.d_bytes + 256, dtype=torch.uint8, device=device)
            off = (-self.d_buf.data_ptr()) % 256
            self._d_base = self.d_buf.data_ptr() + off
            self._d_off = off
            if self.h_bytes and not host_ptr:
                self.h_buf = torch.empty(self.h_bytes, dtype=torch.uint8, pin_memory=True)
            h_ptr = host_ptr or (self.h_buf.data_ptr() if self.h_buf is not None else 0)
            _check(_lib.pie_pool_init(C.byref(self.cfg), C.c_void_p(self._d_base), C.c_size_t(self.d_bytes),
                                      C.c_void_p(h_ptr), C.c_size_t(host_bytes if host_ptr else self.h_bytes),
                                      C.byref(self._h)), "pool_init")
        else:
            _check(_lib.pie_pool_init(C.byref(self.cfg), C.c_void_p(0), C.c_size_t(0), C.c_void_p(0), C.c_size_t(0),
                                      C.byref(self._h)), "pool_init")

    def close(self):
        if self._h:
            _lib.pie_pool_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- views of the pools (plumbing for tests and benchmarks) ------------------
    def gpu_image(self):
        """uint8 view [L][n_gpu + 2*n_stage][block_bytes] of the device pool."""
        n = self.cfg.n_layers * self.n_slots * self.block_bytes
        return self.d_buf[self._d_off:self._d_off + n].view(self.cfg.n_layers, self.n_slots, self.block_bytes)

    def host_image(self):
        """uint8 view [L][n_host][block_bytes] of the pinned host pool."""
        return self.h_buf.view(self.cfg.n_layers, self.cfg.n_host_blocks, self.block_bytes)

    # ---- allocator ------------------------------------------------------------------
    def block_alloc(self, where: int, n: int) -> List[int]:
        out = np.empty(max(n, 1), dtype=np.int32)
        _check(_lib.pie_block_alloc(self._h, C.c_int32(where), C.c_int32(n), _ptr(out)), "block_alloc")
        return out[:n].tolist()

    def block_free(self, handles: Sequence[int]):
        h = _i32(handles)
        _check(_lib.pie_block_free(self._h, C.c_int32(len(h)), _ptr(h)), "block_free")

    def block_where(self, handles: Sequence[int]) -> Tuple[List[int], List[int]]:
        h = _i32(handles)
        w, s = np.empty(max(len(h), 1), np.int32), np.empty(max(len(h), 1), np.int32)
        _check(_lib.pie_block_where(self._h, C.c_int32(len(h)), _ptr(h), _ptr(w), _ptr(s)), "block_where")
        return w[:len(h)].tolist(), s[:len(h)].tolist()

    def block_staged(self, region: int, handles: Sequence[int]):
        h = _i32(handles)
        a, b = np.empty(max(len(h), 1), np.int32), np.empty(max(len(h), 1), np.int32)
        _check(_lib.pie_block_staged(self._h, C.c_int32(region), C.c_int32(len(h)), _ptr(h), _ptr(a), _ptr(b)),
               "block_staged")
        return a[:len(h)].tolist(), b[:len(h)].tolist()

    def n_free(self, where: int) -> int:
        n = C.c_int32(0)
        _check(_lib.pie_pool_free_count(self._h, C.c_int32(where), C.byref(n)), "free_count")
        return n.value

    def block_address(self, where: int, layer: int, slot: int) -> int:
        p = C.c_void_p(0)
        _check(_lib.pie_block_address(self._h, C.c_int32(where), C.c_int32(layer), C.c_int32(slot), C.byref(p)),
               "block_address")
        return p.value or 0

    # ---- swaps ------------------------------------------------------------------------
    def swap_in(self, layer: int, handles: Sequence[int], stream=None):
        h = _i32(handles)
        _check(_lib.pie_swap_in(self._h, C.c_int32(layer), C.c_int32(len(h)), _ptr(h), _stream_ptr(stream)), "swap_in")

    def swap_out(self, layer: int, handles: Sequence[int], stream=None):
        h = _i32(handles)
        _check(_lib.pie_swap_out(self._h, C.c_int32(layer), C.c_int32(len(h)), _ptr(h), _stream_ptr(stream)),
               "swap_out")

    def migrate(self, handles: Sequence[int], to_where: int, stream=None):
        h = _i32(handles)
        _check(_lib.pie_migrate(self._h, C.c_int32(len(h)), _ptr(h), C.c_int32(to_where), _stream_ptr(stream)),
               "migrate")

    def set_host_fraction(self, f: float, order: Sequence[int], stream=None) -> int:
        h = _i32(order)
        k = C.c_int32(0)
        _check(_lib.pie_set_host_fraction(self._h, C.c_float(f), C.c_int32(len(h)), _ptr(h), _stream_ptr(stream),
                                          C.byref(k)), "set_host_fraction")
        return k.value

    def set_swap_path(self, path: int):
        _check(_lib.pie_set_swap_path(self._h, C.c_int32(path)), "set_swap_path")

    def set_attn_partition(self, tokens: int):
        _check(_lib.pie_set_attn_partition(self._h, C.c_int32(tokens)), "set_attn_partition")

    def attn_partition(self) -> int:
        t = C.c_int32(0)
        _check(_lib.pie_get_attn_partition_sync(self._h, C.byref(t)), "get_attn_partition_sync")
        return t.value

    def set_swap_workgroups(self, n: int):
        _check(_lib.pie_set_swap_workgroups(self._h, C.c_int32(n)), "set_swap_workgroups")

    def set_attn_vector_alu(self, on: bool):
        _check(_lib.pie_set_attn_vector_alu(self._h, C.c_int32(1 if on else 0)), "set_attn_vector_alu")

    def set_layer_compute_us(self, us: float):
        _check(_lib.pie_set_layer_compute_us(self._h, C.c_float(us)), "set_layer_compute_us")

    # ---- per-layer operations (tensors are torch device tensors) --------------------------
    def kv_append(self, layer, k, v, block_table, ctx_lens, stream=None):
        B, mb = block_table.shape
        _check(_lib.pie_kv_append(self._h, C.c_int32(layer), _dptr(k), _dptr(v), _dptr(block_table), C.c_int32(mb),
                                  _dptr(ctx_lens), C.c_int32(B), _stream_ptr(stream)), "kv_append")

    def attn_decode(self, layer, q, block_table, ctx_lens, out, stream=None):
        B, mb = block_table.shape
        _check(_lib.pie_attn_decode(self._h, C.c_int32(layer), _dptr(q), _dptr(block_table), C.c_int32(mb),
                                    _dptr(ctx_lens), C.c_int32(B), _dptr(out), _stream_ptr(stream)), "attn_decode")

    def attn_decode_static(self, layer, q, block_table, ctx_lens, out, stream=None):
        """attn_decode with its scratch in the library's static device array (allocates nothing)."""
        B, mb = block_table.shape
        _check(_lib.pie_attn_decode_static(self._h, C.c_int32(layer), _dptr(q), _dptr(block_table), C.c_int32(mb),
                                           _dptr(ctx_lens), C.c_int32(B), _dptr(out), _stream_ptr(stream)),
               "attn_decode_static")

    def attn_stream_probe(self, layer, block_table, ctx_lens, stream=None) -> float:
        """Duration in ms of a kernel that only reads the bytes attn_decode would read."""
        ms = C.c_float(0)
        _check(_lib.pie_attn_stream_probe_sync(self._h, C.c_int32(layer), _dptr(block_table),
                                               C.c_int32(block_table.shape[1]), _dptr(ctx_lens),
                                               C.c_int32(ctx_lens.shape[0]), _stream_ptr(stream), C.byref(ms)),
               "attn_stream_probe")
        return ms.value

    def prefetch_list(self, block_table_host: np.ndarray, ctx_lens_host: np.ndarray):
        t = np.ascontiguousarray(block_table_host, dtype=np.int32)
        c = np.ascontiguousarray(ctx_lens_host, dtype=np.int32)
        B, mb = t.shape
        pf, dirty = np.empty(max(B * mb, 1), np.int32), np.empty(max(B, 1), np.int32)
        npf, nd = C.c_int32(0), C.c_int32(0)
        _check(_lib.pie_prefetch_list(self._h, _ptr(t), C.c_int32(mb), _ptr(c), C.c_int32(B), _ptr(pf), C.byref(npf),
                                      _ptr(dirty), C.byref(nd)), "prefetch_list")
        return pf[:npf.value].copy(), dirty[:nd.value].copy()

    def step(self, q_all, k_new, v_new, block_table, ctx_lens, prefetch, dirty, out_all, compute_stream=None,
             swap_in_stream=None, swap_out_stream=None):
        B, mb = block_table.shape
        pf, dt = _i32(prefetch), _i32(dirty)
        _check(_lib.pie_step(self._h, _dptr(q_all), _dptr(k_new), _dptr(v_new), _dptr(block_table), C.c_int32(mb),
                             _dptr(ctx_lens), C.c_int32(B), C.c_int32(len(pf)), _ptr(pf), C.c_int32(len(dt)), _ptr(dt),
                             _dptr(out_all), _stream_ptr(compute_stream), _stream_ptr(swap_in_stream),
                             _stream_ptr(swap_out_stream)), "step")

    # ---- control ---------------------------------------------------------------------------
    def set_async_submit(self, on: bool):
        """Steps are enqueued by a thread of the pool's own; step() returns at once."""
        _check(_lib.pie_set_async_submit(self._h, C.c_int32(1 if on else 0)), "set_async_submit")

    def step_join(self):
        _check(_lib.pie_step_join_sync(self._h), "step_join_sync")

    def set_cross_step_prefetch(self, on: bool):
        _check(_lib.pie_set_cross_step_prefetch(self._h, C.c_int32(1 if on else 0)), "set_cross_step_prefetch")

    def set_host_presence_check(self, on: bool):
        _check(_lib.pie_set_host_presence_check(self._h, C.c_int32(1 if on else 0)), "set_host_presence_check")

    def set_timing(self, mode):
        """False / TIMING_OFF, True / TIMING_EVENTS, or TIMING_CLOCK (kernels note their own times)."""
        _check(_lib.pie_set_timing(self._h, C.c_int32(int(mode))), "set_timing")

    def sync(self):
        _check(_lib.pie_pool_sync(self._h), "pool_sync")

    def stats(self) -> PieStats:
        s = PieStats()
        _check(_lib.pie_get_stats(self._h, C.byref(s)), "get_stats")
        return s

    def layer_times(self):
        L = self.cfg.n_layers
        arrs = [np.zeros(L, dtype=np.float32) for _ in range(5)]
        ps = [a.ctypes.data_as(C.POINTER(C.c_float)) for a in arrs]
        _check(_lib.pie_get_layer_times(self._h, *ps), "get_layer_times")
        return dict(zip(("attn", "kernel", "swap_in", "swap_out", "stall"), arrs))

    def check_errors(self) -> int:
        f = C.c_uint32(0)
        _check(_lib.pie_check_errors_sync(self._h, C.byref(f)), "check_errors_sync")
        return f.value


class Controller:
    """Adaptive-expansion controller (pure host logic inside the library)."""

    def __init__(self, units: int, k_max: int, rho=0.9, k_up=4, k_down=2, probe_period=64, plateau_eps=0.01,
                 util_max=0.9, stall_eps=0.01):
        self._h = C.c_void_p(0)
        self.units = units
        _check(_lib.pie_controller_create(C.c_int32(units), C.c_int32(k_max), C.byref(self._h)), "controller_create")
        _check(_lib.pie_controller_config(self._h, C.c_double(rho), C.c_int32(k_up), C.c_int32(k_down),
                                          C.c_int32(probe_period), C.c_double(plateau_eps), C.c_double(util_max),
                                          C.c_double(stall_eps)), "controller_config")

    def observe(self, t_attn, t_in, t_stall, link_util: float, throughput: float) -> int:
        a = np.ascontiguousarray(t_attn, dtype=np.float64)
        i = np.ascontiguousarray(t_in, dtype=np.float64)
        s = np.ascontiguousarray(t_stall, dtype=np.float64)
        dp = C.POINTER(C.c_double)
        lvl = C.c_int32(0)
        _check(_lib.pie_controller_observe(self._h, C.c_int32(len(a)), a.ctypes.data_as(dp), i.ctypes.data_as(dp),
                                           s.ctypes.data_as(dp), C.c_double(link_util), C.c_double(throughput),
                                           C.byref(lvl)), "controller_observe")
        return lvl.value

    def level(self) -> Tuple[int, int]:
        k, c = C.c_int32(0), C.c_int32(0)
        _check(_lib.pie_controller_level(self._h, C.byref(k), C.byref(c)), "controller_level")
        return k.value, c.value

    def update_from_pool(self, pool: Pool, throughput: float) -> float:
        f = C.c_float(0)
        _check(_lib.pie_controller_update(pool._h, self._h, C.c_double(throughput), C.byref(f)), "controller_update")
        return f.value

    def close(self):
        if self._h:
            _lib.pie_controller_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- layer-granular swapping ----------------------------------------------------------------------------

LAYER_GPU, LAYER_HOST, LAYER_MOVING_OUT, LAYER_MOVING_IN = 0, 1, 2, 3
WAIT_NONE, WAIT_IN, WAIT_OUT = 0, 1, 2
SKIP_NOT, SKIP_BUSY, SKIP_NO_SLOT, SKIP_COLDER_ON_HOST, SKIP_NONE, SKIP_ROOM_LEFT = 0, 1, 2, 3, 4, 5


class LayerEntry(C.Structure):
    _fields_ = [("state", C.c_int32), ("gpu_slot", C.c_int32), ("host_slot", C.c_int32)]


class LayerAction(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("wait", "gpu_slot", "in_layer", "in_gpu_slot", "in_host_slot", "out_layer",
                                         "out_gpu_slot", "out_host_slot", "forced_in", "out_skipped", "in_skipped")]


class LayerStats(C.Structure):
    _fields_ = [("n_steps", C.c_int64), ("n_swap_in", C.c_int64), ("n_swap_out", C.c_int64),
                ("n_forced_in", C.c_int64), ("bytes_in", C.c_uint64), ("bytes_out", C.c_uint64),
                ("stall_ms", C.c_double)]


class LayerSched:
    """The layer-granular swapping protocol as pure host logic (no GPU)."""

    def __init__(self, n_layers: int, n_gpu_slots: int, n_host_slots: int, on_host: Sequence[int]):
        self._h = C.c_void_p(0)
        self.n_layers = n_layers
        oh = _i32(on_host)
        _check(_lib.pie_layer_sched_create(C.c_int32(n_layers), C.c_int32(n_gpu_slots), C.c_int32(n_host_slots),
                                           C.c_int32(len(oh)), _ptr(oh), C.byref(self._h)), "layer_sched_create")

    def complete(self, which: int):
        _check(_lib.pie_layer_sched_complete(self._h, C.c_int32(which)), "layer_sched_complete")

    def present(self, layer: int) -> LayerAction:
        a = LayerAction()
        _check(_lib.pie_layer_sched_present(self._h, C.c_int32(layer), C.byref(a)), "layer_sched_present")
        return a

    def policy(self, layer: int) -> LayerAction:
        a = LayerAction()
        _check(_lib.pie_layer_sched_policy(self._h, C.c_int32(layer), C.byref(a)), "layer_sched_policy")
        return a

    def table(self) -> List[Tuple[int, int, int]]:
        arr = (LayerEntry * self.n_layers)()
        _check(_lib.pie_layer_sched_table(self._h, arr), "layer_sched_table")
        return [(e.state, e.gpu_slot, e.host_slot) for e in arr]

    def set_gpu_slots(self, n: int):
        _check(_lib.pie_layer_sched_set_gpu_slots(self._h, C.c_int32(n)), "layer_sched_set_gpu_slots")

    def close(self):
        if self._h:
            _lib.pie_layer_sched_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class LayerPool:
    """Logical layers over a Pool of GPU layer slots plus a pinned array of CPU layer slots."""

    def __init__(self, pool: Pool, n_layers: int, n_host_slots: int, on_host: Sequence[int]):
        import torch
        self.pool = pool
        self.n_layers = n_layers
        self._h = C.c_void_p(0)
        hb = C.c_size_t(0)
        _check(_lib.pie_layer_pool_bytes_required(pool._h, C.c_int32(n_host_slots), C.byref(hb)), "layer_pool_bytes")
        self.layer_bytes = pool.cfg.n_gpu_blocks * pool.block_bytes
        self.h_buf = torch.empty(max(hb.value, 1), dtype=torch.uint8, pin_memory=True)
        oh = _i32(on_host)
        _check(_lib.pie_layer_pool_create(pool._h, C.c_int32(n_layers), C.c_int32(n_host_slots),
                                          C.c_void_p(self.h_buf.data_ptr()), C.c_size_t(hb.value), C.c_int32(len(oh)),
                                          _ptr(oh), C.byref(self._h)), "layer_pool_create")

    def step(self, q_all, k_new, v_new, block_table, ctx_lens, out_all, compute_stream=None, swap_in_stream=None,
             swap_out_stream=None):
        _check(_lib.pie_layer_step(self._h, _dptr(q_all), _dptr(k_new), _dptr(v_new), _dptr(block_table),
                                   C.c_int32(block_table.shape[1]), _dptr(ctx_lens), C.c_int32(ctx_lens.shape[0]),
                                   _dptr(out_all), _stream_ptr(compute_stream), _stream_ptr(swap_in_stream),
                                   _stream_ptr(swap_out_stream)), "layer_step")

    def settle(self):
        _check(_lib.pie_layer_pool_settle_sync(self._h), "layer_pool_settle")

    def set_gpu_slots(self, n: int):
        _check(_lib.pie_layer_pool_set_gpu_slots(self._h, C.c_int32(n)), "layer_pool_set_gpu_slots")

    def table(self) -> List[Tuple[int, int, int]]:
        arr = (LayerEntry * self.n_layers)()
        _check(_lib.pie_layer_pool_table(self._h, arr), "layer_pool_table")
        return [(e.state, e.gpu_slot, e.host_slot) for e in arr]

    def layer_image(self, layer: int):
        """uint8 torch tensor [n_gpu_blocks][block_bytes] aliasing the logical layer's image where it is now."""
        where, ptr = C.c_int32(0), C.c_void_p(0)
        _check(_lib.pie_layer_pool_address(self._h, C.c_int32(layer), C.byref(where), C.byref(ptr)), "layer_pool_address")
        if where.value == GPU:
            off = ptr.value - self.pool._d_base
            return self.pool.d_buf[self.pool._d_off + off: self.pool._d_off + off + self.layer_bytes].view(
                self.pool.cfg.n_gpu_blocks, self.pool.block_bytes)
        off = ptr.value - self.h_buf.data_ptr()
        return self.h_buf[off: off + self.layer_bytes].view(self.pool.cfg.n_gpu_blocks, self.pool.block_bytes)

    def stats(self) -> LayerStats:
        s = LayerStats()
        _check(_lib.pie_layer_pool_stats(self._h, C.byref(s)), "layer_pool_stats")
        return s

    def close(self):
        if self._h:
            _lib.pie_layer_pool_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class ChunkBook:
    """Which chunks of GPU memory each layer's cache holds (pure host logic inside the library)."""

    def __init__(self, n_layers: int, n_chunks: int, max_chunks_per_layer: int):
        self._h = C.c_void_p(0)
        self.n_layers, self.k_cap = n_layers, max_chunks_per_layer
        _check(_lib.pie_chunk_book_create(C.c_int32(n_layers), C.c_int32(n_chunks), C.c_int32(max_chunks_per_layer),
                                          C.byref(self._h)), "chunk_book_create")

    def set_layers_on_cpu(self, m: int, chunks_in_use: int) -> bool:
        rc = _lib.pie_chunk_book_set_layers_on_cpu(self._h, C.c_int32(m), C.c_int32(chunks_in_use))
        if rc == ESTATE:
            return False
        _check(rc, "chunk_book_set_layers_on_cpu")
        return True

    def left_gpu(self, layer: int, n_carried: int = -1):
        _check(_lib.pie_chunk_book_left_gpu(self._h, C.c_int32(layer), C.c_int32(n_carried)), "chunk_book_left_gpu")

    def enters_gpu(self, layer: int) -> Tuple[List[int], int]:
        n_data = C.c_int32(0)
        _check(_lib.pie_chunk_book_enters_gpu(self._h, C.c_int32(layer), C.byref(n_data)), "chunk_book_enters_gpu")
        return self.layer(layer)[2], n_data.value

    def layer(self, layer: int) -> Tuple[bool, int, List[int]]:
        """(resident, chunks of data it carries, chunk ids it holds)."""
        res, nd, nc = C.c_int32(0), C.c_int32(0), C.c_int32(0)
        ch = np.zeros(self.k_cap, dtype=np.int32)
        _check(_lib.pie_chunk_book_layer(self._h, C.c_int32(layer), C.byref(res), C.byref(nd), C.byref(nc), _ptr(ch)),
               "chunk_book_layer")
        return bool(res.value), nd.value, ch[:nc.value].tolist()

    def capacity(self) -> Tuple[int, int, int, int]:
        """(visible, target, free chunks, layers asked to be in CPU memory)."""
        v, t, f, m = C.c_int32(0), C.c_int32(0), C.c_int32(0), C.c_int32(0)
        _check(_lib.pie_chunk_book_capacity(self._h, C.byref(v), C.byref(t), C.byref(f), C.byref(m)), "chunk_book_capacity")
        return v.value, t.value, f.value, m.value

    def close(self):
        if self._h:
            _lib.pie_chunk_book_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class ElasticPool:
    """The layer-granular protocol over layer caches made of chunks of a Pool's GPU memory."""

    def __init__(self, pool: Pool, chunk_blocks: int, max_chunks_per_layer: int, n_host_slots: int):
        import torch
        self.pool, self.C, self.k_cap = pool, chunk_blocks, max_chunks_per_layer
        self.n_layers = pool.cfg.n_layers
        self.chunk_bytes = chunk_blocks * pool.block_bytes
        self._h = C.c_void_p(0)
        db, hb = C.c_size_t(0), C.c_size_t(0)
        _check(_lib.pie_elastic_bytes_required(pool._h, C.c_int32(chunk_blocks), C.c_int32(max_chunks_per_layer),
                                               C.c_int32(n_host_slots), C.byref(db), C.byref(hb)), "elastic_bytes")
        self.d_work = torch.empty(max(db.value, 16), dtype=torch.uint8, device=pool.d_buf.device)
        self.h_buf = torch.empty(max(hb.value, 1), dtype=torch.uint8, pin_memory=True)
        _check(_lib.pie_elastic_create(pool._h, C.c_int32(chunk_blocks), C.c_int32(max_chunks_per_layer),
                                       C.c_int32(n_host_slots), C.c_void_p(self.d_work.data_ptr()), C.c_size_t(db.value),
                                       C.c_void_p(self.h_buf.data_ptr()), C.c_size_t(hb.value), C.byref(self._h)),
               "elastic_create")

    def set_layers_on_cpu(self, m: int, blocks_in_use_end: int, compute_stream=None) -> bool:
        rc = _lib.pie_elastic_set_layers_on_cpu(self._h, C.c_int32(m), C.c_int32(blocks_in_use_end),
                                                _stream_ptr(compute_stream))
        if rc == ESTATE:
            return False
        _check(rc, "elastic_set_layers_on_cpu")
        return True

    def blocks_for(self, m: int) -> int:
        """Blocks per layer when m layers are kept in CPU memory and the reallocation is complete."""
        n = C.c_int32(0)
        _check(_lib.pie_elastic_blocks_for(self._h, C.c_int32(m), C.byref(n)), "elastic_blocks_for")
        return n.value

    def move_blocks(self, src: Sequence[int], dst: Sequence[int], compute_stream=None):
        a, b = _i32(src), _i32(dst)
        _check(_lib.pie_elastic_move_blocks(self._h, C.c_int32(len(a)), _ptr(a), _ptr(b), _stream_ptr(compute_stream)),
               "elastic_move_blocks")

    def set_live_blocks(self, blocks_in_use_end: int):
        _check(_lib.pie_elastic_set_live_blocks(self._h, C.c_int32(blocks_in_use_end)), "elastic_set_live_blocks")

    def capacity(self) -> Tuple[int, int, int]:
        """(visible blocks per layer, target blocks per layer, layers asked to be in CPU memory)."""
        v, t, m = C.c_int32(0), C.c_int32(0), C.c_int32(0)
        _check(_lib.pie_elastic_capacity(self._h, C.byref(v), C.byref(t), C.byref(m)), "elastic_capacity")
        return v.value, t.value, m.value

    def step(self, q_all, k_new, v_new, block_table, ctx_lens, out_all, compute_stream=None, swap_in_stream=None,
             swap_out_stream=None):
        _check(_lib.pie_elastic_step(self._h, _dptr(q_all), _dptr(k_new), _dptr(v_new), _dptr(block_table),
                                     C.c_int32(block_table.shape[1]), _dptr(ctx_lens), C.c_int32(ctx_lens.shape[0]),
                                     _dptr(out_all), _stream_ptr(compute_stream), _stream_ptr(swap_in_stream),
                                     _stream_ptr(swap_out_stream)), "elastic_step")

    def settle(self, compute_stream=None):
        _check(_lib.pie_elastic_settle_sync(self._h, _stream_ptr(compute_stream)), "elastic_settle")

    def table(self) -> List[Tuple[int, int, int]]:
        arr = (LayerEntry * self.n_layers)()
        _check(_lib.pie_elastic_table(self._h, arr), "elastic_table")
        return [(e.state, e.gpu_slot, e.host_slot) for e in arr]

    def layer_chunks(self, layer: int):
        """The layer's cache as a list of uint8 torch tensors [chunk_blocks][block_bytes], one per chunk, aliasing
        the memory where it is now (GPU chunks, or the chunks of data in its host image)."""
        where, n, hp = C.c_int32(0), C.c_int32(0), C.c_void_p(0)
        ch = np.zeros(self.k_cap, dtype=np.int32)
        _check(_lib.pie_elastic_layer(self._h, C.c_int32(layer), C.byref(where), C.byref(n), _ptr(ch), C.byref(hp)),
               "elastic_layer")
        out = []
        for i in range(n.value):
            if where.value == GPU:
                off = self.pool._d_off + int(ch[i]) * self.chunk_bytes
                out.append(self.pool.d_buf[off: off + self.chunk_bytes].view(self.C, self.pool.block_bytes))
            else:
                off = hp.value - self.h_buf.data_ptr() + i * self.chunk_bytes
                out.append(self.h_buf[off: off + self.chunk_bytes].view(self.C, self.pool.block_bytes))
        return where.value, out

    def stats(self) -> LayerStats:
        s = LayerStats()
        _check(_lib.pie_elastic_stats(self._h, C.byref(s)), "elastic_stats")
        return s

    def close(self):
        if self._h:
            _lib.pie_elastic_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
