"""GPU memory handed on between the layers' caches when layers move to CPU memory.

The paper (Section 3.1 and Section 4.1, block manager) keeps m of n layers' KV
caches in CPU memory and gives the GPU memory they leave to the layers that
stay: a cache of a bytes per n layers becomes a / (n - m) per layer.  New
blocks are shown to the scheduler only once the reallocation is complete;
when the cache shrinks, blocks are hidden from the scheduler first and freed
afterwards.  A layer that leaves takes along the chunks that hold live blocks
(the caller says how many); the rest it simply gives up.

The paper reallocates a layer's cache as one piece when the layer is swapped
back in.  This build cuts the GPU memory into N chunks of equal size and lets a
layer's cache be any set of chunks (block h of a layer lives in its chunk
h // C), so a resident layer can be given more chunks where it is.  What this
model keeps of the protocol: the target a / (n - m) per layer, in whole chunks;
growth becomes visible when every resident layer holds the new amount, which
cannot happen before the m layers have left; a shrink lowers what is visible
at once and is refused while chunks above the new size are still in use.

Counting only - no bytes, no transfers.  The driver reports "layer j has left
the GPU" (its swap-out completed) and "layer j enters" (its swap-in starts).

TEST INFRASTRUCTURE ONLY - never imported by the product path.
"""
from __future__ import annotations

EINVAL, ENOMEM, ESTATE = -1, -2, -3


class BookError(Exception):
    def __init__(self, code, msg=""):
        super().__init__(f"{code}: {msg}")
        self.code = code


class ChunkBook:
    def __init__(self, n_layers: int, n_chunks: int, max_chunks_per_layer: int):
        if n_layers <= 0 or n_chunks <= 0 or n_chunks % n_layers or max_chunks_per_layer < n_chunks // n_layers:
            raise BookError(EINVAL)
        self.n, self.N, self.k_cap = n_layers, n_chunks, max_chunks_per_layer
        k0 = n_chunks // n_layers
        self.chunks = [list(range(j * k0, (j + 1) * k0)) for j in range(n_layers)]   # chunk ids a resident layer holds
        self.resident = [True] * n_layers
        self.image = [k0] * n_layers       # chunks of data the layer carries (all it holds; what it took to the CPU)
        self.free = []                     # kept sorted
        self.m = 0
        self.k_target = k0
        self.hide = None                   # a refused shrink keeps the visible size down
        self.visible = k0

    def target_for(self, m: int) -> int:
        return min(self.k_cap, self.N // (self.n - m))

    # ---- requests -----------------------------------------------------------------------------------
    def set_layers_on_cpu(self, m: int, chunks_in_use: int) -> bool:
        """Asks for m layers in CPU memory.  chunks_in_use: how many chunks of a layer's cache still hold live
        blocks (the highest live block's chunk + 1).  False: the cache would have to shrink below that; what is
        visible has been lowered all the same, and nothing else has changed."""
        if not 0 <= m < self.n or chunks_in_use < 0:
            raise BookError(EINVAL)
        k_new = self.target_for(m)
        if k_new < self.k_target:
            self.hide = k_new
            self._recount()
            if chunks_in_use > k_new:
                return False
            for j in range(self.n):                      # cut every cache to the new size where it is
                if self.resident[j]:
                    while len(self.chunks[j]) > k_new:
                        self._release(self.chunks[j].pop())
                self.image[j] = min(self.image[j], k_new)
        self.m, self.k_target, self.hide = m, k_new, None
        self._top_up()
        return True

    # ---- what the driver reports ------------------------------------------------------------------
    def left_gpu(self, j: int, n_carried=None):
        """n_carried: how many of its chunks the layer took along (those with live blocks; all by default)."""
        if not self.resident[j]:
            raise BookError(ESTATE)
        if n_carried is not None and not 0 <= n_carried <= len(self.chunks[j]):
            raise BookError(EINVAL)
        self.resident[j] = False
        self.image[j] = len(self.chunks[j]) if n_carried is None else n_carried
        for c in self.chunks[j]:
            self._release(c)
        self.chunks[j] = []
        self._top_up()

    def enters_gpu(self, j: int):
        """Returns (chunks now held, chunks of data to bring).  The lowest free chunks, up to the target."""
        if self.resident[j]:
            raise BookError(ESTATE)
        k = min(self.k_target, len(self.free))
        if k < max(self.image[j], self.visible):         # what is visible never shrinks behind the scheduler's back
            raise BookError(ENOMEM)
        self.chunks[j], self.free = self.free[:k], self.free[k:]
        self.resident[j] = True
        self._recount()
        return list(self.chunks[j]), self.image[j]

    # ---- internals -----------------------------------------------------------------------------------
    def _release(self, c):
        self.free.append(c)
        self.free.sort()

    def _top_up(self):
        """Free chunks go to resident layers below the target, lowest layer first, one layer filled before the
        next; what the GPU slots still to be filled will need is kept back."""
        n_res = sum(self.resident)
        reserve = max(0, (self.n - self.m) - n_res) * self.k_target
        for j in range(self.n):
            if not self.resident[j]:
                continue
            while len(self.chunks[j]) < self.k_target and len(self.free) > reserve:
                self.chunks[j].append(self.free.pop(0))
        self._recount()

    def _recount(self):
        held = [len(self.chunks[j]) for j in range(self.n) if self.resident[j]]
        v = min([self.k_target] + held)
        # layers in CPU memory come back with at least what they carry; until then their size bounds nothing
        self.visible = v if self.hide is None else min(v, self.hide)

    # ---- checks used by the tests ---------------------------------------------------------------------
    def check(self):
        ids = [c for j in range(self.n) for c in self.chunks[j]] + self.free
        assert sorted(ids) == list(range(self.N)), "every chunk is held once or free"
        assert self.free == sorted(self.free)
        for j in range(self.n):
            assert self.resident[j] or not self.chunks[j]
            assert not self.resident[j] or len(self.chunks[j]) >= self.visible
            assert self.image[j] <= self.k_cap
        assert self.visible <= self.k_target <= self.k_cap
