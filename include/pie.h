/*
 * pie.h - C ABI of the MI355X paged-attention decode path with
 * performance-transparent KV-cache swapping.
 *
 * The path follows the paper "Pie: Pooling CPU Memory for LLM Inference":
 *   - Section 3.2 (architecture, mapping table, two-phase update, presence
 *     check before a layer is computed),
 *   - Section 3.3 (prefetch of the data the next layer needs behind the current
 *     layer's computation),
 *   - Section 3.4.2 and Section 1 (adaptive expansion and its three growth
 *     conditions),
 *   - Section 4.1 (block manager: free list, base pointer + unchanged offset).
 * The unit of residency is a KV block (16 tokens of one layer, all KV heads,
 * keys and values) instead of a whole layer: a logical block, named by a
 * handle, is homed in the same slot of every layer of either the GPU pool or
 * the pinned-host pool.
 *
 * Conventions
 *   - Every function returns 0 (PIE_OK) or a negative error code; nothing
 *     throws or aborts across this boundary.  On error no state has changed
 *     unless stated otherwise.
 *   - Pointers named d_* are device pointers, h_* host pointers.  `stream`
 *     arguments are hipStream_t passed as void*; NULL is the default stream.
 *   - No function waits for the GPU unless its name ends in _sync, with one exception: a swap or migration
 *     that goes through the copy engine (PIE_SWAP_DMA, or PIE_SWAP_AUTO choosing it) waits on the host for
 *     the work the copy must follow (the staging region's last reader and write-back), and then enqueues
 *     the copy; this runtime gives the best overlap that way.  pie_step therefore paces the host one layer
 *     behind the GPU on that path - unless the pool submits asynchronously (pie_set_async_submit): pie_step then
 *     returns at once and a thread of the pool's own does the enqueuing and the waiting.
 *   - Ownership: the caller allocates the device buffer, the pinned host buffer
 *     and the streams, and frees them after pie_pool_destroy.  The library
 *     allocates no device memory at any time.
 *   - One pool is driven by one host thread; attention / append calls of one
 *     pool go to one compute stream at a time.
 *   - Pool layout (both pools): [layer][slot][block]; in the device buffer a
 *     layer holds n_gpu_blocks resident slots, then staging region 0, then
 *     staging region 1 (n_stage_blocks each).  A block is one contiguous chunk
 *     of 2 * n_kv_heads * 16 * head_dim elements: the K tiles of kv heads
 *     0..n_kv_heads-1, then their V tiles, each tile 16 tokens x head_dim.
 *     Inside a tile the elements are ordered for 16-byte vector access.  With
 *     v = 16 / sizeof(element) and w = v / 4, element (token t, dim c) sits at
 *       K tile:  (c / v) * (16 * v) + t * v + c % v
 *       V tile:  (((c / (16 * w)) * 4 + t / 4) * 16 + c % 16) * v
 *                + ((c / 16) % w) * 4 + t % 4
 *     (a K vector = v consecutive dims of one token, the 16 tokens' vectors of
 *     those dims adjacent; a V vector = 4 consecutive tokens of one dim and,
 *     for 16-bit types, of the dim 16 further).  pie_kv_append writes rows in
 *     this order; callers that fill blocks through pie_block_address must too.
 *   - Handles are int32 in [0, n_gpu_blocks + n_host_blocks); -1 marks an
 *     unused block-table entry.
 */
#ifndef PIE_H
#define PIE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PIE_OK      0
#define PIE_EINVAL (-1)  /* bad argument */
#define PIE_ENOMEM (-2)  /* pool, staging region or buffer too small */
#define PIE_ESTATE (-3)  /* operation not valid for the block's / pool's state */
#define PIE_EHIP   (-4)  /* HIP runtime error; see pie_last_hip_error */

#define PIE_DTYPE_F32  0
#define PIE_DTYPE_F16  1
#define PIE_DTYPE_BF16 2

#define PIE_WHERE_GPU  0
#define PIE_WHERE_HOST 1

/* swap paths (pie_set_swap_path) */
#define PIE_SWAP_AUTO   0  /* per transfer: the copy engine unless the list is so scattered that the kernel is faster */
#define PIE_SWAP_DMA    1  /* one hipMemcpyAsync per contiguous run of slots */
#define PIE_SWAP_KERNEL 2  /* gather / scatter kernel reading or writing pinned host memory directly */

typedef struct pie_pool pie_pool;
typedef struct pie_controller pie_controller;

typedef struct {
  int32_t n_layers;
  int32_t n_q_heads;
  int32_t n_kv_heads;        /* divides n_q_heads; 16-bit dtypes: n_q_heads / n_kv_heads <= 16 */
  int32_t head_dim;          /* 64 or 128 */
  int32_t block_tokens;      /* 16 */
  int32_t dtype;             /* PIE_DTYPE_*; fp32 caches are served by a plain kernel that reads a kv head's K and V
                                once per query head (G x the traffic with grouped queries): for validation, not speed */
  int32_t n_gpu_blocks;      /* resident slots per layer */
  int32_t n_stage_blocks;    /* slots per staging region (there are two) */
  int32_t n_host_blocks;     /* host slots per layer */
  int32_t max_batch;         /* sizes the split-context workspace */
  int32_t max_blocks_per_seq;/* likewise; also the largest block-table width accepted */
  float   softmax_scale;     /* 0 => 1/sqrt(head_dim) */
} pie_config;

/* Filled by pie_get_stats; times in milliseconds, from the last pie_step's monitoring (pie_set_timing: HIP
 * events or the device clock). */
typedef struct {
  int32_t n_layers;
  int32_t host_blocks_in_use;   /* handles currently homed on the host */
  int32_t gpu_blocks_in_use;
  float   host_fraction;        /* host / (host + gpu) blocks in use */
  float   expansion_simple;     /* 1 / (1 - f): Section 3.1 */
  float   expansion_staged;     /* L / (L (1 - f) + 2 f): Section 3.3's buffer-corrected ratio, block form */
  float   step_ms;              /* first layer's start to last layer's end on the compute stream */
  float   attn_ms;              /* sum over layers of attention + reduction time */
  float   swap_in_ms;           /* sum over layers */
  float   swap_out_ms;
  float   stall_ms;             /* sum over layers of the compute stream's waits for a layer's prefetch */
  uint64_t bytes_in;            /* host -> GPU bytes moved by the last pie_step */
  uint64_t bytes_out;
  uint32_t device_error_flags;  /* PIE_DEVERR_* collected by pie_check_errors_sync calls so far */
  uint32_t first_layer_prestaged; /* 1: the last pie_step found layer 0's host blocks already staged by the step before */
} pie_stats;

#define PIE_DEVERR_BAD_HANDLE   1u  /* a block-table entry outside [0, n_handles) inside a sequence's context */
#define PIE_DEVERR_NOT_PRESENT  2u  /* a block that is neither GPU-homed nor staged for this layer */

/* ---- pool (Section 4.1 block manager; Section 3.2 mapping table) -------- */

/* Bytes the caller must provide: device buffer (KV slots incl. staging, handle maps, split workspace)
 * and pinned host buffer (host slots).  PIE_EINVAL for an unsupported config. */
int pie_pool_bytes_required(const pie_config* cfg, size_t* d_bytes, size_t* h_bytes);

/* Creates a pool over caller-owned memory.  d_base: device memory, 256-byte aligned, >= d_bytes required.
 * h_pinned_base: page-locked host memory the GPU can address (hipHostMalloc / torch pin_memory), >= h_bytes
 * required; may be NULL when n_host_blocks == 0.  Passing d_base == NULL creates a bookkeeping-only pool
 * (allocator, residency, tables; any call that would touch the device returns PIE_ESTATE) - used to test
 * host logic without a GPU.  Neither buffer is cleared.  PIE_ENOMEM if a buffer is too small. */
int pie_pool_init(const pie_config* cfg, void* d_base, size_t d_bytes,
                  void* h_pinned_base, size_t h_bytes, pie_pool** out);

/* Waits for the pool's outstanding work, destroys its events, frees its host bookkeeping.  Caller buffers
 * are untouched. */
int pie_pool_destroy(pie_pool* pool);

/* Takes n blocks from pool `where`: the n lowest free handles paired, ascending, with the n lowest free
 * slots.  All or nothing: PIE_ENOMEM if fewer than n slots (or handles) are free. */
int pie_block_alloc(pie_pool* pool, int32_t where, int32_t n, int32_t* out_handles);

/* Returns blocks to their free lists.  PIE_EINVAL for a handle out of range, PIE_ESTATE for one that is not
 * allocated or is repeated; all or nothing.  The caller must not free blocks that enqueued work still reads. */
int pie_block_free(pie_pool* pool, int32_t n, const int32_t* handles);

/* Home of each handle: out_where[i] = PIE_WHERE_* or -1 if unallocated, out_slot[i] = slot in that pool. */
int pie_block_where(pie_pool* pool, int32_t n, const int32_t* handles, int32_t* out_where, int32_t* out_slot);

/* Staged copy of each handle in staging region `region` (0/1): out_stage_slot[i] = slot in the device pool
 * (n_gpu_blocks + region * n_stage_blocks + rank) or -1; out_state[i] = 0 not staged, 1 copy in flight,
 * 2 present (the region's swap-in event has completed - the second phase of the mapping-table update). */
int pie_block_staged(pie_pool* pool, int32_t region, int32_t n, const int32_t* handles,
                     int32_t* out_stage_slot, int32_t* out_state);

/* Number of free slots in a pool. */
int pie_pool_free_count(pie_pool* pool, int32_t where, int32_t* out_n);

/* Device / host address of a block's bytes for one layer (slot in the device pool, staging included, or in
 * the host pool), for callers that fill or inspect the cache directly. */
int pie_block_address(pie_pool* pool, int32_t where, int32_t layer, int32_t slot, void** out_ptr);

/* ---- swaps (Section 3.2 two-phase update; Section 3.3) ------------------ */

/* Prefetch: copies layer `layer` of the n host-homed blocks into staging region (layer & 1); handles[i] lands
 * in staging slot i, replacing whatever the region held.  Asynchronous on `stream`; the stream first waits
 * for earlier readers and write-backs of the region.  The block becomes "present" when the copy's event
 * completes; pie_attn_decode / pie_kv_append of that layer wait for it on their stream.
 * PIE_ENOMEM if n > n_stage_blocks; PIE_ESTATE if a handle is not allocated, not host-homed or repeated. */
int pie_swap_in(pie_pool* pool, int32_t layer, int32_t n, const int32_t* handles, void* stream);

/* Write-back: copies the staged copies of `layer` for the n handles to their host slots.  The handles must
 * be staged in region (layer & 1) and the region must hold `layer` (PIE_ESTATE otherwise).  Asynchronous on
 * `stream`, after the compute stream's work on that layer enqueued so far. */
int pie_swap_out(pie_pool* pool, int32_t layer, int32_t n, const int32_t* handles, void* stream);

/* Re-homes blocks, all layers, in pool `to_where` (lowest free slots, in list order); handles already there
 * are skipped; staged copies of moved blocks are dropped.  Asynchronous on `stream`, ordered after compute
 * work enqueued so far; later compute work waits for it.  PIE_ENOMEM (nothing moved) if the target lacks slots. */
int pie_migrate(pie_pool* pool, int32_t n, const int32_t* handles, int32_t to_where, void* stream);

/* Fixed-fraction mode (the paper's fixed expansion): of the n handles in `order`, the first
 * floor(f*n + 0.5) are homed on the host and the rest on the GPU (blocks coming back move first).  The caller
 * supplies the order (e.g. a seeded permutation) so that host sets are nested as f grows.  out_n_host may be
 * NULL. */
int pie_set_host_fraction(pie_pool* pool, float f, int32_t n, const int32_t* order, void* stream,
                          int32_t* out_n_host);

/* Chooses how swaps move bytes (PIE_SWAP_*). */
int pie_set_swap_path(pie_pool* pool, int32_t path);

/* Tokens of one sequence handled by one attention workgroup (rounded up to a multiple of 64, clamped to
 * [256, 4096]); longer contexts are split and reduced.  0, the default: chosen on the device for every batch,
 * from 512 / 768 / 1024 / 1536 / 2048 / 3072 / 4096, as the largest size that still leaves the persistent decode
 * grid more than about eight and a half (partition, kv head) units per workgroup (small units even out the
 * workgroups' different streaming rates, every unit has a fixed cost). */
int pie_set_attn_partition(pie_pool* pool, int32_t tokens);

/* The size the last attention planning launch used (the one set, or the one chosen).  Waits for the pool. */
int pie_get_attn_partition_sync(pie_pool* pool, int32_t* out_tokens);

/* 16-bit caches with one query head per kv head (MHA): on != 0 computes the attention's two products on the
 * vector ALU (two-element dot products, fp32 accumulation) instead of the matrix cores, where with a single query
 * head they are matrix-vector products.  Same loads, same order, same softmax; results agree to rounding.  Off by
 * default: on the 7B-shaped workload the kernel takes the same time either way (it is bound by HBM) and a step
 * 0.7 % longer on the vector ALU.  PIE_ESTATE for grouped-query or fp32 pools. */
int pie_set_attn_vector_alu(pie_pool* pool, int32_t on);

/* Workgroups of the gather / scatter kernel (1..1024, default 16).  The kernel is bound by the host link, not
 * by compute.  A transfer of up to 12 MiB - one that can hide behind a layer - is moved by that many workgroups
 * of 256 threads (about 28 GB/s beside a running decode kernel, which slows by 2-3 %); a larger one by that many
 * one-wavefront workgroups with sixteen 16-byte accesses in flight per lane (about 41 GB/s, the decode kernels it
 * runs beside slow by 2-3 %).  More workgroups move more and disturb more; the link's own limit is near 56 GB/s,
 * which the copy engine reaches. */
int pie_set_swap_workgroups(pie_pool* pool, int32_t n);

/* Stand-in for the rest of a transformer layer.  The paper's per-layer compute time (Section 3.1, the
 * t_compute of its swap constraint) covers the whole layer - projections and MLP, i.e. mostly the time to
 * read the layer's weights - while this library computes only the attention.  With us > 0, pie_step keeps
 * the compute stream busy for about `us` microseconds after each layer's attention (one idle wave watching
 * the clock; no memory traffic), and counts that time in the layer's t_attn.  Default 0: off.  It is a
 * knob for experiments on the controller and the overlap, not part of the measured path. */
int pie_set_layer_compute_us(pie_pool* pool, float us);

/* ---- per-layer operations ------------------------------------------------ */

/* Appends this step's key and value rows.  d_k, d_v: [batch][n_kv_heads][head_dim] in the pool's dtype.
 * For sequence b the rows go to token position ctx_lens[b] - 1, i.e. block d_block_table[b][(ctx-1)/T], row
 * (ctx-1)%T, in the block's GPU home or, for a host-homed block, its staged copy for this layer (the block
 * is then dirty until pie_swap_out).  A host-homed block that is not staged raises PIE_DEVERR_NOT_PRESENT on
 * the device and is skipped.  d_block_table: int32 [batch][max_blocks] of handles. */
int pie_kv_append(pie_pool* pool, int32_t layer, const void* d_k, const void* d_v,
                  const int32_t* d_block_table, int32_t max_blocks,
                  const int32_t* d_ctx_lens, int32_t batch, void* stream);

/* Decode attention for one layer: for sequence b and query head h (KV head h / (n_q_heads / n_kv_heads))
 *   out[b][h] = sum_t softmax_t(scale * <q[b][h], K[b][g][t]>) V[b][g][t],  t < ctx_lens[b],
 * reading K and V through the block table (Section 2.3's paged KV cache; the per-layer access of Section
 * 3.2).  d_q, d_out: [batch][n_q_heads][head_dim] in the pool's dtype; accumulation is fp32.  ctx 0 gives
 * zeros.  The stream first waits until the layer's staged blocks are present (the presence check).
 * PIE_EINVAL if batch > max_batch or max_blocks > max_blocks_per_seq. */
int pie_attn_decode(pie_pool* pool, int32_t layer, const void* d_q,
                    const int32_t* d_block_table, int32_t max_blocks,
                    const int32_t* d_ctx_lens, int32_t batch,
                    void* d_out, void* stream);

/* pie_attn_decode for callers that cannot allocate or hand over scratch memory - code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc: same arguments, same kernels, same result bit for bit,
 * but the call's scratch (planning state, ticket counter, split-context partials) lives in a static device array
 * inside the library instead of the pool's workspace in the caller's buffer; the pool's max_batch and
 * max_blocks_per_seq, which size that workspace, do not limit this call.  The array is 40 MiB, held by every
 * GPU the library runs on until the process ends.  A call needs about
 *   batch * n_q_heads * ceil(16 * max_blocks / partition) * (head_dim + 2) * 4 bytes  (partials)
 *   + batch * (2 * max_blocks + 600) * 4 bytes                                         (planning state);
 * PIE_ENOMEM if that exceeds the array (nothing is enqueued), PIE_EINVAL if batch > 4096.  Calls no hipMalloc,
 * hipFree or other allocating routine; clears what it needs with its own kernels.  All calls on one GPU share
 * the array: two calls that overlap in time on one GPU (different streams or pools) race - serialise them. */
int pie_attn_decode_static(pie_pool* pool, int32_t layer, const void* d_q,
                           const int32_t* d_block_table, int32_t max_blocks,
                           const int32_t* d_ctx_lens, int32_t batch,
                           void* d_out, void* stream);

/* Calibration for the roofline of pie_attn_decode: reads exactly the K and V tiles that pie_attn_decode would
 * read for this layer, batch and table - same work items, same order, same loads - and discards them.
 * Waits for it and returns the kernel's duration in *out_ms (events around the launch on `stream`): the rate
 * at which this access pattern can stream from HBM at all. */
int pie_attn_stream_probe_sync(pie_pool* pool, int32_t layer, const int32_t* d_block_table, int32_t max_blocks,
                               const int32_t* d_ctx_lens, int32_t batch, void* stream, float* out_ms);

/* ---- the pipeline ---------------------------------------------------------- */

/* One decode step over all layers.  h_prefetch: the n_prefetch host-homed handles this batch touches, in
 * any order - the host cannot read the device block table, so the caller names them (pie_prefetch_list
 * computes the list from a host copy of the table, ordered by host slot so that the copies are contiguous).
 * h_dirty: the n_dirty of those that receive this step's token (host-homed tail blocks).
 * For l = 0..L-1: layer l runs on compute_stream once its staged blocks are present; layer l+1's blocks are
 * prefetched on swap_in_stream into the other staging region meanwhile.  With a new token (d_k_new), the
 * attention reads the context without it from the cache and takes the token itself from d_k_new / d_v_new, so
 * no layer waits for the rows to be stored: those of the GPU-homed tail blocks of all layers are written by one
 * launch on swap_out_stream beside the first layers (compute_stream is ordered after it when the step ends),
 * those of host-homed tails into their staged copies on swap_out_stream once the copy has arrived, and from
 * there layer l's dirty blocks go home at once (the layer only reads them, so append and write-back run beside
 * it; swap_in_stream carries nothing but the copies, back to back).  Behind the last layer, layer 0's blocks
 * are brought in once more for the step that follows (see pie_set_cross_step_prefetch).
 * d_k_new and d_v_new must be 8-byte aligned and stay valid until the step has run.
 * d_q_all, d_out_all: [L][batch][n_q_heads][head_dim]; d_k_new, d_v_new: [L][batch][n_kv_heads][head_dim]
 * (NULL skips the append).  Argument errors are detected before anything is enqueued; a HIP error in the
 * middle (PIE_EHIP) leaves the step partly enqueued. */
int pie_step(pie_pool* pool, const void* d_q_all, const void* d_k_new, const void* d_v_new,
             const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_ctx_lens, int32_t batch,
             int32_t n_prefetch, const int32_t* h_prefetch, int32_t n_dirty, const int32_t* h_dirty,
             void* d_out_all, void* compute_stream, void* swap_in_stream, void* swap_out_stream);

/* Host-homed handles among h_block_table[b][j], j < ceil(ctx/T), without repeats, in ascending order of their
 * host slot (a densely used host pool is then read as one contiguous run); and of those the tail blocks
 * (entry (ctx-1)/T), same order.  out arrays need room for batch*max_blocks and batch entries. */
int pie_prefetch_list(pie_pool* pool, const int32_t* h_block_table, int32_t max_blocks,
                      const int32_t* h_ctx_lens, int32_t batch,
                      int32_t* out_prefetch, int32_t* out_n_prefetch, int32_t* out_dirty, int32_t* out_n_dirty);

/* Asynchronous submission.  With on != 0, pie_step checks its arguments, copies the two handle lists, hands the
 * step to a thread that belongs to the pool and returns (a few microseconds); the thread enqueues the step
 * exactly as pie_step would have, in the order the steps were given.  For callers whose host thread has other
 * work between steps (scheduling the next iteration), above all on the copy-engine path, where enqueuing a step
 * takes as long as the step.  What changes for the caller:
 *   - the step's work appears on the three streams as the thread gets to it, so work the caller itself puts on
 *     those streams right after pie_step is not ordered after the step; pie_step_join_sync (below) returns when
 *     everything handed over has been enqueued, and from then on stream order holds as usual;
 *   - every other call on the pool (pie_pool_sync included) first waits for the thread to run dry, so calls that
 *     change residency between steps cannot overtake a step;
 *   - an error the thread meets while enqueuing (PIE_EHIP) is returned by the next call that waits for it.
 * Device and host arguments of a step must stay valid until it has run, as always.  Off by default. */
int pie_set_async_submit(pie_pool* pool, int32_t on);

/* Waits until every step handed to the pool's thread has been enqueued (not: has run), and returns the first
 * error met on the way.  Returns at once when asynchronous submission was never switched on. */
int pie_step_join_sync(pie_pool* pool);

/* pie_step ends by bringing layer 0's host blocks in again, behind its last layer, for the step that follows
 * (the paper's swapping runs around the layer loop, token after token: Section 3.3's worked example); the
 * next pie_step uses them if it is given the same prefetch list and none of those blocks was freed, moved or
 * swapped in between, else it copies as usual.  On by default; 0 turns it off.  Whoever writes into the
 * host pool's memory directly between two steps must turn it off or call pie_swap_in for layer 0 afterwards. */
int pie_set_cross_step_prefetch(pie_pool* pool, int32_t on);

/* On the copy-engine path pie_step already paces the host with the GPU; it then also looks for a layer's
 * swap-in from the host (polling its event while the layer before computes, until shortly before that ends)
 * and queues the layer without a wait on the compute stream when it has seen the swap-in complete.  On by
 * default; 0 makes pie_step always wait on the stream (no polling on the host). */
int pie_set_host_presence_check(pie_pool* pool, int32_t on);

/* How pie_step monitors itself (the per-layer times the adaptive expansion needs, Section 3.4.2).
 *   PIE_TIMING_OFF    nothing is measured (default).
 *   PIE_TIMING_EVENTS HIP events around every piece of work.  Exact for every stream, but an event between
 *                     two kernels keeps them from running back to back: about 4 us per event, four events
 *                     per layer on the compute stream.
 *   PIE_TIMING_CLOCK  the kernels note their own first and last moment (device wall clock, atomic min / max
 *                     or words of their own that one kernel per step folds), and a one-thread kernel behind
 *                     each copy on the swap streams notes when it ended.  Nothing is put between the compute
 *                     stream's kernels.  A layer's compute time then runs from the start of its decode kernel
 *                     to the end of its last kernel; a copy's time from the moment everything it had to wait
 *                     for was done (the copy before it on its stream, the compute that frees its staging
 *                     region) to its end.
 * pie_get_layer_times and pie_get_stats read whichever the last step used. */
#define PIE_TIMING_OFF    0
#define PIE_TIMING_EVENTS 1
#define PIE_TIMING_CLOCK  2
int pie_set_timing(pie_pool* pool, int32_t mode);

/* Waits for everything the pool has enqueued on the streams it has seen. */
int pie_pool_sync(pie_pool* pool);

/* Summary of the last pie_step.  Its times are there when timing was on and the step has run: call after
 * pie_pool_sync.  Nothing is waited for: with monitoring by device clock, PIE_ESTATE while the pool's streams
 * still have work; with events, PIE_EHIP (hipErrorNotReady) from the event query. */
int pie_get_stats(pie_pool* pool, pie_stats* out);

/* Per-layer times in ms of the last pie_step; each array has n_layers entries (NULL to skip one).
 * t_attn: attention + reduction; t_kernel: the attention decode kernel alone; t_in / t_out: the
 * layer's prefetch / write-back; t_stall: how long the compute stream, free after the previous layer, still had
 * to wait for this layer's prefetch to finish (0 when the prefetch was hidden). */
int pie_get_layer_times(pie_pool* pool, float* t_attn, float* t_kernel, float* t_in, float* t_out, float* t_stall);

/* Reads and clears the device error flags after synchronising the pool. */
int pie_check_errors_sync(pie_pool* pool, uint32_t* out_flags);

/* ---- adaptive expansion (Section 3.4.2; growth conditions of Section 1) ---- */

/* A controller over integer levels k in [0, k_max]; host fraction = k / units.  Starts at k = 0. */
int pie_controller_create(int32_t units, int32_t k_max, pie_controller** out);
int pie_controller_destroy(pie_controller* ctl);

/* rho: growth keeps the predicted swap-in time within rho x compute; k_up good steps before growing;
 * k_down consecutive bad steps before shrinking; probe_period steps before a ceiling is retried;
 * plateau_eps: minimum relative throughput gain for a level to count as scaling; util_max: link
 * utilisation at or above which growth stops; stall_eps: summed waits above this share of summed compute
 * make a step bad. */
int pie_controller_config(pie_controller* ctl, double rho, int32_t k_up, int32_t k_down, int32_t probe_period,
                          double plateau_eps, double util_max, double stall_eps);

/* Feeds one decode step's measurements (per-layer arrays of n_layers entries, any consistent time unit)
 * and returns the level to use for the next step. */
int pie_controller_observe(pie_controller* ctl, int32_t n_layers, const double* t_attn, const double* t_in,
                           const double* t_stall, double link_util, double throughput, int32_t* out_level);

int pie_controller_level(pie_controller* ctl, int32_t* out_level, int32_t* out_ceiling /* -1 = none */);

/* Convenience: feeds the pool's last-step timings (timing on, step complete) to the controller. */
int pie_controller_update(pie_pool* pool, pie_controller* ctl, double throughput, float* out_host_fraction);

/* ---- layer-granular swapping (Section 3.2 mapping table; Section 3.3 protocol) ------------------------
 *
 * The paper's own unit of swapping is a whole layer's KV cache.  pie_layer_sched is its swapping control as
 * pure host logic: a mapping table logical layer -> (state, GPU layer slot, CPU layer slot), at most one
 * swap-in and one swap-out in flight, and at the beginning of each layer's computation
 *   - a swap-in of the hottest layer in CPU memory (the one accessed soonest) if the previous swap-in has
 *     completed and a GPU slot is free;
 *   - then a swap-out of the coldest layer on the GPU (the one whose next access is farthest: the layer that
 *     just finished) if the previous swap-out has completed, no GPU slot is free (a swap-out makes room for
 *     the next swap-in) and a CPU slot is free - unless every layer in CPU memory is colder still;
 *   - before that, the presence check: a layer that is not physically on the GPU is waited for, and brought
 *     back at once if it is not even on its way.
 * Moves update the table in two phases: starting a move names the destination slot (state MOVING_*);
 * pie_layer_sched_complete, called when the copy has finished, makes the layer present there and frees the
 * slot it left.  Layers are numbered 0 .. n_layers-1 and computed in that order, cyclically. */
typedef struct pie_layer_sched pie_layer_sched;
typedef struct pie_layer_pool pie_layer_pool;

#define PIE_LAYER_GPU        0
#define PIE_LAYER_HOST       1
#define PIE_LAYER_MOVING_OUT 2   /* GPU -> CPU copy in flight; both slots held */
#define PIE_LAYER_MOVING_IN  3

#define PIE_LAYER_WAIT_NONE 0
#define PIE_LAYER_WAIT_IN   1    /* wait for the swap-in in flight, report it complete, ask again */
#define PIE_LAYER_WAIT_OUT  2    /* likewise for the swap-out in flight */

#define PIE_LAYER_SKIP_NOT            0   /* the move was started */
#define PIE_LAYER_SKIP_BUSY           1   /* the previous move in that direction has not completed */
#define PIE_LAYER_SKIP_NO_SLOT        2   /* no free slot on the destination */
#define PIE_LAYER_SKIP_COLDER_ON_HOST 3   /* every layer in CPU memory is colder than the candidate */
#define PIE_LAYER_SKIP_NONE           4   /* no candidate */
#define PIE_LAYER_SKIP_ROOM_LEFT      5   /* a GPU slot is free: no layer has to leave */

typedef struct {
  int32_t state;       /* PIE_LAYER_* */
  int32_t gpu_slot;    /* -1 = none */
  int32_t host_slot;   /* -1 = none */
} pie_layer_entry;

typedef struct {
  int32_t wait;                                      /* PIE_LAYER_WAIT_*; when not NONE, gpu_slot is invalid */
  int32_t gpu_slot;                                  /* where the layer to compute lives */
  int32_t in_layer, in_gpu_slot, in_host_slot;       /* swap-in to start now; in_layer -1 = none */
  int32_t out_layer, out_gpu_slot, out_host_slot;    /* swap-out to start now; out_layer -1 = none */
  int32_t forced_in;                                 /* the swap-in is of the layer to compute itself */
  int32_t out_skipped, in_skipped;                   /* PIE_LAYER_SKIP_* (policy only) */
} pie_layer_action;

/* on_host: the n_on_host layers that start in CPU memory; the others start on the GPU.  Slots are handed
 * out lowest first, in layer order.  PIE_ENOMEM if the placement does not fit the slot counts. */
int pie_layer_sched_create(int32_t n_layers, int32_t n_gpu_slots, int32_t n_host_slots, int32_t n_on_host,
                           const int32_t* on_host, pie_layer_sched** out);
int pie_layer_sched_destroy(pie_layer_sched* s);
/* Phase two of the move in flight: which = 0 swap-in, 1 swap-out.  PIE_ESTATE if none is in flight. */
int pie_layer_sched_complete(pie_layer_sched* s, int32_t which);
/* The presence check for `layer`.  Either out->wait == NONE and out->gpu_slot says where the layer is, or
 * the caller must start the moves named in *out (a forced swap-in of the layer, or the swap-out of a victim
 * that makes room for it), wait as out->wait says, call pie_layer_sched_complete, and ask again. */
int pie_layer_sched_present(pie_layer_sched* s, int32_t layer, pie_layer_action* out);
/* The two checks at the beginning of `layer`'s computation (it must be present: PIE_ESTATE otherwise).  The
 * caller starts the moves named in *out. */
int pie_layer_sched_policy(pie_layer_sched* s, int32_t layer, pie_layer_action* out);
/* The mapping table: n_layers entries. */
int pie_layer_sched_table(pie_layer_sched* s, pie_layer_entry* out);
/* Adaptive expansion in layers (Section 3.4.2: start with every layer on the GPU, put more layers into
 * swapping while computation does not wait, move one back when it does): how many of the GPU layer slots
 * may be in use, 1 .. the count given at creation (PIE_EINVAL if the CPU slots cannot back it: the layers
 * that do not fit need one each, plus the two in flight).  Call between tokens.  Taking slots away retires free
 * slots, highest first, now or as completed swap-outs free them; while more are occupied than allowed the
 * swap-out exception is not applied (a layer has to leave).  Giving slots back re-enables retired ones,
 * lowest first; the next swap-ins fill them. */
int pie_layer_sched_set_gpu_slots(pie_layer_sched* s, int32_t n_gpu_slots);

/* pie_layer_pool runs that protocol on the GPU.  `pool` provides the GPU layer slots: a device pool created
 * with n_stage_blocks = n_host_blocks = 0 whose n_layers is the number of GPU layer slots; a layer's image is
 * its n_gpu_blocks blocks, contiguous, and block handles / tables are those of `pool`, the same for every
 * layer (base pointer per layer, offsets unchanged: Section 4.1).  h_pinned holds n_host_slots layer images
 * (pie_layer_pool_bytes_required).  The pool must outlive the layer pool.  Transfers are whole layers
 * through the copy engine; all ordering between streams is done on the host, so pie_layer_step paces the
 * host with the GPU, one layer ahead. */
typedef struct {
  int64_t n_steps, n_swap_in, n_swap_out, n_forced_in;
  uint64_t bytes_in, bytes_out;
  double  stall_ms;            /* host time spent waiting in presence checks */
} pie_layer_stats;

int pie_layer_pool_bytes_required(pie_pool* pool, int32_t n_host_slots, size_t* h_bytes);
int pie_layer_pool_create(pie_pool* pool, int32_t n_layers, int32_t n_host_slots, void* h_pinned, size_t h_bytes,
                          int32_t n_on_host, const int32_t* on_host, pie_layer_pool** out);
int pie_layer_pool_destroy(pie_layer_pool* lp);
/* One decode step over the n_layers logical layers, in order.  Arguments as pie_step, with
 * d_q_all / d_out_all [n_layers][batch][n_q_heads][head_dim] and d_k_new / d_v_new
 * [n_layers][batch][n_kv_heads][head_dim] indexed by logical layer. */
int pie_layer_step(pie_layer_pool* lp, const void* d_q_all, const void* d_k_new, const void* d_v_new,
                   const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_ctx_lens, int32_t batch,
                   void* d_out_all, void* compute_stream, void* swap_in_stream, void* swap_out_stream);
/* pie_layer_sched_set_gpu_slots for the pool's protocol.  Call between steps. */
int pie_layer_pool_set_gpu_slots(pie_layer_pool* lp, int32_t n_gpu_slots);
/* Waits for the moves in flight and completes them in the table. */
int pie_layer_pool_settle_sync(pie_layer_pool* lp);
/* Where a logical layer's image is now: *out_where = PIE_WHERE_*, *out_ptr its device or host address.
 * PIE_ESTATE while the layer is in flight. */
int pie_layer_pool_address(pie_layer_pool* lp, int32_t layer, int32_t* out_where, void** out_ptr);
int pie_layer_pool_table(pie_layer_pool* lp, pie_layer_entry* out);
int pie_layer_pool_stats(pie_layer_pool* lp, pie_layer_stats* out);

/* ---- layer caches that grow and shrink (Section 3.1: a / (n - m) per layer; Section 4.1: block manager) ----
 *
 * With m of n layers' caches kept in CPU memory, the GPU memory they leave goes to the layers that stay.  The
 * paper reallocates a layer's cache as one piece when it is swapped back in; here the GPU memory is N chunks
 * of chunk_blocks block slots, and a layer's cache is any list of chunks: block h of the layer lives in slot
 * chunk[h / chunk_blocks] * chunk_blocks + h % chunk_blocks of that memory.  A resident layer is given more
 * chunks where it is; a layer travels as one copy-engine transfer per chunk.
 *
 * pie_chunk_book is the bookkeeping as pure host logic.  Every layer starts resident with N / n chunks (layer
 * j: chunks j N/n ...).  The target per layer is min(max_chunks_per_layer, N / (n - m)).  Free chunks go to
 * resident layers below the target, lowest layer first, except what the GPU layer slots still to be filled
 * will need; a layer entering the GPU takes the lowest free chunks, up to the target.  What is visible to a
 * scheduler (chunks per layer usable in every layer) is the smallest list among the resident layers: growth
 * shows when the reallocation is complete; a shrink lowers it at once. */
typedef struct pie_chunk_book pie_chunk_book;
int pie_chunk_book_create(int32_t n_layers, int32_t n_chunks, int32_t max_chunks_per_layer, pie_chunk_book** out);
int pie_chunk_book_destroy(pie_chunk_book* book);
/* Asks for m layers in CPU memory.  chunks_in_use: chunks of a layer's cache that still hold live blocks.
 * PIE_ESTATE: the caches would have to shrink below that; what is visible has been lowered all the same
 * (hidden first), nothing else has changed; ask again when the blocks above have been given up. */
int pie_chunk_book_set_layers_on_cpu(pie_chunk_book* book, int32_t m, int32_t chunks_in_use);
/* The layer's swap-out has completed: its chunks are free (and may go to resident layers at once).  n_carried:
 * how many of its chunks it took along - those that hold live blocks; -1 = all. */
int pie_chunk_book_left_gpu(pie_chunk_book* book, int32_t layer, int32_t n_carried);
/* The layer's swap-in starts: it takes chunks; *out_n_data = how many of them its data fills.  PIE_ENOMEM if
 * fewer chunks are free than it carries or than are visible. */
int pie_chunk_book_enters_gpu(pie_chunk_book* book, int32_t layer, int32_t* out_n_data);
/* out_chunks needs room for max_chunks_per_layer entries; any out pointer may be NULL. */
int pie_chunk_book_layer(pie_chunk_book* book, int32_t layer, int32_t* out_resident, int32_t* out_n_data,
                         int32_t* out_n_chunks, int32_t* out_chunks);
int pie_chunk_book_capacity(pie_chunk_book* book, int32_t* out_visible, int32_t* out_target, int32_t* out_free,
                            int32_t* out_layers_on_cpu);

/* pie_elastic_pool runs the layer-granular protocol (pie_layer_sched) over such caches on the GPU.  `pool`: a
 * device pool with n_stage_blocks = n_host_blocks = 0 whose n_layers are the logical layers and whose
 * n_gpu_blocks (a multiple of chunk_blocks) is a layer's cache while everything is on the GPU; its memory is
 * the N = n_layers * n_gpu_blocks / chunk_blocks chunks.  Block tables hold block indices of a layer's cache
 * (the same in every layer), below the visible capacity.  d_work (device, pie_elastic_bytes_required) holds
 * the layers' block maps; h_pinned holds n_host_slots layer images of max_chunks_per_layer chunks.  The pool
 * must outlive the elastic pool; its own block allocator and swaps are not used.  All ordering between
 * streams is done on the host, as in pie_layer_step. */
typedef struct pie_elastic_pool pie_elastic_pool;
int pie_elastic_bytes_required(pie_pool* pool, int32_t chunk_blocks, int32_t max_chunks_per_layer,
                               int32_t n_host_slots, size_t* d_bytes, size_t* h_bytes);
int pie_elastic_create(pie_pool* pool, int32_t chunk_blocks, int32_t max_chunks_per_layer, int32_t n_host_slots,
                       void* d_work, size_t d_bytes, void* h_pinned, size_t h_bytes, pie_elastic_pool** out);
int pie_elastic_destroy(pie_elastic_pool* ep);
/* Between steps: asks for m layers in CPU memory (needs m + 2 host slots).  blocks_in_use_end: highest live
 * block index + 1.  Completes the moves in flight first.  PIE_ESTATE as pie_chunk_book_set_layers_on_cpu.  The
 * layers then leave (or return) through the protocol during the following steps. */
int pie_elastic_set_layers_on_cpu(pie_elastic_pool* ep, int32_t m, int32_t blocks_in_use_end, void* compute_stream);
/* Tells the pool the highest live block index + 1 (-1: unknown, the default): a layer that leaves the GPU
 * takes along only the chunks below it.  Blocks above must hold nothing that is still needed. */
int pie_elastic_set_live_blocks(pie_elastic_pool* ep, int32_t blocks_in_use_end);
/* Between steps: copies block src[i] of a layer's cache to block dst[i], in every layer, wherever the layer is
 * (on the GPU by a kernel on compute_stream, in CPU memory inside its image).  For a scheduler that wants
 * live blocks out of the part of the caches a shrink will take away.  Each block moves once, targets are not
 * themselves moved, and every resident layer must hold both ends (PIE_ESTATE otherwise).  Completes the
 * moves in flight first.  The caller updates its block tables. */
int pie_elastic_move_blocks(pie_elastic_pool* ep, int32_t n, const int32_t* src, const int32_t* dst,
                            void* compute_stream);
/* Blocks per layer a scheduler may use now, what they will be when the reallocation is complete, and m. */
int pie_elastic_capacity(pie_elastic_pool* ep, int32_t* out_visible_blocks, int32_t* out_target_blocks,
                         int32_t* out_layers_on_cpu);
/* Blocks per layer the caches will have with m layers kept in CPU memory, once that reallocation is complete:
 * min(max_chunks_per_layer, N / (n - m)) chunks (Section 3.1's a / (n - m), in whole chunks).  For a scheduler
 * that must know what fits below a size before it asks for it.  PIE_EINVAL unless 0 <= m < n_layers. */
int pie_elastic_blocks_for(pie_elastic_pool* ep, int32_t m, int32_t* out_blocks);
/* One decode step over the logical layers, in order; arguments as pie_layer_step. */
int pie_elastic_step(pie_elastic_pool* ep, const void* d_q_all, const void* d_k_new, const void* d_v_new,
                     const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_ctx_lens, int32_t batch,
                     void* d_out_all, void* compute_stream, void* swap_in_stream, void* swap_out_stream);
int pie_elastic_settle_sync(pie_elastic_pool* ep, void* compute_stream);
/* Where a layer is: PIE_WHERE_GPU with its chunk list (out_chunks: room for max_chunks_per_layer), or
 * PIE_WHERE_HOST with the address of its image (*out_n_chunks chunks of data).  PIE_ESTATE while in flight. */
int pie_elastic_layer(pie_elastic_pool* ep, int32_t layer, int32_t* out_where, int32_t* out_n_chunks,
                      int32_t* out_chunks, void** out_host_ptr);
int pie_elastic_table(pie_elastic_pool* ep, pie_layer_entry* out);
int pie_elastic_stats(pie_elastic_pool* ep, pie_layer_stats* out);

/* ---- diagnostics -------------------------------------------------------------- */
int pie_last_hip_error(void);            /* hipError_t of the last PIE_EHIP on this thread, 0 if none */
const char* pie_strerror(int code);      /* static string for a PIE_* code */
int pie_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PIE_H */
