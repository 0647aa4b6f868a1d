// Pool: block allocator, residency (the mapping table), staging regions, swaps, and the per-layer
// pipeline.  Host logic only; kernels live in pie_kernels.hip.
//
// Paper passages: Section 3.2 (mapping table, two-phase update, presence check), Section 3.3 (prefetch
// behind the current layer), Section 4.1 (block manager, base pointer + offset addressing).

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "pie_internal.h"

namespace pie {

thread_local int g_last_hip_error = 0;

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int elem_bytes_of(int32_t dtype) {
  switch (dtype) {
    case PIE_DTYPE_F32: return 4;
    case PIE_DTYPE_F16: return 2;
    case PIE_DTYPE_BF16: return 2;
    default: return 0;
  }
}

static bool config_ok(const pie_config* c) {
  if (!c) return false;
  if (c->n_layers <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 || c->block_tokens <= 0)
    return false;
  if (c->n_q_heads % c->n_kv_heads) return false;
  if (c->n_gpu_blocks < 0 || c->n_stage_blocks < 0 || c->n_host_blocks < 0) return false;
  if (c->max_batch < 0 || c->max_blocks_per_seq < 0) return false;
  if (!elem_bytes_of(c->dtype)) return false;
  if ((int64_t)c->n_gpu_blocks + c->n_host_blocks > (int64_t)1 << 30) return false;
  return true;
}

struct Layout {
  size_t block_bytes, d_layer_stride, h_layer_stride;
  size_t off_map0, off_map1, off_ws, off_plan, off_err, off_clock, d_total, h_total;
  size_t ws_floats;
};

static Layout layout_of(const pie_config& c) {
  Layout l;
  const int e = elem_bytes_of(c.dtype);
  l.block_bytes = (size_t)2 * c.n_kv_heads * c.block_tokens * c.head_dim * e;
  l.d_layer_stride = ((size_t)c.n_gpu_blocks + 2 * (size_t)c.n_stage_blocks) * l.block_bytes;
  l.h_layer_stride = (size_t)c.n_host_blocks * l.block_bytes;
  const size_t n_handles = (size_t)c.n_gpu_blocks + c.n_host_blocks;
  size_t off = align_up(l.d_layer_stride * c.n_layers, kAlign);
  l.off_map0 = off; off = align_up(off + n_handles * 4, kAlign);
  l.off_map1 = off; off = align_up(off + n_handles * 4, kAlign);
  l.ws_floats = attn_workspace_floats(c);
  l.off_ws = off; off = align_up(off + l.ws_floats * 4, kAlign);
  l.off_plan = off; off = align_up(off + attn_plan_ints(c) * 4, kAlign);
  l.off_err = off; off += kAlign;
  l.off_clock = off;
  off = align_up(off + (((size_t)c.n_layers + 1) * kClockRow + (size_t)c.n_layers * kClockWgs * 2) * 8, kAlign);
  l.d_total = off;
  l.h_total = l.h_layer_stride * c.n_layers;
  return l;
}

int note_stream(pie_pool* p, hipStream_t s) {
  for (hipStream_t t : p->streams_seen)
    if (t == s) return PIE_OK;
  p->streams_seen.push_back(s);
  return PIE_OK;
}

// ---- the submit thread ------------------------------------------------------------------------------------
static int step_body(pie_pool* p, const StepJob& j);

static void submit_loop(pie_pool* p) {
  (void)hipSetDevice(p->device_id);
  std::unique_lock<std::mutex> lock(p->submit_mutex);
  for (;;) {
    p->submit_wake.wait(lock, [p] { return p->submit_stop || !p->submit_jobs.empty(); });
    if (p->submit_jobs.empty()) return;                       // asked to stop, nothing left
    StepJob job = std::move(p->submit_jobs.front());
    p->submit_jobs.pop_front();
    p->submit_busy = true;
    lock.unlock();
    g_last_hip_error = 0;
    const int rc = step_body(p, job);
    lock.lock();
    if (rc && !p->submit_rc) {
      p->submit_rc = rc;
      p->submit_hip = g_last_hip_error;
    }
    p->submit_busy = false;
    if (p->submit_jobs.empty()) p->submit_idle.notify_all();
  }
}

int submit_drain(pie_pool* p) {
  if (!p->submitter.joinable()) return PIE_OK;
  std::unique_lock<std::mutex> lock(p->submit_mutex);
  p->submit_idle.wait(lock, [p] { return p->submit_jobs.empty() && !p->submit_busy; });
  const int rc = p->submit_rc;
  if (rc) g_last_hip_error = p->submit_hip;
  p->submit_rc = p->submit_hip = 0;
  return rc;
}

// Every call but pie_step first lets the submit thread finish what it was given: one thread at a time touches
// the pool's state.
#define PIE_DRAIN(p)                       \
  do {                                     \
    const int drc_ = submit_drain(p);      \
    if (drc_) return drc_;                 \
  } while (0)

void map_set(pie_pool* p, int region, int32_t handle, int32_t slot) {
  if (p->map_mirror[region][handle] == slot) return;
  p->map_mirror[region][handle] = slot;
  if (!p->map_dirty_flag[region][handle]) {
    p->map_dirty_flag[region][handle] = 1;
    p->map_dirty[region].push_back(handle);
  }
}

// Sends stale map entries to the device on stream s, as by-value kernel arguments so that neither a
// staging buffer nor a later change of the mirror can race with the copy.
int flush_map(pie_pool* p, hipStream_t s) {
  if (!p->device) return PIE_OK;
  for (int r = 0; r < 2; ++r) {
    std::vector<int32_t>& dirty = p->map_dirty[r];
    if (dirty.empty()) continue;
    MapPatch patch;
    size_t i = 0;
    while (i < dirty.size()) {
      patch.n = 0;
      while (i < dirty.size() && patch.n < kMapPatchPairs) {
        const int32_t h = dirty[i++];
        patch.handle[patch.n] = h;
        patch.slot[patch.n] = p->map_mirror[r][h];
        p->map_dirty_flag[r][h] = 0;
        ++patch.n;
      }
      int rc = launch_map_patch(p->d_map[r], patch, s);
      if (rc) return rc;
    }
    dirty.clear();
  }
  return PIE_OK;
}

static int check_handles(const pie_pool* p, int32_t n, const int32_t* handles, int need_where,
                         std::vector<uint8_t>& seen) {
  if (n < 0 || (n > 0 && !handles)) return PIE_EINVAL;
  seen.assign(p->n_handles, 0);
  for (int32_t i = 0; i < n; ++i) {
    const int32_t h = handles[i];
    if (h < 0 || h >= p->n_handles) return PIE_EINVAL;
  }
  for (int32_t i = 0; i < n; ++i) {
    const int32_t h = handles[i];
    if (p->home[h].where < 0 || seen[h]) return PIE_ESTATE;
    if (need_where >= 0 && p->home[h].where != need_where) return PIE_ESTATE;
    seen[h] = 1;
  }
  return PIE_OK;
}

static void drop_staged(pie_pool* p, int32_t h) {
  for (int r = 0; r < 2; ++r) {
    if (p->stage_rank[r][h] >= 0) {
      p->stage_list[r][p->stage_rank[r][h]] = -1;
      p->stage_rank[r][h] = -1;
    }
  }
}

// A list of (src slot -> dst slot) block copies of one layer, cut into contiguous runs, and the way it
// will be moved: the copy engine when the runs are few and long, the gather / scatter kernel otherwise.
struct CopyPlan {
  struct Run { int32_t src, dst, len; };
  std::vector<Run> runs;
  int path = PIE_SWAP_KERNEL;
};

static CopyPlan plan_copy(const pie_pool* p, const std::vector<int32_t>& src, const std::vector<int32_t>& dst) {
  CopyPlan cp;
  const size_t n = src.size();
  for (size_t i = 0; i < n; ++i) {
    if (!cp.runs.empty() && cp.runs.back().src + cp.runs.back().len == src[i] &&
        cp.runs.back().dst + cp.runs.back().len == dst[i])
      ++cp.runs.back().len;
    else
      cp.runs.push_back({src[i], dst[i], 1});
  }
  cp.path = p->swap_path;
  if (cp.path == PIE_SWAP_AUTO && n) {
    // Measured on this machine: a copy-engine transfer costs about 16 us per call and then moves 56 GB/s with
    // no compute unit involved; the gather kernel moves about 2.6 GB/s per workgroup, 41 GB/s at most, after
    // about 12 us.  The copy engine is taken unless the kernel is clearly faster for this list.
    const double bytes = (double)n * (double)p->block_bytes;
    const double dma_us = 16.0 * (double)cp.runs.size() + bytes / 56.0e3;
    const double kernel_us = 12.0 + bytes / (std::min(41.0, 2.6 * p->swap_wgs) * 1.0e3);
    cp.path = dma_us <= 1.1 * kernel_us ? PIE_SWAP_DMA : PIE_SWAP_KERNEL;
  }
  return cp;
}

// kind: 0 host->device, 1 device->host.
static int copy_blocks(pie_pool* p, int kind, int32_t layer, const std::vector<int32_t>& src,
                       const std::vector<int32_t>& dst, const CopyPlan& cp, hipStream_t s) {
  const size_t n = src.size();
  if (!n) return PIE_OK;
  if (cp.path == PIE_SWAP_DMA) {
    for (const CopyPlan::Run& r : cp.runs) {
      const size_t bytes = (size_t)r.len * p->block_bytes;
      if (kind == 0)
        PIE_HIP(hipMemcpyAsync(d_block(p, layer, r.dst), h_block(p, layer, r.src), bytes, hipMemcpyHostToDevice, s));
      else
        PIE_HIP(hipMemcpyAsync(h_block(p, layer, r.dst), d_block(p, layer, r.src), bytes, hipMemcpyDeviceToHost, s));
    }
    return PIE_OK;
  }
  char* dst_base = kind == 0 ? p->d_kv + (size_t)layer * p->d_layer_stride
                             : p->h_kv_dev + (size_t)layer * p->h_layer_stride;
  const char* src_base = kind == 0 ? p->h_kv_dev + (size_t)layer * p->h_layer_stride
                                   : p->d_kv + (size_t)layer * p->d_layer_stride;
  SwapPairs pairs;
  size_t i = 0;
  while (i < n) {
    pairs.n = 0;
    while (i < n && pairs.n < kSwapPairs) {
      pairs.src[pairs.n] = src[i];
      pairs.dst[pairs.n] = dst[i];
      ++pairs.n;
      ++i;
    }
    int rc = launch_swap_copy(dst_base, src_base, p->block_bytes, pairs, p->swap_wgs, s, p->swap_shape,
                              n * p->block_bytes);
    if (rc) return rc;
  }
  return PIE_OK;
}

// Orders stream s after event ev.  Kernels wait on the device.  A copy-engine transfer whose stream has an
// unfinished wait on another stream's event makes the runtime hold the host inside the copy call, for an
// unpredictable time; so for those the host waits for the event itself, and the copy is then enqueued on a
// stream with nothing pending.
static int order_after(hipStream_t s, hipEvent_t ev, bool recorded, bool on_host) {
  if (!recorded) return PIE_OK;
  if (on_host)
    PIE_HIP(hipEventSynchronize(ev));
  else
    PIE_HIP(hipStreamWaitEvent(s, ev, 0));
  return PIE_OK;
}

static int wait_if(hipStream_t s, hipEvent_t ev, bool recorded) {
  if (recorded) PIE_HIP(hipStreamWaitEvent(s, ev, 0));
  return PIE_OK;
}

// ---- internals of the public swap / compute calls (also used by pie_step) ------------------------------

// Phase one of a swap-in: publish where the copies of the listed blocks will be (staging slot = rank).
static void publish_stage_list(pie_pool* p, int r, int32_t n, const int32_t* handles) {
  bool same = (int32_t)p->stage_list[r].size() == n;
  for (int32_t i = 0; same && i < n; ++i) same = p->stage_list[r][i] == handles[i];
  if (same) return;
  for (int32_t h : p->stage_list[r])
    if (h >= 0) {
      p->stage_rank[r][h] = -1;
      map_set(p, r, h, -1);
    }
  p->stage_list[r].assign(handles, handles + n);
  for (int32_t i = 0; i < n; ++i) {
    p->stage_rank[r][handles[i]] = i;
    map_set(p, r, handles[i], stage_slot(p, r, i));
  }
}

// The new token's rows for the tail blocks that a prefetch brings in: written into the staged copies on the
// write-back stream once the copy has arrived, so that the write-back takes them home.  (Not on the swap-in
// stream behind the copy: the next layer's copy on that stream would wait for the kernel, and the link would
// idle between any two transfers for as long as a kernel behind a copy-engine transfer takes to start.)
struct StagedAppend {
  const void* d_k;
  const void* d_v;
  const int32_t* d_table;
  const int32_t* d_ctx;
  int32_t max_blocks, batch;
};

// A moment on a stream noted for the step's timing: by an event, by a device-clock stamp, or not at all.
struct Mark {
  hipEvent_t ev = nullptr;
  unsigned long long* clk = nullptr;
};

static int note(const Mark& m, hipStream_t s) {
  if (m.ev) PIE_HIP(hipEventRecord(m.ev, s));
  if (m.clk) return launch_stamp(m.clk, s);
  return PIE_OK;
}

// skip_copy: the region already holds exactly these blocks of this layer (brought in behind the previous
// step's last layer); only the ordering and the completion event are enqueued.
static int swap_in_impl(pie_pool* p, int32_t layer, int32_t n, const int32_t* handles, hipStream_t s,
                        bool validated, const Mark& t0, const Mark& t1, bool skip_copy = false) {
  const int r = layer & 1;
  p->pre_valid = false;
  if (!validated) {
    if (layer < 0 || layer >= p->cfg.n_layers) return PIE_EINVAL;
    if (n < 0 || (n > 0 && !handles)) return PIE_EINVAL;
    if (n > p->cfg.n_stage_blocks) return PIE_ENOMEM;
    std::vector<uint8_t> seen;
    int rc = check_handles(p, n, handles, PIE_WHERE_HOST, seen);
    if (rc) return rc;
  }
  if (!p->device) return PIE_ESTATE;
  note_stream(p, s);
  publish_stage_list(p, r, n, handles);
  p->region_layer[r] = layer;
  std::vector<int32_t> src(n), dst(n);
  for (int32_t i = 0; i < n; ++i) {
    src[i] = p->home[handles[i]].slot;
    dst[i] = stage_slot(p, r, i);
  }
  const CopyPlan cp = plan_copy(p, src, dst);
  // (also when the copy itself is skipped: a wait enqueued on this stream would make the copy-engine
  // transfers that follow on it block the host)
  const bool on_host = n > 0 && cp.path == PIE_SWAP_DMA && !p->dma_stream_order;
  p->in_on_host[r] = on_host;
  // the region may still be read by compute or written back
  int rc;
  if ((rc = order_after(s, p->ev_read[r], p->ev_read_rec[r], on_host))) return rc;
  if ((rc = order_after(s, p->ev_out[r], p->ev_out_rec[r], on_host))) return rc;
  if ((rc = order_after(s, p->ev_migrate, p->ev_migrate_rec, on_host))) return rc;
  if (!skip_copy) {
    if ((rc = note(t0, s))) return rc;
    if ((rc = copy_blocks(p, 0, layer, src, dst, cp, s))) return rc;
    if ((rc = note(t1, s))) return rc;
  }
  // phase two happens when this event completes
  PIE_HIP(hipEventRecord(p->ev_in[r], s));
  p->ev_in_rec[r] = true;
  if (!skip_copy) p->bytes_in += (uint64_t)n * p->block_bytes;
  return PIE_OK;
}

// after_read: the copies wait for the layer's computation as well.  A caller whose computation only reads the
// staged blocks (pie_step: the new token's rows are appended by `job`, below) passes false, and the blocks go
// home as soon as they are staged and appended to.
// job: the newest token's rows, to be written into the staged tail blocks first (on this stream, ahead of the
// copies that take the blocks home; the stream must have seen the map updates the append reads).
static int swap_out_impl(pie_pool* p, int32_t layer, int32_t n, const int32_t* handles, hipStream_t s,
                         const Mark& t0, const Mark& t1, bool after_read = true, const StagedAppend* job = nullptr) {
  if (layer < 0 || layer >= p->cfg.n_layers) return PIE_EINVAL;
  std::vector<uint8_t> seen;
  int rc = check_handles(p, n, handles, PIE_WHERE_HOST, seen);
  if (rc) return rc;
  const int r = layer & 1;
  if (n > 0 && p->region_layer[r] != layer) return PIE_ESTATE;
  for (int32_t i = 0; i < n; ++i)
    if (p->stage_rank[r][handles[i]] < 0) return PIE_ESTATE;
  if (!p->device) return PIE_ESTATE;
  note_stream(p, s);
  std::vector<int32_t> src(n), dst(n);
  for (int32_t i = 0; i < n; ++i) {
    src[i] = stage_slot(p, r, p->stage_rank[r][handles[i]]);
    dst[i] = p->home[handles[i]].slot;
  }
  const CopyPlan cp = plan_copy(p, src, dst);
  const bool on_host = n > 0 && cp.path == PIE_SWAP_DMA && !p->dma_stream_order;
  if ((rc = order_after(s, p->ev_in[r], p->ev_in_rec[r], on_host))) return rc;
  if (after_read && (rc = order_after(s, p->ev_read[r], p->ev_read_rec[r], on_host))) return rc;
  if (job && (rc = launch_kv_append(p, layer, 1, job->d_k, job->d_v, job->d_table, job->max_blocks, job->d_ctx,
                                    job->batch, kAppendStaged, s)))
    return rc;
  if ((rc = note(t0, s))) return rc;
  if ((rc = copy_blocks(p, 1, layer, src, dst, cp, s))) return rc;
  if ((rc = note(t1, s))) return rc;
  PIE_HIP(hipEventRecord(p->ev_out[r], s));
  p->ev_out_rec[r] = true;
  p->bytes_out += (uint64_t)n * p->block_bytes;
  return PIE_OK;
}

// Everything a compute-stream kernel of `layer` must wait for: the presence check.
static int compute_prologue(pie_pool* p, int32_t layer, hipStream_t s, bool* stage_valid) {
  const int r = layer & 1;
  note_stream(p, s);
  int rc;
  if ((rc = wait_if(s, p->ev_migrate, p->ev_migrate_rec))) return rc;
  *stage_valid = p->region_layer[r] == layer;
  if (*stage_valid && (rc = wait_if(s, p->ev_in[r], p->ev_in_rec[r]))) return rc;
  return flush_map(p, s);
}

static int compute_epilogue(pie_pool* p, int32_t layer, hipStream_t s) {
  const int r = layer & 1;
  PIE_HIP(hipEventRecord(p->ev_read[r], s));
  p->ev_read_rec[r] = true;
  PIE_HIP(hipEventRecord(p->ev_compute, s));
  p->ev_compute_rec = true;
  return PIE_OK;
}

static int check_batch_args(const pie_pool* p, int32_t layer, const void* a, const int32_t* table,
                            int32_t max_blocks, const int32_t* ctx, int32_t batch) {
  if (layer < 0 || layer >= p->cfg.n_layers) return PIE_EINVAL;
  if (batch < 0 || max_blocks < 0) return PIE_EINVAL;
  if (batch > 0 && (!a || !table || !ctx)) return PIE_EINVAL;
  if (batch > p->cfg.max_batch || max_blocks > p->cfg.max_blocks_per_seq) return PIE_EINVAL;
  return PIE_OK;
}

}  // namespace pie

using namespace pie;

extern "C" {

int pie_pool_bytes_required(const pie_config* cfg, size_t* d_bytes, size_t* h_bytes) {
  if (!config_ok(cfg)) return PIE_EINVAL;
  const Layout l = layout_of(*cfg);
  if (d_bytes) *d_bytes = l.d_total;
  if (h_bytes) *h_bytes = l.h_total;
  return PIE_OK;
}

int pie_pool_init(const pie_config* cfg, void* d_base, size_t d_bytes, void* h_pinned_base, size_t h_bytes,
                  pie_pool** out) {
  if (!out || !config_ok(cfg)) return PIE_EINVAL;
  *out = nullptr;
  const Layout l = layout_of(*cfg);
  const bool device = d_base != nullptr;
  if (device) {
    if (!attn_config_supported(*cfg)) return PIE_EINVAL;
    if ((uintptr_t)d_base % kAlign) return PIE_EINVAL;
    if (d_bytes < l.d_total) return PIE_ENOMEM;
    if (cfg->n_host_blocks > 0) {
      if (!h_pinned_base) return PIE_EINVAL;
      if ((uintptr_t)h_pinned_base % 16) return PIE_EINVAL;
      if (h_bytes < l.h_total) return PIE_ENOMEM;
    }
  }
  pie_pool* p = new (std::nothrow) pie_pool();
  if (!p) return PIE_ENOMEM;
  p->cfg = *cfg;
  p->device = device;
  p->n_handles = cfg->n_gpu_blocks + cfg->n_host_blocks;
  p->elem_bytes = elem_bytes_of(cfg->dtype);
  p->block_bytes = l.block_bytes;
  p->d_layer_stride = l.d_layer_stride;
  p->h_layer_stride = l.h_layer_stride;
  const float scale = cfg->softmax_scale != 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  p->scale_log2e = scale * 1.4426950408889634f;
  for (int32_t h = 0; h < p->n_handles; ++h) p->free_handles.insert(h);
  for (int32_t s = 0; s < cfg->n_gpu_blocks; ++s) p->free_slots[0].insert(s);
  for (int32_t s = 0; s < cfg->n_host_blocks; ++s) p->free_slots[1].insert(s);
  p->home.assign(p->n_handles, Home());
  for (int r = 0; r < 2; ++r) {
    p->stage_rank[r].assign(p->n_handles, -1);
    p->map_mirror[r].assign(p->n_handles, -1);
    p->map_dirty_flag[r].assign(p->n_handles, 0);
  }
  p->h_kv = (char*)h_pinned_base;
  // tuning hooks for experiments; the defaults are what the benchmarks use
  if (const char* e = std::getenv("PIE_ATTN_PART")) { const int v = std::atoi(e); if (v >= 0) p->attn_partition = v; }
  if (const char* e = std::getenv("PIE_DMA_STREAM_ORDER")) p->dma_stream_order = std::atoi(e) != 0;
  if (const char* e = std::getenv("PIE_SWAP_SHAPE")) { const int v = std::atoi(e); if (v > 0) p->swap_shape = v; }
  if (device) {
    char* base = (char*)d_base;
    p->d_kv = base;
    p->d_map[0] = (int32_t*)(base + l.off_map0);
    p->d_map[1] = (int32_t*)(base + l.off_map1);
    p->d_ws = (float*)(base + l.off_ws);
    p->ws_floats = l.ws_floats;
    p->d_plan = (int32_t*)(base + l.off_plan);
    p->d_err = (uint32_t*)(base + l.off_err);
    p->d_clock = (unsigned long long*)(base + l.off_clock);
    int rc = PIE_OK;
    {
      int dev = 0, n_cu = 0;
      if (hipGetDevice(&dev) == hipSuccess) p->device_id = dev;
      if (hipGetDevice(&dev) == hipSuccess &&
          hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n_cu > 0)
        p->n_cu = n_cu;
      else
        (void)hipGetLastError();
      int khz = 0;
      if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && khz > 0)
        p->wall_clock_khz = khz;
      else
        (void)hipGetLastError();
    }
    auto fail = [&](int code) { pie_pool_destroy(p); return code; };
    {
      char* static_scratch = nullptr;               // the device's copy of the library's static scratch array
      if ((rc = attn_static_scratch(&static_scratch))) return fail(rc);
    }
    if (cfg->n_host_blocks > 0) {
      void* dev_ptr = nullptr;
      hipError_t e = hipHostGetDevicePointer(&dev_ptr, h_pinned_base, 0);
      if (e != hipSuccess) { g_last_hip_error = (int)e; (void)hipGetLastError(); return fail(PIE_EHIP); }
      p->h_kv_dev = (char*)dev_ptr;
    }
    hipEvent_t* evs[] = {&p->ev_in[0], &p->ev_in[1], &p->ev_read[0], &p->ev_read[1], &p->ev_out[0], &p->ev_out[1],
                         &p->ev_compute, &p->ev_migrate, &p->ev_map, &p->ev_append};
    for (hipEvent_t* e : evs) {
      hipError_t err = hipEventCreateWithFlags(e, hipEventDisableTiming);
      if (err != hipSuccess) { g_last_hip_error = (int)err; (void)hipGetLastError(); return fail(PIE_EHIP); }
    }
    hipError_t err = hipEventCreate(&p->ev_step_start);
    if (err != hipSuccess) { g_last_hip_error = (int)err; return fail(PIE_EHIP); }
    for (hipEvent_t* e : {&p->ev_pre_end[0], &p->ev_pre_end[1]}) {
      err = hipEventCreate(e);
      if (err != hipSuccess) { g_last_hip_error = (int)err; return fail(PIE_EHIP); }
    }
    p->lev.resize(cfg->n_layers);
    for (auto& le : p->lev) {
      hipEvent_t* tev[] = {&le.attn_start, &le.attn_end, &le.k_start, &le.k_end,
                           &le.in_start,   &le.in_end,   &le.out_start, &le.out_end};
      for (hipEvent_t* e : tev) {
        *e = nullptr;
        err = hipEventCreate(e);
        if (err != hipSuccess) { g_last_hip_error = (int)err; return fail(PIE_EHIP); }
      }
    }
    // maps start empty, error flags clear (default stream; synchronised before returning)
    if ((rc = launch_map_fill(p->d_map[0], p->n_handles, -1, nullptr))) return fail(rc);
    if ((rc = launch_map_fill(p->d_map[1], p->n_handles, -1, nullptr))) return fail(rc);
    if ((rc = launch_zero_u32(p->d_err, kAlign / 4, nullptr))) return fail(rc);
    if ((rc = launch_zero_u32((uint32_t*)p->d_clock, (cfg->n_layers + 1) * kClockRow * 2, nullptr))) return fail(rc);
    err = hipStreamSynchronize(nullptr);
    if (err != hipSuccess) { g_last_hip_error = (int)err; return fail(PIE_EHIP); }
  }
  *out = p;
  return PIE_OK;
}

int pie_pool_sync(pie_pool* p) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  if (!p->device) return PIE_OK;
  for (hipStream_t s : p->streams_seen) PIE_HIP(hipStreamSynchronize(s));
  return PIE_OK;
}

int pie_pool_destroy(pie_pool* p) {
  if (!p) return PIE_EINVAL;
  if (p->submitter.joinable()) {
    (void)submit_drain(p);
    {
      std::lock_guard<std::mutex> g(p->submit_mutex);
      p->submit_stop = true;
    }
    p->submit_wake.notify_all();
    p->submitter.join();
  }
  if (p->device) {
    for (hipStream_t s : p->streams_seen) (void)hipStreamSynchronize(s);
    hipEvent_t evs[] = {p->ev_in[0], p->ev_in[1], p->ev_read[0], p->ev_read[1], p->ev_out[0], p->ev_out[1],
                        p->ev_compute, p->ev_migrate, p->ev_map, p->ev_step_start, p->ev_pre_end[0], p->ev_pre_end[1],
                        p->ev_append};
    for (hipEvent_t e : evs)
      if (e) (void)hipEventDestroy(e);
    for (auto& le : p->lev) {
      hipEvent_t tev[] = {le.attn_start, le.attn_end, le.k_start, le.k_end,
                          le.in_start,   le.in_end,   le.out_start, le.out_end};
      for (hipEvent_t e : tev)
        if (e) (void)hipEventDestroy(e);
    }
  }
  delete p;
  return PIE_OK;
}

int pie_block_alloc(pie_pool* p, int32_t where, int32_t n, int32_t* out_handles) {
  if (!p || (where != PIE_WHERE_GPU && where != PIE_WHERE_HOST) || n < 0 || (n > 0 && !out_handles))
    return PIE_EINVAL;
  PIE_DRAIN(p);
  if ((size_t)n > p->free_slots[where].size() || (size_t)n > p->free_handles.size()) return PIE_ENOMEM;
  for (int32_t i = 0; i < n; ++i) {
    const int32_t h = *p->free_handles.begin();
    const int32_t s = *p->free_slots[where].begin();
    p->free_handles.erase(p->free_handles.begin());
    p->free_slots[where].erase(p->free_slots[where].begin());
    p->home[h] = {where, s};
    out_handles[i] = h;
    const int32_t dev_slot = where == PIE_WHERE_GPU ? s : -1;
    map_set(p, 0, h, dev_slot);
    map_set(p, 1, h, dev_slot);
  }
  p->n_in_use[where] += n;
  return PIE_OK;
}

int pie_block_free(pie_pool* p, int32_t n, const int32_t* handles) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  std::vector<uint8_t> seen;
  int rc = check_handles(p, n, handles, -1, seen);
  if (rc) return rc;
  for (int32_t i = 0; i < n; ++i) {
    const int32_t h = handles[i];
    const Home hm = p->home[h];
    p->free_slots[hm.where].insert(hm.slot);
    p->free_handles.insert(h);
    --p->n_in_use[hm.where];
    p->home[h] = Home();
    drop_staged(p, h);
    map_set(p, 0, h, -1);
    map_set(p, 1, h, -1);
  }
  return PIE_OK;
}

int pie_block_where(pie_pool* p, int32_t n, const int32_t* handles, int32_t* out_where, int32_t* out_slot) {
  if (!p || n < 0 || (n > 0 && (!handles || !out_where || !out_slot))) return PIE_EINVAL;
  for (int32_t i = 0; i < n; ++i)
    if (handles[i] < 0 || handles[i] >= p->n_handles) return PIE_EINVAL;
  for (int32_t i = 0; i < n; ++i) {
    out_where[i] = p->home[handles[i]].where;
    out_slot[i] = p->home[handles[i]].slot;
  }
  return PIE_OK;
}

int pie_block_staged(pie_pool* p, int32_t region, int32_t n, const int32_t* handles, int32_t* out_stage_slot,
                     int32_t* out_state) {
  if (!p || (region != 0 && region != 1) || n < 0 || (n > 0 && (!handles || !out_stage_slot || !out_state)))
    return PIE_EINVAL;
  PIE_DRAIN(p);
  for (int32_t i = 0; i < n; ++i)
    if (handles[i] < 0 || handles[i] >= p->n_handles) return PIE_EINVAL;
  bool done = true;
  if (p->device && p->ev_in_rec[region]) {
    hipError_t e = hipEventQuery(p->ev_in[region]);
    if (e == hipErrorNotReady) {
      done = false;
      (void)hipGetLastError();
    } else if (e != hipSuccess) {
      g_last_hip_error = (int)e;
      return PIE_EHIP;
    }
  }
  for (int32_t i = 0; i < n; ++i) {
    const int32_t rank = p->stage_rank[region][handles[i]];
    out_stage_slot[i] = rank < 0 ? -1 : stage_slot(p, region, rank);
    out_state[i] = rank < 0 ? 0 : (done ? 2 : 1);
  }
  return PIE_OK;
}

int pie_pool_free_count(pie_pool* p, int32_t where, int32_t* out_n) {
  if (!p || !out_n || (where != 0 && where != 1)) return PIE_EINVAL;
  *out_n = (int32_t)p->free_slots[where].size();
  return PIE_OK;
}

int pie_block_address(pie_pool* p, int32_t where, int32_t layer, int32_t slot, void** out_ptr) {
  if (!p || !out_ptr || layer < 0 || layer >= p->cfg.n_layers || slot < 0) return PIE_EINVAL;
  if (where == PIE_WHERE_GPU) {
    if (slot >= p->cfg.n_gpu_blocks + 2 * p->cfg.n_stage_blocks) return PIE_EINVAL;
    if (!p->device) return PIE_ESTATE;
    *out_ptr = d_block(p, layer, slot);
  } else if (where == PIE_WHERE_HOST) {
    if (slot >= p->cfg.n_host_blocks) return PIE_EINVAL;
    if (!p->h_kv) return PIE_ESTATE;
    *out_ptr = h_block(p, layer, slot);
  } else {
    return PIE_EINVAL;
  }
  return PIE_OK;
}

int pie_swap_in(pie_pool* p, int32_t layer, int32_t n, const int32_t* handles, void* stream) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  return swap_in_impl(p, layer, n, handles, (hipStream_t)stream, false, Mark(), Mark());
}

int pie_swap_out(pie_pool* p, int32_t layer, int32_t n, const int32_t* handles, void* stream) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  return swap_out_impl(p, layer, n, handles, (hipStream_t)stream, Mark(), Mark());
}

int pie_migrate(pie_pool* p, int32_t n, const int32_t* handles, int32_t to_where, void* stream) {
  if (!p || (to_where != PIE_WHERE_GPU && to_where != PIE_WHERE_HOST)) return PIE_EINVAL;
  PIE_DRAIN(p);
  std::vector<uint8_t> seen;
  int rc = check_handles(p, n, handles, -1, seen);
  if (rc) return rc;
  std::vector<int32_t> movers;
  for (int32_t i = 0; i < n; ++i)
    if (p->home[handles[i]].where != to_where) movers.push_back(handles[i]);
  if (movers.size() > p->free_slots[to_where].size()) return PIE_ENOMEM;
  if (movers.empty()) return PIE_OK;
  hipStream_t s = (hipStream_t)stream;
  std::vector<int32_t> src(movers.size()), dst(movers.size());
  const int from = 1 - to_where;
  for (size_t i = 0; i < movers.size(); ++i) {
    const int32_t h = movers[i];
    const int32_t t = *p->free_slots[to_where].begin();
    p->free_slots[to_where].erase(p->free_slots[to_where].begin());
    src[i] = p->home[h].slot;
    dst[i] = t;
  }
  for (size_t i = 0; i < movers.size(); ++i) {
    const int32_t h = movers[i];
    p->free_slots[from].insert(src[i]);
    p->home[h] = {to_where, dst[i]};
    drop_staged(p, h);
    const int32_t dev_slot = to_where == PIE_WHERE_GPU ? dst[i] : -1;
    map_set(p, 0, h, dev_slot);
    map_set(p, 1, h, dev_slot);
  }
  p->n_in_use[from] -= (int32_t)movers.size();
  p->n_in_use[to_where] += (int32_t)movers.size();
  if (p->device) {
    const CopyPlan cp = plan_copy(p, src, dst);
    const bool on_host = cp.path == PIE_SWAP_DMA && !p->dma_stream_order;
    note_stream(p, s);
    if ((rc = order_after(s, p->ev_compute, p->ev_compute_rec, on_host))) return rc;
    // an earlier migration, possibly on another stream, may still be reading a slot this one is given
    if ((rc = order_after(s, p->ev_migrate, p->ev_migrate_rec, on_host))) return rc;
    for (int r = 0; r < 2; ++r) {
      if ((rc = order_after(s, p->ev_in[r], p->ev_in_rec[r], on_host))) return rc;
      if ((rc = order_after(s, p->ev_out[r], p->ev_out_rec[r], on_host))) return rc;
    }
    for (int32_t layer = 0; layer < p->cfg.n_layers; ++layer)
      if ((rc = copy_blocks(p, to_where == PIE_WHERE_GPU ? 0 : 1, layer, src, dst, cp, s))) return rc;
    PIE_HIP(hipEventRecord(p->ev_migrate, s));
    p->ev_migrate_rec = true;
  }
  return PIE_OK;
}

int pie_set_host_fraction(pie_pool* p, float f, int32_t n, const int32_t* order, void* stream,
                          int32_t* out_n_host) {
  if (!p || !(f >= 0.f && f <= 1.f)) return PIE_EINVAL;
  PIE_DRAIN(p);
  std::vector<uint8_t> seen;
  int rc = check_handles(p, n, order, -1, seen);
  if (rc) return rc;
  const int32_t k = (int32_t)std::floor((double)f * n + 0.5);
  // capacity check for both moves before anything changes
  int32_t to_gpu = 0, to_host = 0;
  for (int32_t i = 0; i < n; ++i) {
    const int w = p->home[order[i]].where;
    if (i < k && w == PIE_WHERE_GPU) ++to_host;
    if (i >= k && w == PIE_WHERE_HOST) ++to_gpu;
  }
  if ((size_t)to_gpu > p->free_slots[0].size()) return PIE_ENOMEM;
  if ((size_t)to_host > p->free_slots[1].size() + (size_t)to_gpu) return PIE_ENOMEM;
  if ((rc = pie_migrate(p, n - k, order + k, PIE_WHERE_GPU, stream))) return rc;
  if ((rc = pie_migrate(p, k, order, PIE_WHERE_HOST, stream))) return rc;
  if (out_n_host) *out_n_host = k;
  return PIE_OK;
}

int pie_set_swap_path(pie_pool* p, int32_t path) {
  if (!p || path < PIE_SWAP_AUTO || path > PIE_SWAP_KERNEL) return PIE_EINVAL;
  PIE_DRAIN(p);
  p->swap_path = path;
  return PIE_OK;
}

int pie_set_attn_partition(pie_pool* p, int32_t tokens) {
  if (!p || tokens < 0) return PIE_EINVAL;
  PIE_DRAIN(p);
  p->attn_partition = tokens;
  return PIE_OK;
}

int pie_get_attn_partition_sync(pie_pool* p, int32_t* out_tokens) {
  if (!p || !out_tokens) return PIE_EINVAL;
  if (!p->device) return PIE_ESTATE;
  int rc = pie_pool_sync(p);
  if (rc) return rc;
  PIE_HIP(hipMemcpy(out_tokens, p->d_plan + 1, sizeof(int32_t), hipMemcpyDeviceToHost));
  return PIE_OK;
}

int pie_set_attn_vector_alu(pie_pool* p, int32_t on) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  if (on && (p->cfg.n_q_heads != p->cfg.n_kv_heads || p->cfg.dtype == PIE_DTYPE_F32)) return PIE_ESTATE;
  p->attn_valu = on != 0;
  return PIE_OK;
}

int pie_set_layer_compute_us(pie_pool* p, float us) {
  if (!p || !(us >= 0.f) || us > 1.0e6f) return PIE_EINVAL;
  PIE_DRAIN(p);
  p->layer_compute_us = us;
  return PIE_OK;
}

int pie_set_swap_workgroups(pie_pool* p, int32_t n) {
  if (!p || n < 1 || n > 1024) return PIE_EINVAL;
  PIE_DRAIN(p);
  p->swap_wgs = n;
  return PIE_OK;
}

int pie_kv_append(pie_pool* p, int32_t layer, const void* d_k, const void* d_v, const int32_t* d_block_table,
                  int32_t max_blocks, const int32_t* d_ctx_lens, int32_t batch, void* stream) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  int rc = check_batch_args(p, layer, d_k, d_block_table, max_blocks, d_ctx_lens, batch);
  if (rc) return rc;
  if (batch > 0 && !d_v) return PIE_EINVAL;
  if (!p->device) return PIE_ESTATE;
  if (batch == 0) return PIE_OK;
  hipStream_t s = (hipStream_t)stream;
  bool stage_valid = false;
  if ((rc = compute_prologue(p, layer, s, &stage_valid))) return rc;
  if ((rc = launch_kv_append(p, layer, 1, d_k, d_v, d_block_table, max_blocks, d_ctx_lens, batch,
                             stage_valid ? kAppendPresent : kAppendGpuStrict, s)))
    return rc;
  return compute_epilogue(p, layer, s);
}

// work: the scratch the call's kernels use (NULL: the pool's own); ticket: which of its ticket counters.
static int attn_decode_impl(pie_pool* p, int32_t layer, const void* d_q, const int32_t* d_block_table,
                            int32_t max_blocks, const int32_t* d_ctx_lens, int32_t batch, void* d_out,
                            hipStream_t s, const AttnWork* work, int32_t ticket) {
  bool stage_valid = false;
  int rc;
  if ((rc = compute_prologue(p, layer, s, &stage_valid))) return rc;
  const int r = layer & 1;
  if ((rc = launch_attn_plan(p, d_ctx_lens, batch, max_blocks, s, false, work))) return rc;
  if ((rc = launch_attn_resolve(p, d_block_table, d_ctx_lens, batch, max_blocks, r == 0, stage_valid, r == 1,
                                stage_valid, s, nullptr, work)))
    return rc;
  if ((rc = launch_attn_decode(p, layer, d_q, max_blocks, d_ctx_lens, batch, d_out, s, nullptr, nullptr, ticket,
                               nullptr, nullptr, nullptr, work)))
    return rc;
  return compute_epilogue(p, layer, s);
}

int pie_attn_decode(pie_pool* p, int32_t layer, const void* d_q, const int32_t* d_block_table, int32_t max_blocks,
                    const int32_t* d_ctx_lens, int32_t batch, void* d_out, void* stream) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  int rc = check_batch_args(p, layer, d_q, d_block_table, max_blocks, d_ctx_lens, batch);
  if (rc) return rc;
  if (batch > 0 && !d_out) return PIE_EINVAL;
  if (!p->device) return PIE_ESTATE;
  if (batch == 0) return PIE_OK;
  return attn_decode_impl(p, layer, d_q, d_block_table, max_blocks, d_ctx_lens, batch, d_out, (hipStream_t)stream,
                          nullptr, -1);
}

int pie_attn_decode_static(pie_pool* p, int32_t layer, const void* d_q, const int32_t* d_block_table,
                           int32_t max_blocks, const int32_t* d_ctx_lens, int32_t batch, void* d_out, void* stream) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  if (layer < 0 || layer >= p->cfg.n_layers || batch < 0 || max_blocks < 0) return PIE_EINVAL;
  if (batch > 0 && (!d_q || !d_block_table || !d_ctx_lens || !d_out)) return PIE_EINVAL;
  if (!p->device) return PIE_ESTATE;
  if (batch == 0) return PIE_OK;
  AttnWork work;
  int rc = attn_static_work(p, batch, max_blocks, &work);   // PIE_ENOMEM: more than the static array holds
  if (rc) return rc;
  return attn_decode_impl(p, layer, d_q, d_block_table, max_blocks, d_ctx_lens, batch, d_out, (hipStream_t)stream,
                          &work, 0);
}

static int elapsed(hipEvent_t a, hipEvent_t b, float* ms);

int pie_attn_stream_probe_sync(pie_pool* p, int32_t layer, const int32_t* d_block_table, int32_t max_blocks,
                          const int32_t* d_ctx_lens, int32_t batch, void* stream, float* out_ms) {
  if (!p || !out_ms) return PIE_EINVAL;
  PIE_DRAIN(p);
  *out_ms = 0.f;
  int rc = check_batch_args(p, layer, d_block_table, d_block_table, max_blocks, d_ctx_lens, batch);
  if (rc) return rc;
  if (!p->device) return PIE_ESTATE;
  if (batch == 0) return PIE_OK;
  hipStream_t s = (hipStream_t)stream;
  bool stage_valid = false;
  if ((rc = compute_prologue(p, layer, s, &stage_valid))) return rc;
  const int r = layer & 1;
  if ((rc = launch_attn_plan(p, d_ctx_lens, batch, max_blocks, s))) return rc;
  if ((rc = launch_attn_resolve(p, d_block_table, d_ctx_lens, batch, max_blocks, r == 0, stage_valid, r == 1,
                                stage_valid, s)))
    return rc;
  PIE_HIP(hipEventRecord(p->lev[layer].k_start, s));
  if ((rc = launch_stream_probe(p, layer, max_blocks, batch, s))) return rc;
  PIE_HIP(hipEventRecord(p->lev[layer].k_end, s));
  if ((rc = compute_epilogue(p, layer, s))) return rc;
  PIE_HIP(hipEventSynchronize(p->lev[layer].k_end));
  return elapsed(p->lev[layer].k_start, p->lev[layer].k_end, out_ms);
}

int pie_prefetch_list(pie_pool* p, const int32_t* h_block_table, int32_t max_blocks, const int32_t* h_ctx_lens,
                      int32_t batch, int32_t* out_prefetch, int32_t* out_n_prefetch, int32_t* out_dirty,
                      int32_t* out_n_dirty) {
  if (!p || batch < 0 || max_blocks < 0 || !out_n_prefetch || !out_n_dirty) return PIE_EINVAL;
  if (batch > 0 && (!h_block_table || !h_ctx_lens || !out_prefetch || !out_dirty)) return PIE_EINVAL;
  const int32_t T = p->cfg.block_tokens;
  std::vector<uint8_t> seen(p->n_handles, 0), seen_dirty(p->n_handles, 0);
  int32_t np = 0, nd = 0;
  for (int32_t b = 0; b < batch; ++b) {
    const int32_t ctx = h_ctx_lens[b];
    if (ctx <= 0) continue;
    const int32_t nb = (ctx + T - 1) / T;
    if (nb > max_blocks) return PIE_EINVAL;
    for (int32_t j = 0; j < nb; ++j) {
      const int32_t h = h_block_table[(size_t)b * max_blocks + j];
      if (h < 0 || h >= p->n_handles) return PIE_EINVAL;
      if (p->home[h].where != PIE_WHERE_HOST) continue;
      if (!seen[h]) {
        seen[h] = 1;
        out_prefetch[np++] = h;
      }
      if (j == (ctx - 1) / T && !seen_dirty[h]) {
        seen_dirty[h] = 1;
        out_dirty[nd++] = h;
      }
    }
  }
  // ascending host slot: a densely used host pool is then one contiguous run, copied by one DMA transfer
  auto by_slot = [p](int32_t x, int32_t y) { return p->home[x].slot < p->home[y].slot; };
  std::sort(out_prefetch, out_prefetch + np, by_slot);
  std::sort(out_dirty, out_dirty + nd, by_slot);
  *out_n_prefetch = np;
  *out_n_dirty = nd;
  return PIE_OK;
}

}  // extern "C"

namespace pie {

// The step itself: everything pie_step enqueues, for arguments that have been checked.
static int step_body(pie_pool* p, const StepJob& j) {
  const void* d_q_all = j.d_q_all;
  const void* d_k_new = j.d_k_new;
  const void* d_v_new = j.d_v_new;
  const int32_t* d_block_table = j.d_block_table;
  const int32_t* d_ctx_lens = j.d_ctx_lens;
  const int32_t max_blocks = j.max_blocks, batch = j.batch;
  const int32_t n_prefetch = (int32_t)j.prefetch.size(), n_dirty = (int32_t)j.dirty.size();
  const int32_t* h_prefetch = j.prefetch.data();
  const int32_t* h_dirty = j.dirty.data();
  void* d_out_all = j.d_out_all;
  int rc;
  hipStream_t cs = j.cs, is = j.is, os = j.os;
  const int32_t L = p->cfg.n_layers;
  const size_t q_stride = (size_t)batch * p->cfg.n_q_heads * p->cfg.head_dim * p->elem_bytes;
  const size_t kv_stride = (size_t)batch * p->cfg.n_kv_heads * p->cfg.head_dim * p->elem_bytes;
  // Monitoring: by events (one recorded before and after every piece of work, which keeps the compute
  // stream's kernels from running back to back) or by the device clock (the kernels note their own times).
  const bool timed = p->timing == PIE_TIMING_EVENTS, clocked = p->timing == PIE_TIMING_CLOCK;
  auto clock_row = [&](int32_t l) { return clocked ? p->d_clock + (size_t)l * kClockRow : nullptr; };
  // by device clock only the end of a copy is stamped (a stamp is a kernel launch the copies behind it wait
  // for); when it began follows from what it had to wait for
  auto mark = [&](hipEvent_t ev, int32_t l, int word) {
    Mark m;
    if (timed) m.ev = ev;
    if (clocked && (word == kClockInEnd || word == kClockOutEnd)) m.clk = p->d_clock + (size_t)l * kClockRow + word;
    return m;
  };
  // Region 0 may already hold layer 0's blocks: the previous step brought them in behind its last layer.
  bool pre_hit = p->pre_valid && n_prefetch > 0 && p->region_layer[0] == 0 &&
                 (int32_t)p->stage_list[0].size() == n_prefetch;
  for (int32_t i = 0; pre_hit && i < n_prefetch; ++i) pre_hit = p->stage_list[0][i] == h_prefetch[i];
  p->pre_valid = false;
  p->step_pre_hit = pre_hit;
  p->step_pre_timed = pre_hit ? p->pre_timed : 0;
  p->step_pre_idx = p->pre_idx;                  // which of the two time marks that copy wrote
  p->bytes_in = p->bytes_out = 0;
  p->step_timed = 0;
  note_stream(p, cs);
  if (timed) PIE_HIP(hipEventRecord(p->ev_step_start, cs));
  if (timed || clocked)
    for (auto& le : p->lev) le.in_used = le.out_used = false;
  // The prefetch list is the same for every layer, so both staging regions' slot assignments are known now:
  // publish them, send the map changes, and plan the attention work once for the whole step.
  publish_stage_list(p, 0, n_prefetch, h_prefetch);
  if (L > 1) publish_stage_list(p, 1, n_prefetch, h_prefetch);
  if ((rc = wait_if(cs, p->ev_migrate, p->ev_migrate_rec))) return rc;
  if ((rc = flush_map(p, cs))) return rc;
  // With a new token, the attention reads the context without it from the cache and takes the token itself from
  // the new rows (the reduction kernel adds it), so no layer waits for the appends that store the rows: the one
  // launch for the GPU-homed tail blocks of every layer runs on the write-back stream beside the first layers
  // (the compute stream waits for it when the step ends, and then only if the host does not see it finished),
  // and the host-homed tails get theirs on the same stream once the copy that stages them for a layer has
  // arrived, just ahead of their write-back.
  const bool with_new = d_k_new != nullptr;
  const bool staged_tails = with_new && n_dirty > 0;
  if (with_new) {                                // the appends read the maps sent above
    PIE_HIP(hipEventRecord(p->ev_map, cs));
    p->ev_map_rec = true;
  }
  if ((rc = launch_attn_plan(p, d_ctx_lens, batch, max_blocks, cs, clocked, nullptr, with_new))) return rc;
  if ((rc = launch_attn_resolve(p, d_block_table, d_ctx_lens, batch, max_blocks, true, true, L > 1, true, cs)))
    return rc;
  if (with_new) {
    note_stream(p, os);
    if (os != cs) PIE_HIP(hipStreamWaitEvent(os, p->ev_map, 0));
    if ((rc = launch_kv_append(p, 0, L, d_k_new, d_v_new, d_block_table, max_blocks, d_ctx_lens, batch,
                               staged_tails ? kAppendGpuHomed : kAppendGpuStrict, os)))
      return rc;
    PIE_HIP(hipEventRecord(p->ev_append, os));
  }
  StagedAppend job{nullptr, nullptr, d_block_table, d_ctx_lens, max_blocks, batch};
  auto job_for = [&](int32_t l) -> const StagedAppend* {
    if (!staged_tails) return nullptr;
    job.d_k = (const char*)d_k_new + l * kv_stride;
    job.d_v = (const char*)d_v_new + l * kv_stride;
    return &job;
  };
  // layer 0's blocks have no earlier layer to hide behind
  if (n_prefetch > 0) {
    if ((rc = swap_in_impl(p, 0, n_prefetch, h_prefetch, is, true, mark(p->lev[0].in_start, 0, kClockInStart),
                           mark(p->lev[0].in_end, 0, kClockInEnd), pre_hit)))
      return rc;
    p->lev[0].in_used = (timed || clocked) && !pre_hit;
  }
  // When the host itself orders the copies (copy-engine path) it passes, once per layer, the moment the
  // previous layer's computation has ended; from two of those it knows how long a layer takes.
  auto now_us = [] {
    return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
  };
  double t_free = -1.0, layer_us = -1.0;
  for (int32_t l = 0; l < L; ++l) {
    // The presence check: the layer's staged blocks have arrived (migrations and map updates were waited
    // for and sent once, at the start of the step).  A wait on the compute stream costs about 8 us even when
    // the event has long completed, so the host first looks for itself: the layer before is still computing,
    // and until shortly before it ends (this layer's kernels must be queued by then) the host polls the
    // swap-in's event.  A swap-in the host has seen complete needs no wait on the stream.
    if (n_prefetch > 0 && p->ev_in_rec[l & 1]) {
      bool arrived = false;
      if (p->presence_poll && p->in_on_host[l & 1] && layer_us > 0.0) {
        const double deadline = t_free + layer_us - (50.0 + 0.1 * layer_us);
        for (;;) {
          const hipError_t e = hipEventQuery(p->ev_in[l & 1]);
          if (e == hipSuccess) { arrived = true; break; }
          (void)hipGetLastError();
          if (e != hipErrorNotReady || now_us() >= deadline) break;
        }
      }
      if (!arrived && (rc = wait_if(cs, p->ev_in[l & 1], true))) return rc;
    }
    if (timed) PIE_HIP(hipEventRecord(p->lev[l].attn_start, cs));
    // The next user of this layer's staging region (layer l + 2's prefetch, this layer's write-back) waits
    // for the event that completes with the layer's last kernel.
    const bool standin = p->layer_compute_us > 0.f;
    hipEvent_t read_done = n_prefetch > 0 ? p->ev_read[l & 1] : nullptr;
    if ((rc = launch_attn_decode(p, l, (const char*)d_q_all + l * q_stride, max_blocks, d_ctx_lens, batch,
                                 (char*)d_out_all + l * q_stride, cs, timed ? p->lev[l].k_start : nullptr,
                                 timed ? p->lev[l].k_end : nullptr, -1, clock_row(l), nullptr,
                                 standin ? nullptr : read_done, nullptr,
                                 with_new ? (const char*)d_k_new + l * kv_stride : nullptr,
                                 with_new ? (const char*)d_v_new + l * kv_stride : nullptr)))
      return rc;
    if (standin && (rc = launch_busy(p->layer_compute_us, p->wall_clock_khz, cs, clock_row(l), read_done)))
      return rc;
    if (timed) PIE_HIP(hipEventRecord(p->lev[l].attn_end, cs));
    if (n_prefetch > 0) p->ev_read_rec[l & 1] = true;
    if (l + 1 < L && n_prefetch > 0) {
      // The next layer's prefetch goes into the region layer l - 1 used, so it starts when that layer ends
      // and runs behind this one.  It is enqueued after this layer's kernels because a copy-engine
      // transfer makes the host wait for layer l - 1 here (see order_after): the compute stream must
      // already hold this layer's work then.
      if ((rc = swap_in_impl(p, l + 1, n_prefetch, h_prefetch, is, true,
                             mark(p->lev[l + 1].in_start, l + 1, kClockInStart),
                             mark(p->lev[l + 1].in_end, l + 1, kClockInEnd))))
        return rc;
      p->lev[l + 1].in_used = timed || clocked;
      if (p->in_on_host[(l + 1) & 1]) {            // the host has just waited for layer l - 1 to end
        const double t = now_us();
        if (t_free >= 0.0) layer_us = t - t_free;
        t_free = t;
      }
    }
    if (n_dirty > 0 && d_k_new) {
      // The attention only reads the staged tail blocks.  So they get the new rows and go home as soon as this
      // layer's swap-in has completed, beside the layer's computation, not after it: the write-back is then
      // neither something the host waits for at the layer's end (with the next layer's kernels not yet
      // queued) nor a link in the chain  layer l ends -> write back -> prefetch layer l + 2 into the region.
      if ((rc = swap_out_impl(p, l, n_dirty, h_dirty, os, mark(p->lev[l].out_start, l, kClockOutStart),
                              mark(p->lev[l].out_end, l, kClockOutEnd), false, job_for(l))))
        return rc;
      p->lev[l].out_used = timed || clocked;
    }
  }
  // The next step will most likely touch the same host blocks: bring layer 0's in now, behind this step's
  // last layer, into the region the layer before last has just left.  If anything about those blocks changes
  // first, the copy is repeated.
  if (p->cross_step_prefetch && n_prefetch > 0 && L >= 2) {
    Mark m1;                                     // two marks in turn: the step that uses the copy reads its mark
    p->pre_idx ^= 1;                             // after this step has written the other one
    if (timed) m1.ev = p->ev_pre_end[p->pre_idx];
    if (clocked) m1.clk = p->d_clock + (size_t)L * kClockRow + 1 + p->pre_idx;
    if ((rc = swap_in_impl(p, 0, n_prefetch, h_prefetch, is, true, Mark(), m1))) return rc;
    p->pre_valid = true;
    p->pre_timed = p->timing;
  }
  if (clocked && (rc = launch_clock_fold(p->d_clock, L, cs))) return rc;
  // Whatever follows this step on the compute stream, or waits for the step's compute work, finds the new rows
  // in the GPU-homed tail blocks.  That launch ran beside the first layers: usually the host sees it finished.
  if (with_new && os != cs) {
    const hipError_t e = hipEventQuery(p->ev_append);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      if (e != hipErrorNotReady) { g_last_hip_error = (int)e; return PIE_EHIP; }
      PIE_HIP(hipStreamWaitEvent(cs, p->ev_append, 0));
    }
  }
  // later migrations wait for the step's compute work
  PIE_HIP(hipEventRecord(p->ev_compute, cs));
  p->ev_compute_rec = true;
  p->step_timed = p->timing;
  return PIE_OK;
}

}  // namespace pie

extern "C" {

int pie_step(pie_pool* p, const void* d_q_all, const void* d_k_new, const void* d_v_new,
             const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_ctx_lens, int32_t batch,
             int32_t n_prefetch, const int32_t* h_prefetch, int32_t n_dirty, const int32_t* h_dirty,
             void* d_out_all, void* compute_stream, void* swap_in_stream, void* swap_out_stream) {
  if (!p) return PIE_EINVAL;
  int rc = check_batch_args(p, 0, d_q_all, d_block_table, max_blocks, d_ctx_lens, batch);
  if (rc) return rc;
  if (batch > 0 && !d_out_all) return PIE_EINVAL;
  if ((d_k_new == nullptr) != (d_v_new == nullptr)) return PIE_EINVAL;
  if (n_prefetch < 0 || n_dirty < 0) return PIE_EINVAL;
  if (n_prefetch > p->cfg.n_stage_blocks) return PIE_ENOMEM;
  std::vector<uint8_t> seen;
  if ((rc = check_handles(p, n_prefetch, h_prefetch, PIE_WHERE_HOST, seen))) return rc;
  {
    std::vector<uint8_t> seen_d;
    if ((rc = check_handles(p, n_dirty, h_dirty, PIE_WHERE_HOST, seen_d))) return rc;
    for (int32_t i = 0; i < n_dirty; ++i)
      if (!seen[h_dirty[i]]) return PIE_ESTATE;  // a dirty block must be among the prefetched ones
  }
  if (!p->device) return PIE_ESTATE;
  if (batch == 0) return PIE_OK;
  StepJob job{d_q_all, d_k_new, d_v_new, d_block_table, max_blocks, d_ctx_lens, batch,
              std::vector<int32_t>(h_prefetch, h_prefetch + n_prefetch), std::vector<int32_t>(h_dirty, h_dirty + n_dirty),
              d_out_all, (hipStream_t)compute_stream, (hipStream_t)swap_in_stream, (hipStream_t)swap_out_stream};
  if (!p->async_submit) return step_body(p, job);
  {                                              // hand it to the submit thread and return
    std::lock_guard<std::mutex> g(p->submit_mutex);
    p->submit_jobs.push_back(std::move(job));
  }
  p->submit_wake.notify_one();
  return PIE_OK;
}

int pie_set_async_submit(pie_pool* p, int32_t on) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  if (!p->device) return PIE_ESTATE;
  if (on && !p->submitter.joinable()) {
    try {
      p->submitter = std::thread(submit_loop, p);
    } catch (...) {
      return PIE_ENOMEM;
    }
  }
  p->async_submit = on != 0;
  return PIE_OK;
}

int pie_step_join_sync(pie_pool* p) {
  if (!p) return PIE_EINVAL;
  return submit_drain(p);
}

int pie_set_cross_step_prefetch(pie_pool* p, int32_t on) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  p->cross_step_prefetch = on != 0;
  if (!on) p->pre_valid = false;
  return PIE_OK;
}

int pie_set_host_presence_check(pie_pool* p, int32_t on) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  p->presence_poll = on != 0;
  return PIE_OK;
}

int pie_set_timing(pie_pool* p, int32_t mode) {
  if (!p || mode < PIE_TIMING_OFF || mode > PIE_TIMING_CLOCK) return PIE_EINVAL;
  PIE_DRAIN(p);
  p->timing = mode;
  return PIE_OK;
}

static int elapsed(hipEvent_t a, hipEvent_t b, float* ms) {
  hipError_t e = hipEventElapsedTime(ms, a, b);
  if (e != hipSuccess) {
    g_last_hip_error = (int)e;
    (void)hipGetLastError();
    return PIE_EHIP;
  }
  return PIE_OK;
}

// The clock table of the last step, copied to the host.  The step must have run: nothing is waited for here.
static int read_clock(pie_pool* p, std::vector<unsigned long long>& t) {
  for (hipStream_t s : p->streams_seen) {
    const hipError_t e = hipStreamQuery(s);
    if (e == hipErrorNotReady) {
      (void)hipGetLastError();
      return PIE_ESTATE;                          // still running: call pie_pool_sync first
    }
    PIE_HIP(e);
  }
  t.resize(((size_t)p->cfg.n_layers + 1) * kClockRow);
  PIE_HIP(hipMemcpy(t.data(), p->d_clock, t.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
  return PIE_OK;
}

static int layer_times_from_clock(pie_pool* p, float* t_attn, float* t_kernel, float* t_in, float* t_out,
                                  float* t_stall, float* step_ms) {
  std::vector<unsigned long long> t;
  int rc = read_clock(p, t);
  if (rc) return rc;
  const int32_t L = p->cfg.n_layers;
  const double per_ms = (double)p->wall_clock_khz;
  auto at = [&](int32_t l, int w) { return t[(size_t)l * kClockRow + w]; };
  auto span = [&](unsigned long long a, unsigned long long b) { return b > a ? (float)((double)(b - a) / per_ms) : 0.f; };
  const unsigned long long step_start = at(L, 0);
  for (int32_t l = 0; l < L; ++l) {
    if (t_attn) t_attn[l] = span(at(l, kClockKernelStart), at(l, kClockLayerEnd));
    if (t_kernel) t_kernel[l] = span(at(l, kClockKernelStart), at(l, kClockKernelEnd));
    // A swap-in starts when the one before it on its stream has ended and the staging region is free, i.e.
    // the layer two back has been computed; a write-back when its layer's swap-in and the write-back before
    // it have ended.
    if (t_in) {
      unsigned long long from = l >= 2 ? at(l - 2, kClockLayerEnd) : step_start;
      if (l >= 1 && p->lev[l - 1].in_used && at(l - 1, kClockInEnd) > from) from = at(l - 1, kClockInEnd);
      t_in[l] = p->lev[l].in_used ? span(from, at(l, kClockInEnd)) : 0.f;
    }
    if (t_out) {
      unsigned long long from = p->lev[l].in_used ? at(l, kClockInEnd) : step_start;
      if (l >= 1 && p->lev[l - 1].out_used && at(l - 1, kClockOutEnd) > from) from = at(l - 1, kClockOutEnd);
      t_out[l] = p->lev[l].out_used ? span(from, at(l, kClockOutEnd)) : 0.f;
    }
    if (t_stall) {
      const unsigned long long free_at = l == 0 ? step_start : at(l - 1, kClockLayerEnd);
      t_stall[l] = p->lev[l].in_used ? span(free_at, at(l, kClockInEnd)) : 0.f;
      // a first layer staged by the step before: what was left of that copy when this step began
      if (l == 0 && p->step_pre_hit && p->step_pre_timed == PIE_TIMING_CLOCK)
        t_stall[0] = span(step_start, at(L, 1 + p->step_pre_idx));
    }
  }
  if (step_ms) *step_ms = span(step_start, at(L - 1, kClockLayerEnd));
  return PIE_OK;
}

int pie_get_layer_times(pie_pool* p, float* t_attn, float* t_kernel, float* t_in, float* t_out, float* t_stall) {
  if (!p) return PIE_EINVAL;
  PIE_DRAIN(p);
  if (!p->device || !p->step_timed) return PIE_ESTATE;
  if (p->step_timed == PIE_TIMING_CLOCK) return layer_times_from_clock(p, t_attn, t_kernel, t_in, t_out, t_stall, nullptr);
  const int32_t L = p->cfg.n_layers;
  int rc;
  for (int32_t l = 0; l < L; ++l) {
    float ms = 0.f;
    if (t_attn) {
      if ((rc = elapsed(p->lev[l].attn_start, p->lev[l].attn_end, &ms))) return rc;
      t_attn[l] = ms;
    }
    if (t_kernel) {
      if ((rc = elapsed(p->lev[l].k_start, p->lev[l].k_end, &ms))) return rc;
      t_kernel[l] = ms;
    }
    if (t_in) {
      ms = 0.f;
      if (p->lev[l].in_used && (rc = elapsed(p->lev[l].in_start, p->lev[l].in_end, &ms))) return rc;
      t_in[l] = ms;
    }
    if (t_out) {
      ms = 0.f;
      if (p->lev[l].out_used && (rc = elapsed(p->lev[l].out_start, p->lev[l].out_end, &ms))) return rc;
      t_out[l] = ms;
    }
    if (t_stall) {
      // time the compute stream, free since the previous layer ended (or the step began), still had to wait
      // for this layer's prefetch: from that moment to the end of the swap-in, if the swap-in ended later
      ms = 0.f;
      if (p->lev[l].in_used &&
          (rc = elapsed(l == 0 ? p->ev_step_start : p->lev[l - 1].attn_end, p->lev[l].in_end, &ms)))
        return rc;
      if (l == 0 && p->step_pre_hit && p->step_pre_timed == PIE_TIMING_EVENTS &&
          (rc = elapsed(p->ev_step_start, p->ev_pre_end[p->step_pre_idx], &ms)))
        return rc;
      t_stall[l] = ms > 0.f ? ms : 0.f;
    }
  }
  return PIE_OK;
}

int pie_get_stats(pie_pool* p, pie_stats* out) {
  if (!p || !out) return PIE_EINVAL;
  PIE_DRAIN(p);
  std::memset(out, 0, sizeof(*out));
  out->n_layers = p->cfg.n_layers;
  out->host_blocks_in_use = p->n_in_use[1];
  out->gpu_blocks_in_use = p->n_in_use[0];
  const int32_t tot = p->n_in_use[0] + p->n_in_use[1];
  const float f = tot ? (float)p->n_in_use[1] / (float)tot : 0.f;
  out->host_fraction = f;
  out->expansion_simple = f < 1.f ? 1.f / (1.f - f) : INFINITY;
  const float L = (float)p->cfg.n_layers;
  out->expansion_staged = L / (L * (1.f - f) + 2.f * f);
  out->bytes_in = p->bytes_in;
  out->bytes_out = p->bytes_out;
  if (p->device && p->step_timed) {
    const int32_t n = p->cfg.n_layers;
    std::vector<float> a(n), i(n), o(n), s(n);
    const bool clocked = p->step_timed == PIE_TIMING_CLOCK;
    int rc = clocked ? layer_times_from_clock(p, a.data(), nullptr, i.data(), o.data(), s.data(), &out->step_ms)
                     : pie_get_layer_times(p, a.data(), nullptr, i.data(), o.data(), s.data());
    if (rc) return rc;
    for (int32_t l = 0; l < n; ++l) {
      out->attn_ms += a[l];
      out->swap_in_ms += i[l];
      out->swap_out_ms += o[l];
      out->stall_ms += s[l];
    }
    if (!clocked && (rc = elapsed(p->ev_step_start, p->lev[n - 1].attn_end, &out->step_ms))) return rc;
  }
  out->device_error_flags = p->last_err_flags;
  out->first_layer_prestaged = p->step_pre_hit ? 1u : 0u;
  return PIE_OK;
}

int pie_check_errors_sync(pie_pool* p, uint32_t* out_flags) {
  if (!p || !out_flags) return PIE_EINVAL;
  PIE_DRAIN(p);
  *out_flags = 0;
  if (!p->device) return PIE_OK;
  int rc = pie_pool_sync(p);
  if (rc) return rc;
  PIE_HIP(hipMemcpy(out_flags, p->d_err, sizeof(uint32_t), hipMemcpyDeviceToHost));
  p->last_err_flags |= *out_flags;
  if (*out_flags) {
    if ((rc = launch_zero_u32(p->d_err, 1, nullptr))) return rc;
    PIE_HIP(hipStreamSynchronize(nullptr));
  }
  return PIE_OK;
}

int pie_last_hip_error(void) { return g_last_hip_error; }

const char* pie_strerror(int code) {
  switch (code) {
    case PIE_OK: return "ok";
    case PIE_EINVAL: return "invalid argument";
    case PIE_ENOMEM: return "pool, staging region or buffer too small";
    case PIE_ESTATE: return "operation not valid in this state";
    case PIE_EHIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

int pie_version(void) { return 1; }

}  // extern "C"
