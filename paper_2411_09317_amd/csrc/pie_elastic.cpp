// Layer caches that grow and shrink as layers move to CPU memory (Section 3.1: a cache of a bytes over n
// layers becomes a / (n - m) per layer when m layers are kept in CPU memory; Section 4.1, block manager: new
// blocks are shown to the scheduler once the reallocation is complete, and on shrinking blocks are hidden
// first and freed afterwards).
//
// The paper reallocates a layer's cache as one piece when the layer is swapped back in.  Here the GPU memory
// is cut into equal chunks of `chunk_blocks` block slots and a layer's cache is any set of chunks: block h of
// a layer lives in slot chunk[h / chunk_blocks] * chunk_blocks + h % chunk_blocks.  A resident layer can be
// given more chunks where it is, a layer travels as a few large transfers (one per chunk), and nothing has to
// be contiguous.
//
// pie_chunk_book is the bookkeeping as pure host logic; pie_elastic_pool drives it, together with the
// layer-granular swapping protocol (pie_layer_sched), on the GPU.
#include <algorithm>
#include <chrono>
#include <cstring>
#include <new>
#include <vector>

#include "pie.h"
#include "pie_internal.h"
#include "pie_layer_core.h"

struct pie_chunk_book {
  int32_t n = 0, N = 0, k_cap = 0;
  std::vector<std::vector<int32_t>> chunks;   // chunk ids a resident layer holds, in block order
  std::vector<uint8_t> resident;
  std::vector<int32_t> image;                 // chunks of data a layer carries
  std::vector<int32_t> free;                  // ascending
  int32_t m = 0, k_target = 0, hide = -1, visible = 0;

  int32_t target_for(int32_t m_) const { return std::min(k_cap, N / (n - m_)); }
  void release(int32_t c) { free.insert(std::upper_bound(free.begin(), free.end(), c), c); }
  void recount() {
    int32_t v = k_target;
    for (int32_t j = 0; j < n; ++j)
      if (resident[j]) v = std::min(v, (int32_t)chunks[j].size());
    visible = hide < 0 ? v : std::min(v, hide);
  }
  // Free chunks go to resident layers below the target, lowest layer first; what the GPU layer slots still to
  // be filled will need is kept back.  Returns through `grown` the layers whose chunk list changed.
  void top_up(std::vector<int32_t>* grown) {
    int32_t n_res = 0;
    for (int32_t j = 0; j < n; ++j) n_res += resident[j];
    const int64_t reserve = (int64_t)std::max(0, (n - m) - n_res) * k_target;
    for (int32_t j = 0; j < n; ++j) {
      if (!resident[j]) continue;
      bool changed = false;
      while ((int32_t)chunks[j].size() < k_target && (int64_t)free.size() > reserve) {
        chunks[j].push_back(free.front());
        free.erase(free.begin());
        changed = true;
      }
      if (changed && grown) grown->push_back(j);
    }
    recount();
  }
};

extern "C" {

int pie_chunk_book_create(int32_t n_layers, int32_t n_chunks, int32_t max_chunks_per_layer, pie_chunk_book** out) {
  if (!out) return PIE_EINVAL;
  *out = nullptr;
  if (n_layers <= 0 || n_chunks <= 0 || n_chunks % n_layers || max_chunks_per_layer < n_chunks / n_layers ||
      max_chunks_per_layer > pie::kMaxLayerChunks)
    return PIE_EINVAL;
  pie_chunk_book* b = new (std::nothrow) pie_chunk_book();
  if (!b) return PIE_ENOMEM;
  b->n = n_layers;
  b->N = n_chunks;
  b->k_cap = max_chunks_per_layer;
  const int32_t k0 = n_chunks / n_layers;
  b->chunks.resize(n_layers);
  for (int32_t j = 0; j < n_layers; ++j)
    for (int32_t i = 0; i < k0; ++i) b->chunks[j].push_back(j * k0 + i);
  b->resident.assign(n_layers, 1);
  b->image.assign(n_layers, k0);
  b->k_target = b->visible = k0;
  *out = b;
  return PIE_OK;
}

int pie_chunk_book_destroy(pie_chunk_book* b) {
  if (!b) return PIE_EINVAL;
  delete b;
  return PIE_OK;
}

// changed (optional, n_layers entries): set to 1 for every layer whose chunk list this call changed
static int book_set(pie_chunk_book* b, int32_t m, int32_t chunks_in_use, uint8_t* changed) {
  if (!b || m < 0 || m >= b->n || chunks_in_use < 0) return PIE_EINVAL;
  const int32_t k_new = b->target_for(m);
  if (k_new < b->k_target) {
    b->hide = k_new;
    b->recount();
    if (chunks_in_use > k_new) return PIE_ESTATE;
    for (int32_t j = 0; j < b->n; ++j) {          // cut every cache to the new size where it is
      if (b->resident[j]) {
        while ((int32_t)b->chunks[j].size() > k_new) {
          b->release(b->chunks[j].back());
          b->chunks[j].pop_back();
          if (changed) changed[j] = 1;
        }
      }
      b->image[j] = std::min(b->image[j], k_new);
    }
  }
  b->m = m;
  b->k_target = k_new;
  b->hide = -1;
  std::vector<int32_t> grown;
  b->top_up(&grown);
  if (changed)
    for (int32_t j : grown) changed[j] = 1;
  return PIE_OK;
}

int pie_chunk_book_set_layers_on_cpu(pie_chunk_book* b, int32_t m, int32_t chunks_in_use) {
  return book_set(b, m, chunks_in_use, nullptr);
}

static int book_left(pie_chunk_book* b, int32_t layer, int32_t n_carried, std::vector<int32_t>* grown) {
  if (!b || layer < 0 || layer >= b->n) return PIE_EINVAL;
  if (!b->resident[layer]) return PIE_ESTATE;
  if (n_carried > (int32_t)b->chunks[layer].size()) return PIE_EINVAL;
  b->resident[layer] = 0;
  b->image[layer] = n_carried < 0 ? (int32_t)b->chunks[layer].size() : n_carried;
  for (int32_t c : b->chunks[layer]) b->release(c);
  b->chunks[layer].clear();
  b->top_up(grown);
  return PIE_OK;
}

int pie_chunk_book_left_gpu(pie_chunk_book* b, int32_t layer, int32_t n_carried) {
  return book_left(b, layer, n_carried, nullptr);
}

int pie_chunk_book_enters_gpu(pie_chunk_book* b, int32_t layer, int32_t* out_n_data) {
  if (!b || layer < 0 || layer >= b->n) return PIE_EINVAL;
  if (b->resident[layer]) return PIE_ESTATE;
  const int32_t k = std::min(b->k_target, (int32_t)b->free.size());
  if (k < std::max(b->image[layer], b->visible)) return PIE_ENOMEM;   // what is visible never shrinks unasked
  b->chunks[layer].assign(b->free.begin(), b->free.begin() + k);
  b->free.erase(b->free.begin(), b->free.begin() + k);
  b->resident[layer] = 1;
  b->recount();
  if (out_n_data) *out_n_data = b->image[layer];
  return PIE_OK;
}

int pie_chunk_book_layer(pie_chunk_book* b, int32_t layer, int32_t* out_resident, int32_t* out_n_data,
                         int32_t* out_n_chunks, int32_t* out_chunks) {
  if (!b || layer < 0 || layer >= b->n) return PIE_EINVAL;
  if (out_resident) *out_resident = b->resident[layer];
  if (out_n_data) *out_n_data = b->image[layer];
  if (out_n_chunks) *out_n_chunks = (int32_t)b->chunks[layer].size();
  if (out_chunks) std::copy(b->chunks[layer].begin(), b->chunks[layer].end(), out_chunks);
  return PIE_OK;
}

int pie_chunk_book_capacity(pie_chunk_book* b, int32_t* out_visible, int32_t* out_target, int32_t* out_free,
                            int32_t* out_layers_on_cpu) {
  if (!b) return PIE_EINVAL;
  if (out_visible) *out_visible = b->visible;
  if (out_target) *out_target = b->k_target;
  if (out_free) *out_free = (int32_t)b->free.size();
  if (out_layers_on_cpu) *out_layers_on_cpu = b->m;
  return PIE_OK;
}

}  // extern "C"

// ---------------------------------------------------------------------------------------------------------
// the driver: the swapping protocol over chunked layer caches
// ---------------------------------------------------------------------------------------------------------

struct pie_elastic_pool {
  pie_pool* pool = nullptr;            // n_layers logical layers x (n_chunks / n_layers) chunks of GPU memory
  pie_layer_sched* sched = nullptr;
  pie_chunk_book* book = nullptr;
  int32_t n = 0, C = 0, k_cap = 0, H = 0, N = 0, n_host_slots = 0;
  size_t chunk_bytes = 0, host_slot_bytes = 0;
  char* h_base = nullptr;
  int32_t* d_maps = nullptr;           // [n][H] handle -> slot of the whole GPU memory, -1 = none
  hipEvent_t ev_in = nullptr, ev_out = nullptr;
  std::vector<hipEvent_t> ev_layer;    // last compute work on a layer
  std::vector<uint8_t> ev_layer_rec;
  pie_layer_stats stats;
  int32_t prev_layer = -1;
  int32_t live_chunks = -1;            // chunks of a cache that hold live blocks (-1: all)
  int32_t out_carried = 0;             // chunks the swap-out in flight copies
};

namespace {

using pie::g_last_hip_error;

char* chunk_dev(const pie_elastic_pool* lp, int32_t chunk) { return lp->pool->d_kv + (size_t)chunk * lp->chunk_bytes; }
char* slot_host(const pie_elastic_pool* lp, int32_t slot) { return lp->h_base + (size_t)slot * lp->host_slot_bytes; }

// Sends layer j's block map (from its chunk list) on stream s.
int send_map(pie_elastic_pool* lp, int32_t j, hipStream_t s) {
  pie::ChunkList list;
  const std::vector<int32_t>& c = lp->book->chunks[j];
  list.n = (int32_t)c.size();
  std::copy(c.begin(), c.end(), list.chunk);
  return pie::launch_chunk_map_fill(lp->d_maps + (size_t)j * lp->H, lp->H, lp->C, list, s);
}

int on_out_complete(pie_elastic_pool* lp, hipStream_t cs) {
  const int32_t layer = lp->sched->moving_out;
  pie_layer_sched_complete(lp->sched, 1);
  std::vector<int32_t> grown;
  int rc = book_left(lp->book, layer, lp->out_carried, &grown);
  if (rc) return rc;
  for (int32_t j : grown)                          // resident layers that were given its chunks
    if ((rc = send_map(lp, j, cs))) return rc;
  return PIE_OK;
}

int poll_moves(pie_elastic_pool* lp, hipStream_t cs) {
  pie_layer_sched* s = lp->sched;
  if (s->moving_in >= 0) {
    hipError_t e = hipEventQuery(lp->ev_in);
    if (e == hipSuccess) pie_layer_sched_complete(s, 0);
    else if (e != hipErrorNotReady) { g_last_hip_error = (int)e; (void)hipGetLastError(); return PIE_EHIP; }
    else (void)hipGetLastError();
  }
  if (s->moving_out >= 0) {
    hipError_t e = hipEventQuery(lp->ev_out);
    if (e == hipSuccess) { int rc = on_out_complete(lp, cs); if (rc) return rc; }
    else if (e != hipErrorNotReady) { g_last_hip_error = (int)e; (void)hipGetLastError(); return PIE_EHIP; }
    else (void)hipGetLastError();
  }
  return PIE_OK;
}

// Starts the transfers an action names, one copy-engine transfer per chunk.  All ordering is done on the
// host: a swap-out first waits for the last computation on its layer; a swap-in takes chunks that are free,
// i.e. whose previous tenant's swap-out the host has seen complete.  The incoming layer's block map goes out
// on the compute stream, ahead of the layer's kernels.
// The first n chunks of a layer to or from its image in CPU memory (kind 0: in, 1: out), one copy-engine transfer
// per run of neighbouring chunks: a transfer costs the host some 10-20 us to enqueue whatever it carries, and a
// layer's chunks mostly are neighbours.
int copy_chunks(pie_elastic_pool* lp, int kind, char* host_image, const std::vector<int32_t>& c, size_t n, hipStream_t s) {
  for (size_t i = 0; i < n;) {
    size_t j = i + 1;
    while (j < n && c[j] == c[j - 1] + 1) ++j;
    const size_t bytes = (j - i) * lp->chunk_bytes;
    char* h = host_image + i * lp->chunk_bytes;
    if (kind == 0) PIE_HIP(hipMemcpyAsync(chunk_dev(lp, c[i]), h, bytes, hipMemcpyHostToDevice, s));
    else PIE_HIP(hipMemcpyAsync(h, chunk_dev(lp, c[i]), bytes, hipMemcpyDeviceToHost, s));
    i = j;
  }
  return PIE_OK;
}

int start_moves(pie_elastic_pool* lp, const pie_layer_action& a, hipStream_t cs, hipStream_t is, hipStream_t os) {
  int rc_copy;
  if (a.out_layer >= 0) {
    if (lp->ev_layer_rec[a.out_layer]) PIE_HIP(hipEventSynchronize(lp->ev_layer[a.out_layer]));
    const std::vector<int32_t>& c = lp->book->chunks[a.out_layer];
    // only the chunks that hold live blocks travel; the others are simply given up
    const size_t n_carry = lp->live_chunks < 0 ? c.size() : std::min(c.size(), (size_t)lp->live_chunks);
    if ((rc_copy = copy_chunks(lp, 1, slot_host(lp, a.out_host_slot), c, n_carry, os))) return rc_copy;
    PIE_HIP(hipEventRecord(lp->ev_out, os));
    lp->out_carried = (int32_t)n_carry;
    ++lp->stats.n_swap_out;
    lp->stats.bytes_out += n_carry * lp->chunk_bytes;
  }
  if (a.in_layer >= 0) {
    int32_t n_data = 0;
    int rc = pie_chunk_book_enters_gpu(lp->book, a.in_layer, &n_data);
    if (rc) return rc;
    if ((rc = send_map(lp, a.in_layer, cs))) return rc;
    const std::vector<int32_t>& c = lp->book->chunks[a.in_layer];
    if ((rc = copy_chunks(lp, 0, slot_host(lp, a.in_host_slot), c, (size_t)n_data, is))) return rc;
    PIE_HIP(hipEventRecord(lp->ev_in, is));
    ++lp->stats.n_swap_in;
    lp->stats.bytes_in += (uint64_t)n_data * lp->chunk_bytes;
    if (a.forced_in) ++lp->stats.n_forced_in;
  }
  return PIE_OK;
}

}  // namespace

extern "C" {

int pie_elastic_bytes_required(pie_pool* pool, int32_t chunk_blocks, int32_t max_chunks_per_layer,
                               int32_t n_host_slots, size_t* d_bytes, size_t* h_bytes) {
  if (!pool || chunk_blocks <= 0 || max_chunks_per_layer <= 0 || n_host_slots < 0) return PIE_EINVAL;
  if (d_bytes) *d_bytes = (size_t)pool->cfg.n_layers * max_chunks_per_layer * chunk_blocks * sizeof(int32_t);
  if (h_bytes) *h_bytes = (size_t)n_host_slots * max_chunks_per_layer * chunk_blocks * pool->block_bytes;
  return PIE_OK;
}

int pie_elastic_create(pie_pool* pool, int32_t chunk_blocks, int32_t max_chunks_per_layer, int32_t n_host_slots,
                       void* d_work, size_t d_bytes, void* h_pinned, size_t h_bytes, pie_elastic_pool** out) {
  if (!pool || !out || chunk_blocks <= 0) return PIE_EINVAL;
  *out = nullptr;
  if (!pool->device) return PIE_ESTATE;
  const pie_config& c = pool->cfg;
  if (c.n_host_blocks != 0 || c.n_stage_blocks != 0 || c.n_gpu_blocks % chunk_blocks) return PIE_EINVAL;
  if (pool->d_layer_stride != (size_t)c.n_gpu_blocks * pool->block_bytes) return PIE_EINVAL;
  const int32_t k0 = c.n_gpu_blocks / chunk_blocks;
  if (max_chunks_per_layer < k0 || max_chunks_per_layer > pie::kMaxLayerChunks) return PIE_EINVAL;
  size_t need_d = 0, need_h = 0;
  pie_elastic_bytes_required(pool, chunk_blocks, max_chunks_per_layer, n_host_slots, &need_d, &need_h);
  if (!d_work || d_bytes < need_d || (uintptr_t)d_work % 16) return PIE_ENOMEM;
  if (n_host_slots > 0 && (!h_pinned || h_bytes < need_h)) return PIE_ENOMEM;
  pie_elastic_pool* lp = new (std::nothrow) pie_elastic_pool();
  if (!lp) return PIE_ENOMEM;
  lp->pool = pool;
  lp->n = c.n_layers;
  lp->C = chunk_blocks;
  lp->k_cap = max_chunks_per_layer;
  lp->H = max_chunks_per_layer * chunk_blocks;
  lp->N = c.n_layers * k0;
  lp->n_host_slots = n_host_slots;
  lp->chunk_bytes = (size_t)chunk_blocks * pool->block_bytes;
  lp->host_slot_bytes = (size_t)max_chunks_per_layer * lp->chunk_bytes;
  lp->h_base = (char*)h_pinned;
  lp->d_maps = (int32_t*)d_work;
  lp->stats = pie_layer_stats();
  int rc = pie_layer_sched_create(lp->n, lp->n, n_host_slots, 0, nullptr, &lp->sched);
  if (!rc) rc = pie_chunk_book_create(lp->n, lp->N, max_chunks_per_layer, &lp->book);
  if (rc) {
    pie_elastic_destroy(lp);
    return rc;
  }
  lp->ev_layer.assign(lp->n, nullptr);
  lp->ev_layer_rec.assign(lp->n, 0);
  bool ok = hipEventCreateWithFlags(&lp->ev_in, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&lp->ev_out, hipEventDisableTiming) == hipSuccess;
  for (hipEvent_t& e : lp->ev_layer) ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    pie_elastic_destroy(lp);
    return PIE_EHIP;
  }
  // every layer starts on the GPU in the pool's own layout: layer j in chunks j k0 .. j k0 + k0 - 1
  for (int32_t j = 0; j < lp->n && !rc; ++j) rc = send_map(lp, j, nullptr);
  if (!rc && hipStreamSynchronize(nullptr) != hipSuccess) { (void)hipGetLastError(); rc = PIE_EHIP; }
  if (rc) {
    pie_elastic_destroy(lp);
    return rc;
  }
  *out = lp;
  return PIE_OK;
}

int pie_elastic_destroy(pie_elastic_pool* lp) {
  if (!lp) return PIE_EINVAL;
  if (lp->sched) {
    if (lp->sched->moving_in >= 0 && lp->ev_in) (void)hipEventSynchronize(lp->ev_in);
    if (lp->sched->moving_out >= 0 && lp->ev_out) (void)hipEventSynchronize(lp->ev_out);
    pie_layer_sched_destroy(lp->sched);
  }
  if (lp->book) pie_chunk_book_destroy(lp->book);
  if (lp->ev_in) (void)hipEventDestroy(lp->ev_in);
  if (lp->ev_out) (void)hipEventDestroy(lp->ev_out);
  for (hipEvent_t e : lp->ev_layer)
    if (e) (void)hipEventDestroy(e);
  delete lp;
  return PIE_OK;
}

int pie_elastic_settle_sync(pie_elastic_pool* lp, void* compute_stream) {
  if (!lp) return PIE_EINVAL;
  if (lp->sched->moving_in >= 0) {
    PIE_HIP(hipEventSynchronize(lp->ev_in));
    pie_layer_sched_complete(lp->sched, 0);
  }
  if (lp->sched->moving_out >= 0) {
    PIE_HIP(hipEventSynchronize(lp->ev_out));
    int rc = on_out_complete(lp, (hipStream_t)compute_stream);
    if (rc) return rc;
  }
  return PIE_OK;
}

int pie_elastic_set_layers_on_cpu(pie_elastic_pool* lp, int32_t m, int32_t blocks_in_use_end, void* compute_stream) {
  if (!lp || m < 0 || m >= lp->n || blocks_in_use_end < 0) return PIE_EINVAL;
  if (m > 0 && m + 2 > lp->n_host_slots) return PIE_EINVAL;          // the protocol's two CPU-side buffers
  hipStream_t cs = (hipStream_t)compute_stream;
  int rc = pie_elastic_settle_sync(lp, compute_stream);
  if (rc) return rc;
  std::vector<uint8_t> changed(lp->n, 0);
  rc = book_set(lp->book, m, (blocks_in_use_end + lp->C - 1) / lp->C, changed.data());
  if (rc) return rc;                                                  // PIE_ESTATE: hidden, nothing else changed
  for (int32_t j = 0; j < lp->n; ++j)
    if (changed[j] && (rc = send_map(lp, j, cs))) return rc;
  return pie_layer_sched_set_gpu_slots(lp->sched, lp->n - m);
}

int pie_elastic_set_live_blocks(pie_elastic_pool* lp, int32_t blocks_in_use_end) {
  if (!lp || blocks_in_use_end < -1) return PIE_EINVAL;
  lp->live_chunks = blocks_in_use_end < 0 ? -1 : (blocks_in_use_end + lp->C - 1) / lp->C;
  return PIE_OK;
}

int pie_elastic_move_blocks(pie_elastic_pool* lp, int32_t n, const int32_t* src, const int32_t* dst,
                            void* compute_stream) {
  if (!lp || n < 0 || (n > 0 && (!src || !dst))) return PIE_EINVAL;
  if (n == 0) return PIE_OK;
  std::vector<uint8_t> is_src(lp->H, 0), is_dst(lp->H, 0);
  for (int32_t i = 0; i < n; ++i) {
    if (src[i] < 0 || src[i] >= lp->H || dst[i] < 0 || dst[i] >= lp->H) return PIE_EINVAL;
    if (is_src[src[i]] || is_dst[dst[i]]) return PIE_EINVAL;        // each block moves once, to a place of its own
    is_src[src[i]] = is_dst[dst[i]] = 1;
  }
  for (int32_t i = 0; i < n; ++i)
    if (is_src[dst[i]]) return PIE_EINVAL;                           // no chains: a target is not itself moved
  hipStream_t cs = (hipStream_t)compute_stream;
  int rc = pie_elastic_settle_sync(lp, compute_stream);
  if (rc) return rc;
  pie_chunk_book* b = lp->book;
  for (int32_t j = 0; j < lp->n; ++j)                                // every resident layer must have the targets
    if (b->resident[j])
      for (int32_t i = 0; i < n; ++i)
        if (dst[i] / lp->C >= (int32_t)b->chunks[j].size() || src[i] / lp->C >= (int32_t)b->chunks[j].size())
          return PIE_ESTATE;
  const size_t bb = lp->pool->block_bytes;
  for (int32_t j = 0; j < lp->n; ++j) {
    if (b->resident[j]) {
      const std::vector<int32_t>& c = b->chunks[j];
      auto slot = [&](int32_t h) { return c[h / lp->C] * lp->C + h % lp->C; };
      pie::SwapPairs pairs;
      for (int32_t i = 0; i < n;) {
        pairs.n = 0;
        for (; i < n && pairs.n < pie::kSwapPairs; ++i) {
          pairs.src[pairs.n] = slot(src[i]);
          pairs.dst[pairs.n] = slot(dst[i]);
          ++pairs.n;
        }
        if ((rc = pie::launch_swap_copy(lp->pool->d_kv, lp->pool->d_kv, bb, pairs, 32, cs, 25604))) return rc;
      }
      PIE_HIP(hipEventRecord(lp->ev_layer[j], cs));                  // a later swap-out of the layer waits for this
      lp->ev_layer_rec[j] = 1;
    } else {
      // in CPU memory: inside its image; a source beyond what it carries holds nothing for this layer yet
      char* img = slot_host(lp, lp->sched->table[j].host_slot);
      for (int32_t i = 0; i < n; ++i) {
        if (src[i] / lp->C >= b->image[j]) continue;
        std::memcpy(img + (size_t)dst[i] * bb, img + (size_t)src[i] * bb, bb);
        b->image[j] = std::max(b->image[j], dst[i] / lp->C + 1);
      }
    }
  }
  return PIE_OK;
}

int pie_elastic_capacity(pie_elastic_pool* lp, int32_t* out_visible_blocks, int32_t* out_target_blocks,
                         int32_t* out_layers_on_cpu) {
  if (!lp) return PIE_EINVAL;
  int32_t v = 0, t = 0, m = 0;
  pie_chunk_book_capacity(lp->book, &v, &t, nullptr, &m);
  if (out_visible_blocks) *out_visible_blocks = v * lp->C;
  if (out_target_blocks) *out_target_blocks = t * lp->C;
  if (out_layers_on_cpu) *out_layers_on_cpu = m;
  return PIE_OK;
}

int pie_elastic_blocks_for(pie_elastic_pool* lp, int32_t m, int32_t* out_blocks) {
  if (!lp || !out_blocks || m < 0 || m >= lp->n) return PIE_EINVAL;
  *out_blocks = lp->book->target_for(m) * lp->C;
  return PIE_OK;
}

int pie_elastic_layer(pie_elastic_pool* lp, int32_t layer, int32_t* out_where, int32_t* out_n_chunks,
                      int32_t* out_chunks, void** out_host_ptr) {
  if (!lp || layer < 0 || layer >= lp->n || !out_where || !out_n_chunks) return PIE_EINVAL;
  const pie_layer_entry& e = lp->sched->table[layer];
  if (e.state == PIE_LAYER_GPU) {
    *out_where = PIE_WHERE_GPU;
    *out_n_chunks = (int32_t)lp->book->chunks[layer].size();
    if (out_chunks) std::copy(lp->book->chunks[layer].begin(), lp->book->chunks[layer].end(), out_chunks);
    if (out_host_ptr) *out_host_ptr = nullptr;
  } else if (e.state == PIE_LAYER_HOST) {
    *out_where = PIE_WHERE_HOST;
    *out_n_chunks = lp->book->image[layer];
    if (out_host_ptr) *out_host_ptr = slot_host(lp, e.host_slot);
  } else {
    return PIE_ESTATE;                                                // in flight: settle first
  }
  return PIE_OK;
}

int pie_elastic_table(pie_elastic_pool* lp, pie_layer_entry* out) {
  if (!lp) return PIE_EINVAL;
  return pie_layer_sched_table(lp->sched, out);
}

int pie_elastic_stats(pie_elastic_pool* lp, pie_layer_stats* out) {
  if (!lp || !out) return PIE_EINVAL;
  *out = lp->stats;
  return PIE_OK;
}

int pie_elastic_step(pie_elastic_pool* lp, const void* d_q_all, const void* d_k_new, const void* d_v_new,
                     const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_ctx_lens, int32_t batch,
                     void* d_out_all, void* compute_stream, void* swap_in_stream, void* swap_out_stream) {
  if (!lp || batch < 0 || max_blocks <= 0) return PIE_EINVAL;
  if (batch == 0) return PIE_OK;
  if (!d_q_all || !d_block_table || !d_ctx_lens || !d_out_all) return PIE_EINVAL;
  if ((d_k_new == nullptr) != (d_v_new == nullptr)) return PIE_EINVAL;
  pie_pool* p = lp->pool;
  if (batch > p->cfg.max_batch || max_blocks > p->cfg.max_blocks_per_seq) return PIE_EINVAL;
  hipStream_t cs = (hipStream_t)compute_stream, is = (hipStream_t)swap_in_stream, os = (hipStream_t)swap_out_stream;
  const size_t q_stride = (size_t)batch * p->cfg.n_q_heads * p->cfg.head_dim * p->elem_bytes;
  const size_t kv_stride = (size_t)batch * p->cfg.n_kv_heads * p->cfg.head_dim * p->elem_bytes;
  pie::note_stream(p, cs);
  pie::note_stream(p, is);
  pie::note_stream(p, os);
  int rc;
  // with a new token the attention takes it from the new rows, the rest of the context from the cache
  if ((rc = pie::launch_attn_plan(p, d_ctx_lens, batch, max_blocks, cs, false, nullptr, d_k_new != nullptr))) return rc;
  for (int32_t k = 0; k < lp->n; ++k) {
    // the presence check: wait until the layer is physically on the GPU
    if ((rc = poll_moves(lp, cs))) return rc;
    pie_layer_action act;
    const auto t_wait0 = std::chrono::steady_clock::now();
    bool waited = false;
    for (;;) {
      if ((rc = pie_layer_sched_present(lp->sched, k, &act))) return rc;
      if ((rc = start_moves(lp, act, cs, is, os))) return rc;
      if (act.wait == PIE_LAYER_WAIT_NONE) break;
      waited = true;
      if (act.wait == PIE_LAYER_WAIT_IN) {
        PIE_HIP(hipEventSynchronize(lp->ev_in));
        pie_layer_sched_complete(lp->sched, 0);
      } else {
        PIE_HIP(hipEventSynchronize(lp->ev_out));
        if ((rc = on_out_complete(lp, cs))) return rc;
      }
    }
    if (waited)
      lp->stats.stall_ms += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_wait0).count();
    // the layer's blocks through its own map: every slot of the GPU memory counts as resident
    pie::LayerView view{p->d_kv, lp->d_maps + (size_t)k * lp->H, lp->H, lp->N * lp->C};
    if (d_k_new) {
      if ((rc = pie::launch_kv_append(p, k, 1, (const char*)d_k_new + k * kv_stride, (const char*)d_v_new + k * kv_stride,
                                      d_block_table, max_blocks, d_ctx_lens, batch, pie::kAppendGpuStrict, cs, &view)))
        return rc;
    }
    if ((rc = pie::launch_attn_resolve(p, d_block_table, d_ctx_lens, batch, max_blocks, true, false, false, false, cs,
                                       &view)))
      return rc;
    if ((rc = pie::launch_attn_decode(p, k, (const char*)d_q_all + k * q_stride, max_blocks, d_ctx_lens, batch,
                                      (char*)d_out_all + k * q_stride, cs, nullptr, nullptr, k, nullptr, &view, nullptr,
                                      nullptr, d_k_new ? (const char*)d_k_new + k * kv_stride : nullptr,
                                      d_v_new ? (const char*)d_v_new + k * kv_stride : nullptr)))
      return rc;
    if (p->layer_compute_us > 0.f && (rc = pie::launch_busy(p->layer_compute_us, p->wall_clock_khz, cs))) return rc;
    PIE_HIP(hipEventRecord(lp->ev_layer[k], cs));
    lp->ev_layer_rec[k] = 1;
    // The protocol's two checks belong to the moment this layer starts computing, which is when the previous
    // one has ended: the host waits for that (this layer's work is already queued behind it), then looks.
    if (lp->prev_layer >= 0 && lp->prev_layer != k) PIE_HIP(hipEventSynchronize(lp->ev_layer[lp->prev_layer]));
    if ((rc = poll_moves(lp, cs))) return rc;
    if ((rc = pie_layer_sched_policy(lp->sched, k, &act))) return rc;
    if ((rc = start_moves(lp, act, cs, is, os))) return rc;
    lp->prev_layer = k;
  }
  ++lp->stats.n_steps;
  return PIE_OK;
}

}  // extern "C"
