// Layer-granular swapping as the paper states it: a mapping table from logical layer to CPU / GPU layer slot,
// updated in two phases around a background copy (Section 3.2), and the protocol run at the beginning of
// every layer's computation (Section 3.3): if the previous swap-in has finished, bring in the hottest layer
// in CPU memory (the one accessed soonest) when a GPU slot is free; if the previous swap-out has finished,
// send out the coldest layer on the GPU (the one accessed last, i.e. the layer that just finished), unless
// every layer in CPU memory is colder still; and before a layer computes, wait until it is physically present.
//
// pie_layer_sched is the protocol as pure host logic (no GPU): the caller reports completed moves and asks,
// per layer, what to wait for and what to start.  pie_layer_pool drives it over a pool whose "layers" are
// the GPU's physical layer slots, with whole-layer copy-engine transfers.  Readings where the text is
// silent: swap-in is considered before swap-out, and a swap-out starts only when no GPU slot is free (it
// exists to make room for the next swap-in); coldness is the number of layer computations until the
// next access, (j - k) mod n while layer k computes; layers in flight are neither candidates nor counted as
// "in CPU memory"; a slot is released when the copy that leaves it has completed; a layer that is needed
// while it is neither present nor on its way is brought back at once.

#include <chrono>
#include <new>
#include <vector>

#include "pie_internal.h"

#include "pie_layer_core.h"

static void clear_action(pie_layer_action* a) {
  a->wait = PIE_LAYER_WAIT_NONE;
  a->gpu_slot = -1;
  a->in_layer = a->in_gpu_slot = a->in_host_slot = -1;
  a->out_layer = a->out_gpu_slot = a->out_host_slot = -1;
  a->forced_in = 0;
  a->out_skipped = a->in_skipped = PIE_LAYER_SKIP_NOT;
}

extern "C" {

int pie_layer_sched_create(int32_t n_layers, int32_t n_gpu_slots, int32_t n_host_slots, int32_t n_on_host,
                           const int32_t* on_host, pie_layer_sched** out) {
  if (!out || n_layers <= 0 || n_gpu_slots <= 0 || n_host_slots < 0 || n_on_host < 0 || (n_on_host > 0 && !on_host))
    return PIE_EINVAL;
  std::vector<uint8_t> host(n_layers, 0);
  int32_t n_host = 0;
  for (int32_t i = 0; i < n_on_host; ++i) {
    if (on_host[i] < 0 || on_host[i] >= n_layers) return PIE_EINVAL;
    if (!host[on_host[i]]) ++n_host;
    host[on_host[i]] = 1;
  }
  if (n_host > n_host_slots || n_layers - n_host > n_gpu_slots) return PIE_ENOMEM;
  pie_layer_sched* s = new (std::nothrow) pie_layer_sched();
  if (!s) return PIE_ENOMEM;
  s->n = n_layers;
  s->n_gpu_total = s->n_enabled = s->target = n_gpu_slots;
  s->n_host_total = n_host_slots;
  for (int32_t i = 0; i < n_gpu_slots; ++i) s->free_gpu.push_back(i);
  for (int32_t i = 0; i < n_host_slots; ++i) s->free_host.push_back(i);
  s->table.resize(n_layers);
  for (int32_t j = 0; j < n_layers; ++j) {                  // lowest free slot first, in layer order
    pie_layer_entry& e = s->table[j];
    e.gpu_slot = e.host_slot = -1;
    if (host[j]) {
      e.state = PIE_LAYER_HOST;
      e.host_slot = pie_layer_sched::take_lowest(s->free_host);
    } else {
      e.state = PIE_LAYER_GPU;
      e.gpu_slot = pie_layer_sched::take_lowest(s->free_gpu);
    }
  }
  *out = s;
  return PIE_OK;
}

int pie_layer_sched_destroy(pie_layer_sched* s) {
  if (!s) return PIE_EINVAL;
  delete s;
  return PIE_OK;
}

int pie_layer_sched_complete(pie_layer_sched* s, int32_t which) {
  if (!s || (which != 0 && which != 1)) return PIE_EINVAL;
  if (which == 0) {                                          // phase two of a swap-in
    if (s->moving_in < 0) return PIE_ESTATE;
    pie_layer_entry& e = s->table[s->moving_in];
    pie_layer_sched::give_back(s->free_host, e.host_slot);
    e.host_slot = -1;
    e.state = PIE_LAYER_GPU;
    s->moving_in = -1;
  } else {
    if (s->moving_out < 0) return PIE_ESTATE;
    pie_layer_entry& e = s->table[s->moving_out];
    pie_layer_sched::give_back(s->free_gpu, e.gpu_slot);
    e.gpu_slot = -1;
    e.state = PIE_LAYER_HOST;
    s->moving_out = -1;
    s->rebalance();
  }
  return PIE_OK;
}

int pie_layer_sched_set_gpu_slots(pie_layer_sched* s, int32_t n_gpu_slots) {
  if (!s || n_gpu_slots < 1 || n_gpu_slots > s->n_gpu_total) return PIE_EINVAL;
  // the layers that do not fit the GPU slots need a CPU slot each, plus the two in flight
  if (s->n - n_gpu_slots + 2 > s->n_host_total) return PIE_EINVAL;
  s->target = n_gpu_slots;
  s->rebalance();
  return PIE_OK;
}

int pie_layer_sched_present(pie_layer_sched* s, int32_t k, pie_layer_action* a) {
  if (!s || !a || k < 0 || k >= s->n) return PIE_EINVAL;
  clear_action(a);
  pie_layer_entry& e = s->table[k];
  switch (e.state) {
    case PIE_LAYER_GPU:
      a->gpu_slot = e.gpu_slot;
      return PIE_OK;
    case PIE_LAYER_MOVING_IN:
      a->wait = PIE_LAYER_WAIT_IN;
      return PIE_OK;
    case PIE_LAYER_MOVING_OUT:                               // leaving while it is needed: let it finish first
      a->wait = PIE_LAYER_WAIT_OUT;
      return PIE_OK;
    default: break;
  }
  // in CPU memory and not on its way
  if (s->moving_in >= 0) {
    a->wait = PIE_LAYER_WAIT_IN;                             // the link is taken: that transfer first
    return PIE_OK;
  }
  if (s->free_gpu.empty()) {
    if (s->moving_out < 0) {
      const int32_t victim = s->coldest_on_gpu(k);
      if (victim < 0 || s->free_host.empty()) return PIE_ENOMEM;
      s->start_out(victim, a);
    }
    a->wait = PIE_LAYER_WAIT_OUT;
    return PIE_OK;
  }
  s->start_in(k, a);
  a->forced_in = 1;
  a->wait = PIE_LAYER_WAIT_IN;
  return PIE_OK;
}

int pie_layer_sched_policy(pie_layer_sched* s, int32_t k, pie_layer_action* a) {
  if (!s || !a || k < 0 || k >= s->n) return PIE_EINVAL;
  if (s->table[k].state != PIE_LAYER_GPU) return PIE_ESTATE;
  clear_action(a);
  a->gpu_slot = s->table[k].gpu_slot;
  // swap-in of the hottest layer in CPU memory
  if (s->moving_in >= 0) {
    a->in_skipped = PIE_LAYER_SKIP_BUSY;
  } else {
    const int32_t cand = s->hottest_on_host(k);
    if (cand < 0)
      a->in_skipped = PIE_LAYER_SKIP_NONE;
    else if (s->free_gpu.empty())
      a->in_skipped = PIE_LAYER_SKIP_NO_SLOT;
    else
      s->start_in(cand, a);
  }
  // swap-out of the coldest layer on the GPU
  if (s->moving_out >= 0) {
    a->out_skipped = PIE_LAYER_SKIP_BUSY;
  } else {
    const int32_t cand = s->coldest_on_gpu(k);
    if (cand < 0) {
      a->out_skipped = PIE_LAYER_SKIP_NONE;
    } else {
      bool all_colder = true;                                // also when nothing is in CPU memory at all
      for (int32_t j = 0; j < s->n; ++j)
        if (s->table[j].state == PIE_LAYER_HOST && s->distance(j, k) <= s->distance(cand, k)) all_colder = false;
      if (all_colder && !s->oversubscribed())
        a->out_skipped = PIE_LAYER_SKIP_COLDER_ON_HOST;
      else if (!s->free_gpu.empty())
        a->out_skipped = PIE_LAYER_SKIP_ROOM_LEFT;           // a GPU slot is free: nothing has to leave
      else if (s->free_host.empty())
        a->out_skipped = PIE_LAYER_SKIP_NO_SLOT;
      else
        s->start_out(cand, a);
    }
  }
  return PIE_OK;
}

int pie_layer_sched_table(pie_layer_sched* s, pie_layer_entry* out) {
  if (!s || !out) return PIE_EINVAL;
  for (int32_t j = 0; j < s->n; ++j) out[j] = s->table[j];
  return PIE_OK;
}

}  // extern "C"

// ---------------------------------------------------------------------------------------------------------
// the driver: logical layers over a pool of GPU layer slots and a pinned array of CPU layer slots
// ---------------------------------------------------------------------------------------------------------

struct pie_layer_pool {
  pie_pool* pool = nullptr;            // its n_layers are the GPU layer slots; every block is GPU-homed
  pie_layer_sched* sched = nullptr;
  int32_t n_layers = 0, n_host_slots = 0;
  char* h_base = nullptr;
  size_t layer_bytes = 0;
  hipEvent_t ev_in = nullptr, ev_out = nullptr;
  std::vector<hipEvent_t> ev_slot;     // last compute work on a GPU slot
  std::vector<uint8_t> ev_slot_rec;
  pie_layer_stats stats;
  int32_t prev_slot = -1;              // GPU slot of the layer computed last
};

namespace {

using pie::g_last_hip_error;

char* slot_dev(const pie_layer_pool* lp, int32_t slot) { return lp->pool->d_kv + (size_t)slot * lp->pool->d_layer_stride; }
char* slot_host(const pie_layer_pool* lp, int32_t slot) { return lp->h_base + (size_t)slot * lp->layer_bytes; }

// Reports finished transfers to the protocol (phase two of the mapping-table update).
int poll_moves(pie_layer_pool* lp) {
  pie_layer_sched* s = lp->sched;
  if (s->moving_in >= 0) {
    hipError_t e = hipEventQuery(lp->ev_in);
    if (e == hipSuccess) pie_layer_sched_complete(s, 0);
    else if (e != hipErrorNotReady) { g_last_hip_error = (int)e; (void)hipGetLastError(); return PIE_EHIP; }
    else (void)hipGetLastError();
  }
  if (s->moving_out >= 0) {
    hipError_t e = hipEventQuery(lp->ev_out);
    if (e == hipSuccess) pie_layer_sched_complete(s, 1);
    else if (e != hipErrorNotReady) { g_last_hip_error = (int)e; (void)hipGetLastError(); return PIE_EHIP; }
    else (void)hipGetLastError();
  }
  return PIE_OK;
}

// Starts the transfers an action names.  All ordering is done on the host (the copy engine's streams carry
// no waits): a swap-out first waits for the last computation on its GPU slot; a swap-in goes into a slot
// whose previous tenant's swap-out the host has already seen complete.
int start_moves(pie_layer_pool* lp, const pie_layer_action& a, hipStream_t is, hipStream_t os) {
  if (a.out_layer >= 0) {
    if (lp->ev_slot_rec[a.out_gpu_slot]) PIE_HIP(hipEventSynchronize(lp->ev_slot[a.out_gpu_slot]));
    PIE_HIP(hipMemcpyAsync(slot_host(lp, a.out_host_slot), slot_dev(lp, a.out_gpu_slot), lp->layer_bytes,
                           hipMemcpyDeviceToHost, os));
    PIE_HIP(hipEventRecord(lp->ev_out, os));
    ++lp->stats.n_swap_out;
    lp->stats.bytes_out += lp->layer_bytes;
  }
  if (a.in_layer >= 0) {
    PIE_HIP(hipMemcpyAsync(slot_dev(lp, a.in_gpu_slot), slot_host(lp, a.in_host_slot), lp->layer_bytes,
                           hipMemcpyHostToDevice, is));
    PIE_HIP(hipEventRecord(lp->ev_in, is));
    ++lp->stats.n_swap_in;
    lp->stats.bytes_in += lp->layer_bytes;
    if (a.forced_in) ++lp->stats.n_forced_in;
  }
  return PIE_OK;
}

}  // namespace

extern "C" {

int pie_layer_pool_bytes_required(pie_pool* pool, int32_t n_host_slots, size_t* h_bytes) {
  if (!pool || n_host_slots < 0 || !h_bytes) return PIE_EINVAL;
  *h_bytes = (size_t)n_host_slots * pool->cfg.n_gpu_blocks * pool->block_bytes;
  return PIE_OK;
}

int pie_layer_pool_create(pie_pool* pool, int32_t n_layers, int32_t n_host_slots, void* h_pinned, size_t h_bytes,
                          int32_t n_on_host, const int32_t* on_host, pie_layer_pool** out) {
  if (!pool || !out) return PIE_EINVAL;
  if (!pool->device) return PIE_ESTATE;
  if (pool->cfg.n_host_blocks != 0 || pool->cfg.n_stage_blocks != 0) return PIE_EINVAL;   // layers move whole
  const size_t layer_bytes = (size_t)pool->cfg.n_gpu_blocks * pool->block_bytes;
  if (pool->d_layer_stride != layer_bytes) return PIE_EINVAL;
  if (n_host_slots > 0 && (!h_pinned || h_bytes < (size_t)n_host_slots * layer_bytes)) return PIE_ENOMEM;
  pie_layer_pool* lp = new (std::nothrow) pie_layer_pool();
  if (!lp) return PIE_ENOMEM;
  int rc = pie_layer_sched_create(n_layers, pool->cfg.n_layers, n_host_slots, n_on_host, on_host, &lp->sched);
  if (rc) {
    delete lp;
    return rc;
  }
  lp->pool = pool;
  lp->n_layers = n_layers;
  lp->n_host_slots = n_host_slots;
  lp->h_base = (char*)h_pinned;
  lp->layer_bytes = layer_bytes;
  lp->stats = pie_layer_stats();
  lp->ev_slot.assign(pool->cfg.n_layers, nullptr);
  lp->ev_slot_rec.assign(pool->cfg.n_layers, 0);
  bool ok = hipEventCreateWithFlags(&lp->ev_in, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&lp->ev_out, hipEventDisableTiming) == hipSuccess;
  for (hipEvent_t& e : lp->ev_slot) ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    pie_layer_pool_destroy(lp);
    return PIE_EHIP;
  }
  *out = lp;
  return PIE_OK;
}

int pie_layer_pool_destroy(pie_layer_pool* lp) {
  if (!lp) return PIE_EINVAL;
  if (lp->sched) {
    if (lp->sched->moving_in >= 0 && lp->ev_in) (void)hipEventSynchronize(lp->ev_in);
    if (lp->sched->moving_out >= 0 && lp->ev_out) (void)hipEventSynchronize(lp->ev_out);
    pie_layer_sched_destroy(lp->sched);
  }
  if (lp->ev_in) (void)hipEventDestroy(lp->ev_in);
  if (lp->ev_out) (void)hipEventDestroy(lp->ev_out);
  for (hipEvent_t e : lp->ev_slot)
    if (e) (void)hipEventDestroy(e);
  delete lp;
  return PIE_OK;
}

int pie_layer_pool_table(pie_layer_pool* lp, pie_layer_entry* out) {
  if (!lp) return PIE_EINVAL;
  return pie_layer_sched_table(lp->sched, out);
}

int pie_layer_pool_set_gpu_slots(pie_layer_pool* lp, int32_t n_gpu_slots) {
  if (!lp) return PIE_EINVAL;
  return pie_layer_sched_set_gpu_slots(lp->sched, n_gpu_slots);
}

int pie_layer_pool_settle_sync(pie_layer_pool* lp) {
  if (!lp) return PIE_EINVAL;
  if (lp->sched->moving_in >= 0) {
    PIE_HIP(hipEventSynchronize(lp->ev_in));
    pie_layer_sched_complete(lp->sched, 0);
  }
  if (lp->sched->moving_out >= 0) {
    PIE_HIP(hipEventSynchronize(lp->ev_out));
    pie_layer_sched_complete(lp->sched, 1);
  }
  return PIE_OK;
}

int pie_layer_pool_address(pie_layer_pool* lp, int32_t layer, int32_t* out_where, void** out_ptr) {
  if (!lp || layer < 0 || layer >= lp->n_layers || !out_where || !out_ptr) return PIE_EINVAL;
  const pie_layer_entry& e = lp->sched->table[layer];
  if (e.state == PIE_LAYER_GPU) {
    *out_where = PIE_WHERE_GPU;
    *out_ptr = slot_dev(lp, e.gpu_slot);
  } else if (e.state == PIE_LAYER_HOST) {
    *out_where = PIE_WHERE_HOST;
    *out_ptr = slot_host(lp, e.host_slot);
  } else {
    return PIE_ESTATE;                                       // in flight: settle first
  }
  return PIE_OK;
}

int pie_layer_pool_stats(pie_layer_pool* lp, pie_layer_stats* out) {
  if (!lp || !out) return PIE_EINVAL;
  *out = lp->stats;
  return PIE_OK;
}

int pie_layer_step(pie_layer_pool* lp, const void* d_q_all, const void* d_k_new, const void* d_v_new,
                   const int32_t* d_block_table, int32_t max_blocks, const int32_t* d_ctx_lens, int32_t batch,
                   void* d_out_all, void* compute_stream, void* swap_in_stream, void* swap_out_stream) {
  if (!lp || batch < 0 || max_blocks <= 0) return PIE_EINVAL;
  if (batch == 0) return PIE_OK;
  if (!d_q_all || !d_block_table || !d_ctx_lens || !d_out_all) return PIE_EINVAL;
  if ((d_k_new == nullptr) != (d_v_new == nullptr)) return PIE_EINVAL;
  pie_pool* p = lp->pool;
  if (batch > p->cfg.max_batch || max_blocks > p->cfg.max_blocks_per_seq) return PIE_EINVAL;
  hipStream_t cs = (hipStream_t)compute_stream, is = (hipStream_t)swap_in_stream, os = (hipStream_t)swap_out_stream;
  const int32_t n_slots = p->cfg.n_layers;
  const size_t q_stride = (size_t)batch * p->cfg.n_q_heads * p->cfg.head_dim * p->elem_bytes;
  const size_t kv_stride = (size_t)batch * p->cfg.n_kv_heads * p->cfg.head_dim * p->elem_bytes;
  pie::note_stream(p, cs);
  pie::note_stream(p, is);
  pie::note_stream(p, os);
  int rc;
  if ((rc = pie::flush_map(p, cs))) return rc;
  for (int32_t k = 0; k < lp->n_layers; ++k) {
    // one ticket counter per launch since the last planning kernel; there are as many as GPU slots
    if (k % n_slots == 0) {
      // with a new token the attention takes it from the new rows, the rest of the context from the cache
      if ((rc = pie::launch_attn_plan(p, d_ctx_lens, batch, max_blocks, cs, false, nullptr, d_k_new != nullptr))) return rc;
      if (k == 0 && (rc = pie::launch_attn_resolve(p, d_block_table, d_ctx_lens, batch, max_blocks, true, false, true,
                                                   false, cs)))
        return rc;
    }
    // the presence check: wait until the layer is physically on the GPU
    if ((rc = poll_moves(lp))) return rc;
    pie_layer_action act;
    const auto t_wait0 = std::chrono::steady_clock::now();
    bool waited = false;
    for (;;) {
      if ((rc = pie_layer_sched_present(lp->sched, k, &act))) return rc;
      if ((rc = start_moves(lp, act, is, os))) return rc;
      if (act.wait == PIE_LAYER_WAIT_NONE) break;
      waited = true;
      if (act.wait == PIE_LAYER_WAIT_IN) {
        PIE_HIP(hipEventSynchronize(lp->ev_in));
        pie_layer_sched_complete(lp->sched, 0);
      } else {
        PIE_HIP(hipEventSynchronize(lp->ev_out));
        pie_layer_sched_complete(lp->sched, 1);
      }
    }
    if (waited)
      lp->stats.stall_ms += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_wait0).count();
    const int32_t slot = act.gpu_slot;
    if (d_k_new) {
      if ((rc = pie::launch_kv_append(p, slot, 1, (const char*)d_k_new + k * kv_stride, (const char*)d_v_new + k * kv_stride,
                                      d_block_table, max_blocks, d_ctx_lens, batch, pie::kAppendGpuStrict, cs)))
        return rc;
    }
    if ((rc = pie::launch_attn_decode(p, slot, (const char*)d_q_all + k * q_stride, max_blocks, d_ctx_lens, batch,
                                      (char*)d_out_all + k * q_stride, cs, nullptr, nullptr, k % n_slots, nullptr,
                                      nullptr, nullptr, nullptr,
                                      d_k_new ? (const char*)d_k_new + k * kv_stride : nullptr,
                                      d_v_new ? (const char*)d_v_new + k * kv_stride : nullptr)))
      return rc;
    if (p->layer_compute_us > 0.f && (rc = pie::launch_busy(p->layer_compute_us, p->wall_clock_khz, cs))) return rc;
    PIE_HIP(hipEventRecord(lp->ev_slot[slot], cs));
    lp->ev_slot_rec[slot] = 1;
    // The protocol's two checks belong to the moment this layer starts computing, which is when the previous
    // one has ended: the host waits for that (this layer's work is already queued behind it), then looks.
    if (lp->prev_slot >= 0 && lp->prev_slot != slot) PIE_HIP(hipEventSynchronize(lp->ev_slot[lp->prev_slot]));
    if ((rc = poll_moves(lp))) return rc;
    if ((rc = pie_layer_sched_policy(lp->sched, k, &act))) return rc;
    if ((rc = start_moves(lp, act, is, os))) return rc;
    lp->prev_slot = slot;
  }
  ++lp->stats.n_steps;
  return PIE_OK;
}

}  // extern "C"
