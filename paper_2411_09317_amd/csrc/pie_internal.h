// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <condition_variable>
#include <cstdint>
#include <deque>
#include <mutex>
#include <set>
#include <thread>
#include <vector>

#include "pie.h"

namespace pie {

extern thread_local int g_last_hip_error;

#define PIE_HIP(call)                                  \
  do {                                                 \
    hipError_t e_ = (call);                            \
    if (e_ != hipSuccess) {                            \
      ::pie::g_last_hip_error = (int)e_;               \
      (void)hipGetLastError();                         \
      return PIE_EHIP;                                 \
    }                                                  \
  } while (0)

constexpr int kMapPatchPairs = 448;   // (handle, slot) pairs passed by value per patch launch
constexpr int kSwapPairs = 448;       // (src slot, dst slot) pairs passed by value per gather launch
constexpr uint32_t kAlign = 256;

// The clock table of monitoring by device clock: one row of kClockRow 64-bit words per layer, one more row
// whose first word is the moment the step began, then kClockWgs pairs of words per layer for the decode
// kernel's workgroups.  Values are ticks of the device's wall clock.
constexpr int kClockRow = 8;
constexpr int kClockKernelStart = 0;  // first workgroup of the layer's decode kernel started
constexpr int kClockKernelEnd = 1;    // last workgroup of it ended
constexpr int kClockLayerEnd = 2;     // last compute-stream work of the layer ended (decode, reduction, stand-in)
constexpr int kClockInStart = 3;      // (not stamped: a copy's start follows from what it waited for)
constexpr int kClockInEnd = 4;        // the layer's swap-in: its copy has ended
constexpr int kClockOutStart = 5;     // (not stamped)
constexpr int kClockOutEnd = 6;       // the layer's write-back has ended
constexpr int kClockGrid = 7;         // workgroups of the decode kernel that wrote per-workgroup words (0: none)
constexpr int kClockWgs = 2048;       // per-workgroup (first, last moment) pairs per layer, after the rows

struct Home {
  int32_t where = -1;  // PIE_WHERE_* or -1 = unallocated
  int32_t slot = -1;
};

struct LayerEvents {
  hipEvent_t attn_start = nullptr, attn_end = nullptr, k_start = nullptr, k_end = nullptr, in_start = nullptr,
             in_end = nullptr, out_start = nullptr, out_end = nullptr;
  bool in_used = false, out_used = false;
};

struct MapPatch {  // by-value kernel argument
  int32_t n;
  int32_t handle[kMapPatchPairs];
  int32_t slot[kMapPatchPairs];
};

constexpr int kMaxLayerChunks = 512;  // chunks one layer can hold

struct ChunkList {  // by-value kernel argument
  int32_t n;
  int32_t chunk[kMaxLayerChunks];
};

// Where one layer's blocks are when they are not in the pool's own [layer][slot] layout.
struct LayerView {
  char* kv_base;        // base of the memory its slots index
  const int32_t* map;   // device: handle -> slot, -1 = none
  int32_t n_handles, n_slots;
};

// Scratch of one attention call: the planning state (header, ticket counters, item records, slot lists) and
// the split-context partials, laid out for lay_batch sequences of lay_max_blocks blocks.
struct AttnWork {
  int32_t* plan;
  float* ws;
  size_t ws_floats;
  int32_t n_counters;       // ticket counters the planning kernel zeroes
  int32_t lay_batch, lay_max_blocks;
};

// One pie_step call, as handed to the pool's submit thread.
struct StepJob {
  const void* d_q_all;
  const void* d_k_new;
  const void* d_v_new;
  const int32_t* d_block_table;
  int32_t max_blocks;
  const int32_t* d_ctx_lens;
  int32_t batch;
  std::vector<int32_t> prefetch, dirty;
  void* d_out_all;
  hipStream_t cs, is, os;
};

struct SwapPairs {  // by-value kernel argument
  int32_t n;
  int32_t src[kSwapPairs];
  int32_t dst[kSwapPairs];
};

}  // namespace pie

struct pie_pool {
  pie_config cfg;
  bool device = false;          // false: bookkeeping only
  int32_t n_handles = 0;
  int32_t elem_bytes = 0;
  size_t block_bytes = 0;       // one layer of one block
  size_t d_layer_stride = 0;    // bytes between layers in the device pool
  size_t h_layer_stride = 0;
  float scale_log2e = 0.f;

  char* d_kv = nullptr;         // device pool base
  int32_t* d_map[2] = {nullptr, nullptr};   // per staging region: handle -> device slot, or -1
  float* d_ws = nullptr;        // split-context partials
  size_t ws_floats = 0;
  int32_t* d_plan = nullptr;    // attention planning state: header, ticket counters, items, resolved tables
  int32_t n_cu = 256;           // compute units of the device
  uint32_t* d_err = nullptr;    // device error flags
  unsigned long long* d_clock = nullptr;   // clock table: (n_layers + 1) rows of kClockRow words
  char* h_kv = nullptr;         // host pool base (host address)
  char* h_kv_dev = nullptr;     // same memory as seen from the device

  // allocator and residency
  std::set<int32_t> free_handles;
  std::set<int32_t> free_slots[2];
  std::vector<pie::Home> home;
  int32_t n_in_use[2] = {0, 0};

  // staging regions
  std::vector<int32_t> stage_rank[2];       // handle -> rank in the region's list, or -1
  std::vector<int32_t> stage_list[2];       // the region's current list
  int32_t region_layer[2] = {-1, -1};

  // host mirror of the device maps and what still has to be sent
  std::vector<int32_t> map_mirror[2];
  std::vector<int32_t> map_dirty[2];        // handles whose device entry is stale
  std::vector<uint8_t> map_dirty_flag[2];

  // ordering between streams
  hipEvent_t ev_in[2] = {nullptr, nullptr};       // last swap-in into region r
  hipEvent_t ev_read[2] = {nullptr, nullptr};     // last compute work that may touch region r
  hipEvent_t ev_out[2] = {nullptr, nullptr};      // last write-back from region r
  hipEvent_t ev_compute = nullptr;                // last compute work
  hipEvent_t ev_migrate = nullptr;                // last migration
  hipEvent_t ev_map = nullptr;                    // last map update sent on the compute stream
  hipEvent_t ev_append = nullptr;                 // a step's append into the GPU-homed tail blocks (write-back stream)
  bool ev_in_rec[2] = {false, false}, ev_read_rec[2] = {false, false}, ev_out_rec[2] = {false, false};
  bool ev_compute_rec = false, ev_migrate_rec = false, ev_map_rec = false, migrate_pending = false;
  std::vector<hipStream_t> streams_seen;

  // options
  int32_t swap_path = PIE_SWAP_AUTO;
  int32_t attn_partition = 0;     // tokens per work item (one workgroup); 0: the planning kernel chooses
  bool attn_valu = false;         // MHA (one query head per kv head): products on the vector ALU, not the matrix cores
  int32_t swap_wgs = 16;          // workgroups of the gather / scatter kernel
  int32_t swap_shape = 0;         // its threads per workgroup * 100 + loads in flight per lane; 0: by transfer size
  float layer_compute_us = 0.f;   // stand-in for the rest of a layer's compute in pie_step (0 = none)
  int32_t wall_clock_khz = 100000;
  int32_t timing = 0;             // PIE_TIMING_*
  uint32_t last_err_flags = 0;    // device error flags seen by pie_check_errors_sync so far

  // timing of the last step
  std::vector<pie::LayerEvents> lev;
  hipEvent_t ev_step_start = nullptr;
  int32_t step_timed = 0;         // the timing mode the last step ran with
  bool in_on_host[2] = {false, false};   // the region's last swap-in was ordered on the host (copy-engine path)
  bool dma_stream_order = false;         // copy-engine transfers ordered by stream waits instead of on the host
  bool presence_poll = true;             // look for a swap-in's completion from the host before waiting on the stream
  // the first layer's blocks staged ahead, behind the previous step's last layer
  bool cross_step_prefetch = true;
  bool pre_valid = false;         // region 0 holds layer 0's blocks of stage_list[0], nothing has changed since
  int32_t pre_timed = 0;          // timing mode that copy was issued under
  bool step_pre_hit = false;      // the last step found them there
  int32_t step_pre_timed = 0;
  int32_t pre_idx = 0, step_pre_idx = 0;
  hipEvent_t ev_pre_end[2] = {nullptr, nullptr};
  uint64_t bytes_in = 0, bytes_out = 0;

  // Asynchronous submission: pie_step hands the step to a thread of the pool's own, which enqueues it (and does
  // the waiting the copy-engine path needs).  Everything but the job queue is touched by one thread at a time:
  // the caller's thread drains the queue before any other call on the pool.
  int device_id = 0;
  bool async_submit = false;
  std::thread submitter;
  std::mutex submit_mutex;
  std::condition_variable submit_wake, submit_idle;
  std::deque<pie::StepJob> submit_jobs;
  bool submit_busy = false, submit_stop = false;
  int submit_rc = 0, submit_hip = 0;          // first error of a step enqueued by the thread, until reported
};

namespace pie {

// host-side pieces used across files
int submit_drain(pie_pool* p);          // waits for the submit thread to run dry; returns (and clears) its first error
int note_stream(pie_pool* p, hipStream_t s);
int flush_map(pie_pool* p, hipStream_t s);
void map_set(pie_pool* p, int region, int32_t handle, int32_t slot);
inline int32_t stage_slot(const pie_pool* p, int region, int32_t rank) {
  return p->cfg.n_gpu_blocks + region * p->cfg.n_stage_blocks + rank;
}
inline char* d_block(const pie_pool* p, int32_t layer, int32_t slot) {
  return p->d_kv + (size_t)layer * p->d_layer_stride + (size_t)slot * p->block_bytes;
}
inline char* h_block(const pie_pool* p, int32_t layer, int32_t slot) {
  return p->h_kv + (size_t)layer * p->h_layer_stride + (size_t)slot * p->block_bytes;
}

// kernel launchers (pie_kernels.hip)
int launch_busy(double us, int wall_clock_khz, hipStream_t s, unsigned long long* clock_row = nullptr,
                hipEvent_t done = nullptr);
int launch_stamp(unsigned long long* slot, hipStream_t s);
int launch_clock_fold(unsigned long long* rows, int32_t n_layers, hipStream_t s);
int launch_map_fill(int32_t* d_map, int32_t n, int32_t value, hipStream_t s);
int launch_map_patch(int32_t* d_map, const MapPatch& patch, hipStream_t s);
int launch_zero_u32(uint32_t* d, int32_t n, hipStream_t s);
int launch_swap_copy(char* dst_layer_base, const char* src_layer_base, size_t block_bytes, const SwapPairs& pairs,
                     int n_wgs, hipStream_t s, int shape = 0, size_t transfer_bytes = 0);
// which tail blocks an append launch writes (a tail block is GPU-homed, staged for the layer, or neither)
constexpr int32_t kAppendPresent = 0;     // GPU-homed or staged; neither raises NOT_PRESENT
constexpr int32_t kAppendGpuStrict = 1;   // GPU-homed; anything else raises NOT_PRESENT (the layer's region is not valid)
constexpr int32_t kAppendGpuHomed = 2;    // GPU-homed; host-homed tails are left to a kAppendStaged launch
constexpr int32_t kAppendStaged = 3;      // staged copies only; GPU-homed tails were written before
int launch_kv_append(const pie_pool* p, int32_t layer, int32_t n_layers, const void* d_k, const void* d_v,
                     const int32_t* d_table, int32_t max_blocks, const int32_t* d_ctx, int32_t batch,
                     int32_t mode, hipStream_t s, const LayerView* view = nullptr);
int launch_chunk_map_fill(int32_t* d_map, int32_t n_handles, int32_t chunk_blocks, const ChunkList& list, hipStream_t s);
// work: the scratch to use; NULL = the pool's own (in the caller's device buffer)
int launch_attn_plan(const pie_pool* p, const int32_t* d_ctx, int32_t batch, int32_t max_blocks, hipStream_t s,
                     bool reset_clock = false, const AttnWork* work = nullptr, bool without_last = false);
int launch_attn_resolve(const pie_pool* p, const int32_t* d_table, const int32_t* d_ctx, int32_t batch,
                        int32_t max_blocks, bool region0, bool valid0, bool region1, bool valid1, hipStream_t s,
                        const LayerView* view = nullptr, const AttnWork* work = nullptr);
int launch_attn_decode(const pie_pool* p, int32_t layer, const void* d_q, int32_t max_blocks, const int32_t* d_ctx,
                       int32_t batch, void* d_out, hipStream_t s, hipEvent_t k_start = nullptr,
                       hipEvent_t k_end = nullptr, int32_t ticket_index = -1,
                       unsigned long long* clock_row = nullptr, const LayerView* view = nullptr,
                       hipEvent_t done = nullptr, const AttnWork* work = nullptr, const void* d_k_new = nullptr,
                       const void* d_v_new = nullptr);
int launch_stream_probe(const pie_pool* p, int32_t layer, int32_t max_blocks, int32_t batch, hipStream_t s);
int attn_static_scratch(char** out);
int attn_static_work(const pie_pool* p, int32_t batch, int32_t max_blocks, AttnWork* out);
size_t attn_plan_ints(const pie_config& c);
size_t attn_workspace_floats(const pie_config& c);
bool attn_config_supported(const pie_config& c);

}  // namespace pie
