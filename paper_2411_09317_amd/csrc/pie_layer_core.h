// The layer-granular swapping protocol's state (see pie_layer_sched.cpp), shared by the drivers that run it.
#ifndef PIE_LAYER_CORE_H
#define PIE_LAYER_CORE_H

#include <algorithm>
#include <vector>

#include "pie.h"

struct pie_layer_sched {
  int32_t n = 0;
  std::vector<pie_layer_entry> table;
  std::vector<int32_t> free_gpu, free_host;      // kept ascending; lowest slot first
  int32_t moving_in = -1, moving_out = -1;
  // Adaptive expansion in layers (Section 3.4.2): how many GPU layer slots may be in use.  Slots beyond the
  // target are retired as they become free; while more are occupied than allowed, a layer has to leave.
  int32_t n_gpu_total = 0, n_host_total = 0, n_enabled = 0, target = 0;
  std::vector<int32_t> retired;                  // ascending

  void rebalance() {
    while (n_enabled > target && !free_gpu.empty()) {
      give_back(retired, free_gpu.back());       // the highest free slot
      free_gpu.pop_back();
      --n_enabled;
    }
    while (n_enabled < target && !retired.empty()) {
      give_back(free_gpu, take_lowest(retired));
      ++n_enabled;
    }
  }
  bool oversubscribed() const { return n_enabled > target; }

  int32_t distance(int32_t j, int32_t k) const { return ((j - k) % n + n) % n; }

  static int32_t take_lowest(std::vector<int32_t>& v) {
    const int32_t s = v.front();
    v.erase(v.begin());
    return s;
  }
  static void give_back(std::vector<int32_t>& v, int32_t s) {
    auto it = v.begin();
    while (it != v.end() && *it < s) ++it;
    v.insert(it, s);
  }

  int32_t hottest_on_host(int32_t k) const {
    int32_t best = -1;
    for (int32_t j = 0; j < n; ++j)
      if (table[j].state == PIE_LAYER_HOST && (best < 0 || distance(j, k) < distance(best, k))) best = j;
    return best;
  }
  int32_t coldest_on_gpu(int32_t k) const {
    int32_t best = -1;
    for (int32_t j = 0; j < n; ++j)
      if (j != k && table[j].state == PIE_LAYER_GPU && (best < 0 || distance(j, k) > distance(best, k))) best = j;
    return best;
  }
  void start_in(int32_t j, pie_layer_action* a) {          // phase one: the destination is named
    table[j].gpu_slot = take_lowest(free_gpu);
    table[j].state = PIE_LAYER_MOVING_IN;
    moving_in = j;
    a->in_layer = j;
    a->in_gpu_slot = table[j].gpu_slot;
    a->in_host_slot = table[j].host_slot;
  }
  void start_out(int32_t j, pie_layer_action* a) {
    table[j].host_slot = take_lowest(free_host);
    table[j].state = PIE_LAYER_MOVING_OUT;
    moving_out = j;
    a->out_layer = j;
    a->out_gpu_slot = table[j].gpu_slot;
    a->out_host_slot = table[j].host_slot;
  }
};

#endif  // PIE_LAYER_CORE_H
