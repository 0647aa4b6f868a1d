// Adaptive expansion: the online controller that chooses how much of the KV cache is host-resident.
//
// Paper: Section 3.4.2 (start with everything on the GPU; add swapping while it stays hidden; move one
// unit back when compute had to wait; stop when the workload stops scaling; probe periodically; tolerate
// brief interference) and the three growth conditions of Section 1 (link not saturated, swap latency below
// compute latency, throughput still rising).  The paper gives no constants; the defaults below are this
// library's choice and can be changed with pie_controller_config.
//
// The amount of swapping is an integer level k; host fraction = k / units.  A step is bad when some
// layer's swap-in took longer than its compute or the summed waits exceed stall_eps of the summed compute.

#include <map>
#include <new>
#include <vector>

#include "pie_internal.h"

struct pie_controller {
  int32_t units = 1, k_max = 0;
  double rho = 0.9;
  int32_t k_up = 4, k_down = 2, probe_period = 64;
  double plateau_eps = 0.01, util_max = 0.9, stall_eps = 0.01;

  int32_t k = 0, clean = 0, bad = 0;
  bool has_ceiling = false;
  int32_t ceiling = 0, since_ceiling = 0;
  bool grew = false;
  double win_sum = 0.0;
  int64_t win_n = 0;
  std::map<int32_t, double> rec;   // level -> mean throughput while sustained

  void set_level(int32_t level, bool by_growing) {
    k = level;
    grew = by_growing;
    clean = bad = 0;
    win_sum = 0.0;
    win_n = 0;
  }
};

extern "C" {

int pie_controller_create(int32_t units, int32_t k_max, pie_controller** out) {
  if (!out || units <= 0 || k_max < 0 || k_max > units) return PIE_EINVAL;
  pie_controller* c = new (std::nothrow) pie_controller();
  if (!c) return PIE_ENOMEM;
  c->units = units;
  c->k_max = k_max;
  *out = c;
  return PIE_OK;
}

int pie_controller_destroy(pie_controller* c) {
  if (!c) return PIE_EINVAL;
  delete c;
  return PIE_OK;
}

int pie_controller_config(pie_controller* c, double rho, int32_t k_up, int32_t k_down, int32_t probe_period,
                          double plateau_eps, double util_max, double stall_eps) {
  if (!c || !(rho > 0.0) || k_up < 1 || k_down < 1 || probe_period < 0 || !(util_max > 0.0) || stall_eps < 0.0)
    return PIE_EINVAL;
  c->rho = rho;
  c->k_up = k_up;
  c->k_down = k_down;
  c->probe_period = probe_period;
  c->plateau_eps = plateau_eps;
  c->util_max = util_max;
  c->stall_eps = stall_eps;
  return PIE_OK;
}

int pie_controller_observe(pie_controller* c, int32_t n_layers, const double* t_attn, const double* t_in,
                           const double* t_stall, double link_util, double throughput, int32_t* out_level) {
  if (!c || n_layers <= 0 || !t_attn || !t_in || !t_stall || !out_level) return PIE_EINVAL;
  if (c->has_ceiling) ++c->since_ceiling;
  double tot_attn = 0.0, tot_stall = 0.0;
  bool over = false;
  for (int32_t l = 0; l < n_layers; ++l) {
    tot_attn += t_attn[l];
    tot_stall += t_stall[l];
    if (t_in[l] > t_attn[l]) over = true;   // swap latency above compute latency
  }
  const bool is_bad = c->k > 0 && (over || tot_stall > c->stall_eps * tot_attn);
  if (is_bad) {
    ++c->bad;
    c->clean = 0;
  } else {
    ++c->clean;
    c->bad = 0;
    c->win_sum += throughput;
    ++c->win_n;
  }

  if (c->bad >= c->k_down) {               // compute had to wait: one unit back, remember the ceiling
    c->has_ceiling = true;
    c->ceiling = c->k;
    c->since_ceiling = 0;
    c->set_level(c->k - 1, false);
    *out_level = c->k;
    return PIE_OK;
  }
  if (c->clean < c->k_up) {
    *out_level = c->k;
    return PIE_OK;
  }

  c->rec[c->k] = c->win_sum / (double)c->win_n;   // the level is sustained
  if (c->grew) {
    auto below = c->rec.find(c->k - 1);
    if (below != c->rec.end() && c->rec[c->k] < below->second * (1.0 + c->plateau_eps)) {
      c->has_ceiling = true;                     // the workload stopped scaling: step back and hold
      c->ceiling = c->k;
      c->since_ceiling = 0;
      c->set_level(c->k - 1, false);
      *out_level = c->k;
      return PIE_OK;
    }
  }
  c->grew = false;

  *out_level = c->k;
  if (c->k >= c->k_max) return PIE_OK;
  if (link_util >= c->util_max) return PIE_OK;                              // condition 1: link saturated
  const bool at_ceiling = c->has_ceiling && c->k + 1 >= c->ceiling;
  if (at_ceiling && c->since_ceiling < c->probe_period) return PIE_OK;
  if (c->k > 0) {
    for (int32_t l = 0; l < n_layers; ++l)                                  // condition 2, one level ahead
      if (t_in[l] * (double)(c->k + 1) / (double)c->k > c->rho * t_attn[l]) return PIE_OK;
  }
  if (at_ceiling) c->has_ceiling = false;                                   // periodic upward probe
  c->set_level(c->k + 1, true);
  *out_level = c->k;
  return PIE_OK;
}

int pie_controller_level(pie_controller* c, int32_t* out_level, int32_t* out_ceiling) {
  if (!c || !out_level) return PIE_EINVAL;
  *out_level = c->k;
  if (out_ceiling) *out_ceiling = c->has_ceiling ? c->ceiling : -1;
  return PIE_OK;
}

int pie_controller_update(pie_pool* p, pie_controller* c, double throughput, float* out_host_fraction) {
  if (!p || !c || !out_host_fraction) return PIE_EINVAL;
  const int32_t L = p->cfg.n_layers;
  std::vector<float> a(L), i(L), s(L);
  int rc = pie_get_layer_times(p, a.data(), nullptr, i.data(), nullptr, s.data());
  if (rc) return rc;
  std::vector<double> ad(a.begin(), a.end()), id(i.begin(), i.end()), sd(s.begin(), s.end());
  double in_sum = 0.0, span = 0.0;
  for (int32_t l = 0; l < L; ++l) {
    in_sum += id[l];
    span += ad[l] + sd[l];
  }
  // the first layer's prefetch cannot overlap anything; its wait is the pipeline's fill, not a steady-state stall
  sd[0] = 0.0;
  const double util = span > 0.0 ? (in_sum < span ? in_sum / span : 1.0) : 0.0;
  int32_t level = 0;
  if ((rc = pie_controller_observe(c, L, ad.data(), id.data(), sd.data(), util, throughput, &level))) return rc;
  *out_host_fraction = (float)level / (float)c->units;
  return PIE_OK;
}

}  // extern "C"
