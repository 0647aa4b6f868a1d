// The host code of the GPU paths, meant to be built with the address and undefined-behaviour sanitizers on the host
// side only (the device code is compiled as usual): pie_step in every monitoring mode and swap path with residency
// changes in between, the per-layer calls by hand, the layer pool and the elastic pool, all through the C boundary
// with the program's own device and pinned memory.  Return codes and device error flags are checked, results are
// not (the parity tests do that).  Built by __graft_entry__.build(); run by tests/test_zx_gpu_host_sanitized.py.
// Prints "gpu host check ok" and exits 0.
#include <hip/hip_runtime_api.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include "pie.h"
#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e_)); exit(2); } } while (0)
#define OK(x) do { int r_ = (x); if (r_ != PIE_OK) { printf("line %d: %s -> %s (hip %d)\n", __LINE__, #x, pie_strerror(r_), pie_last_hip_error()); exit(3); } } while (0)
static hipStream_t cs, is, os;
struct Mem { void* d = nullptr; void* h = nullptr; };
static Mem make(const pie_config& cfg, pie_pool** p) {
  size_t db = 0, hb = 0; OK(pie_pool_bytes_required(&cfg, &db, &hb));
  Mem m; HIP_OK(hipMalloc(&m.d, db)); HIP_OK(hipMemset(m.d, 0, db));
  if (hb) { HIP_OK(hipHostMalloc(&m.h, hb, hipHostMallocDefault)); memset(m.h, 0, hb); }
  OK(pie_pool_init(&cfg, m.d, db, m.h, hb, p));
  return m;
}
static void* dzero(size_t bytes) { void* p; HIP_OK(hipMalloc(&p, bytes)); HIP_OK(hipMemset(p, 0, bytes)); return p; }

static void part_step() {
  pie_config cfg; memset(&cfg, 0, sizeof cfg);
  const int L = 4, B = 4, MB = 16;
  cfg.n_layers = L; cfg.n_q_heads = 8; cfg.n_kv_heads = 4; cfg.head_dim = 128; cfg.block_tokens = 16; cfg.dtype = PIE_DTYPE_F16;
  cfg.n_gpu_blocks = 64; cfg.n_stage_blocks = 48; cfg.n_host_blocks = 64; cfg.max_batch = B; cfg.max_blocks_per_seq = MB;
  pie_pool* p; Mem m = make(cfg, &p);
  std::vector<int32_t> table(B * MB, -1), all;
  for (int b = 0; b < B; ++b) {
    const int nb = 6 + 2 * b;
    std::vector<int32_t> h(nb);
    OK(pie_block_alloc(p, b % 2 ? PIE_WHERE_HOST : PIE_WHERE_GPU, nb, h.data()));
    for (int j = 0; j < nb; ++j) { table[b * MB + j] = h[j]; all.push_back(h[j]); }
  }
  int32_t* d_table = (int32_t*)dzero(table.size() * 4); int32_t* d_ctx = (int32_t*)dzero(B * 4);
  void* q = dzero((size_t)L * B * 8 * 128 * 2); void* out = dzero((size_t)L * B * 8 * 128 * 2);
  void* k = dzero((size_t)L * B * 4 * 128 * 2); void* v = dzero((size_t)L * B * 4 * 128 * 2);
  pie_controller* ctl; OK(pie_controller_create(16, 8, &ctl));
  std::vector<int32_t> ctx(B), pf(B * MB), dirty(B);
  std::vector<float> t0(L), t1(L), t2(L), t3(L), t4(L);
  for (int step = 0; step < 60; ++step) {
    for (int b = 0; b < B; ++b) ctx[b] = 20 + step + 16 * b;          // grows through block boundaries
    OK(pie_set_timing(p, step % 3));
    OK(pie_set_swap_path(p, (step / 3) % 3));
    OK(pie_set_cross_step_prefetch(p, (step / 9) % 2));
    OK(pie_set_host_presence_check(p, (step / 18) % 2));
    OK(pie_set_async_submit(p, (step / 6) % 2));                      // every other six steps by the pool's own thread
    if (step % 10 == 5) { int32_t nh; OK(pie_set_host_fraction(p, 0.1f * (step / 10), (int32_t)all.size(), all.data(), is, &nh)); }
    if (step % 10 == 8) OK(pie_migrate(p, 3, all.data() + step % 5, (step / 10) % 2, is));
    HIP_OK(hipMemcpy(d_table, table.data(), table.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_ctx, ctx.data(), B * 4, hipMemcpyHostToDevice));
    int32_t npf, nd;
    OK(pie_prefetch_list(p, table.data(), MB, ctx.data(), B, pf.data(), &npf, dirty.data(), &nd));
    OK(pie_step(p, q, k, v, d_table, MB, d_ctx, B, npf, pf.data(), nd, dirty.data(), out, cs, is, os));
    if (step % 4 == 1) {                                              // two in a row; the lists may go away at once
      std::vector<int32_t> pf2(pf.begin(), pf.begin() + npf), dirty2(dirty.begin(), dirty.begin() + nd);
      OK(pie_step(p, q, k, v, d_table, MB, d_ctx, B, npf, pf2.data(), nd, dirty2.data(), out, cs, is, os));
      pf2.assign(pf2.size(), -7);
      dirty2.assign(dirty2.size(), -7);
      OK(pie_step_join_sync(p));
    }
    OK(pie_pool_sync(p));
    if (step % 3) {
      pie_stats st; OK(pie_get_stats(p, &st));
      OK(pie_get_layer_times(p, t0.data(), t1.data(), t2.data(), t3.data(), t4.data()));
      float f; OK(pie_controller_update(p, ctl, 1000.0, &f));
    }
  }
  // the per-layer calls by hand
  int32_t npf, nd; OK(pie_prefetch_list(p, table.data(), MB, ctx.data(), B, pf.data(), &npf, dirty.data(), &nd));
  for (int l = 0; l < L; ++l) {
    OK(pie_swap_in(p, l, npf, pf.data(), is));
    OK(pie_kv_append(p, l, k, v, d_table, MB, d_ctx, B, cs));
    OK(pie_attn_decode(p, l, q, d_table, MB, d_ctx, B, out, cs));
    OK(pie_swap_out(p, l, nd, dirty.data(), os));
    float ms; OK(pie_attn_stream_probe_sync(p, l, d_table, MB, d_ctx, B, cs, &ms));
  }
  uint32_t flags; OK(pie_check_errors_sync(p, &flags));
  if (flags) { printf("step part: device flags %u\n", flags); exit(4); }
  OK(pie_set_async_submit(p, 1));                                     // destroyed with the thread alive and a step handed over
  OK(pie_step(p, q, k, v, d_table, MB, d_ctx, B, npf, pf.data(), nd, dirty.data(), out, cs, is, os));
  OK(pie_block_free(p, (int32_t)all.size(), all.data()));
  OK(pie_controller_destroy(ctl));
  OK(pie_pool_destroy(p));
  hipFree(m.d); hipHostFree(m.h); hipFree(d_table); hipFree(d_ctx); hipFree(q); hipFree(out); hipFree(k); hipFree(v);
  printf("step part ok\n"); fflush(stdout);
}

static void part_layers() {
  pie_config cfg; memset(&cfg, 0, sizeof cfg);
  const int LOG = 6, SLOTS = 4, B = 3, MB = 8;
  cfg.n_layers = SLOTS; cfg.n_q_heads = 8; cfg.n_kv_heads = 2; cfg.head_dim = 64; cfg.block_tokens = 16; cfg.dtype = PIE_DTYPE_BF16;
  cfg.n_gpu_blocks = 24; cfg.max_batch = B; cfg.max_blocks_per_seq = MB;
  pie_pool* p; Mem m = make(cfg, &p);
  size_t hb; OK(pie_layer_pool_bytes_required(p, 5, &hb));
  void* hp; HIP_OK(hipHostMalloc(&hp, hb, hipHostMallocDefault)); memset(hp, 0, hb);
  const int32_t on_host[2] = {4, 5};
  pie_layer_pool* lp; OK(pie_layer_pool_create(p, LOG, 5, hp, hb, 2, on_host, &lp));
  std::vector<int32_t> table(B * MB, -1), h(B * MB);
  OK(pie_block_alloc(p, PIE_WHERE_GPU, B * MB, h.data()));
  for (int i = 0; i < B * MB; ++i) table[i] = h[i];
  int32_t* d_table = (int32_t*)dzero(table.size() * 4); int32_t* d_ctx = (int32_t*)dzero(B * 4);
  HIP_OK(hipMemcpy(d_table, table.data(), table.size() * 4, hipMemcpyHostToDevice));
  void* q = dzero((size_t)LOG * B * 8 * 64 * 2); void* out = dzero((size_t)LOG * B * 8 * 64 * 2);
  void* k = dzero((size_t)LOG * B * 2 * 64 * 2); void* v = dzero((size_t)LOG * B * 2 * 64 * 2);
  std::vector<pie_layer_entry> tab(LOG);
  for (int step = 0; step < 40; ++step) {
    int32_t ctx[B]; for (int b = 0; b < B; ++b) ctx[b] = 5 + step * 2 + b;
    HIP_OK(hipMemcpy(d_ctx, ctx, sizeof ctx, hipMemcpyHostToDevice));
    if (step == 10) OK(pie_layer_pool_set_gpu_slots(lp, 3));
    if (step == 20) OK(pie_layer_pool_set_gpu_slots(lp, 4));
    OK(pie_layer_step(lp, q, k, v, d_table, MB, d_ctx, B, out, cs, is, os));
    OK(pie_layer_pool_table(lp, tab.data()));
    if (step % 7 == 0) {
      OK(pie_layer_pool_settle_sync(lp));
      for (int j = 0; j < LOG; ++j) { int32_t w; void* ptr; OK(pie_layer_pool_address(lp, j, &w, &ptr)); }
    }
  }
  OK(pie_layer_pool_settle_sync(lp));
  pie_layer_stats st; OK(pie_layer_pool_stats(lp, &st));
  uint32_t flags; OK(pie_check_errors_sync(p, &flags));
  if (flags) { printf("layer part: device flags %u\n", flags); exit(4); }
  printf("layer part ok: %lld swap-ins, %lld forced\n", (long long)st.n_swap_in, (long long)st.n_forced_in); fflush(stdout);
  OK(pie_layer_pool_destroy(lp)); OK(pie_pool_destroy(p));
  hipFree(m.d); hipHostFree(hp); hipFree(d_table); hipFree(d_ctx); hipFree(q); hipFree(out); hipFree(k); hipFree(v);
}

static void part_elastic() {
  pie_config cfg; memset(&cfg, 0, sizeof cfg);
  const int N = 6, B = 3, C = 4, K0 = 3, KCAP = 6;
  cfg.n_layers = N; cfg.n_q_heads = 8; cfg.n_kv_heads = 2; cfg.head_dim = 128; cfg.block_tokens = 16; cfg.dtype = PIE_DTYPE_F16;
  cfg.n_gpu_blocks = C * K0; cfg.max_batch = B; cfg.max_blocks_per_seq = C * KCAP;
  pie_pool* p; Mem m = make(cfg, &p);
  size_t db, hb; OK(pie_elastic_bytes_required(p, C, KCAP, 5, &db, &hb));
  void* dw = dzero(db); void* hp; HIP_OK(hipHostMalloc(&hp, hb, hipHostMallocDefault)); memset(hp, 0, hb);
  pie_elastic_pool* ep; OK(pie_elastic_create(p, C, KCAP, 5, dw, db, hp, hb, &ep));
  const int MB = C * KCAP;
  std::vector<int32_t> table(B * MB, -1);
  for (int b = 0; b < B; ++b) for (int j = 0; j < 4; ++j) table[b * MB + j] = b * 4 + j;       // blocks 0..11 of a layer's cache
  int32_t* d_table = (int32_t*)dzero(table.size() * 4); int32_t* d_ctx = (int32_t*)dzero(B * 4);
  void* q = dzero((size_t)N * B * 8 * 128 * 2); void* out = dzero((size_t)N * B * 8 * 128 * 2);
  void* k = dzero((size_t)N * B * 2 * 128 * 2); void* v = dzero((size_t)N * B * 2 * 128 * 2);
  std::vector<pie_layer_entry> tab(N); std::vector<int32_t> chunks(KCAP);
  const int plan[] = {0, 2, 2, 3, 1, 0};
  for (int step = 0; step < 60; ++step) {
    int32_t ctx[B]; for (int b = 0; b < B; ++b) ctx[b] = 10 + (step % 50) + b;                   // <= 64 tokens = 4 blocks
    HIP_OK(hipMemcpy(d_table, table.data(), table.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_ctx, ctx, sizeof ctx, hipMemcpyHostToDevice));
    if (step % 10 == 0) {
      int rc = pie_elastic_set_layers_on_cpu(ep, plan[step / 10], 12, cs);
      if (rc != PIE_OK && rc != PIE_ESTATE) OK(rc);
      OK(pie_elastic_set_live_blocks(ep, 12));
    }
    if (step == 25) { const int32_t src[2] = {3, 7}, dst[2] = {12, 13}; int rc = pie_elastic_move_blocks(ep, 2, src, dst, cs); if (rc != PIE_OK && rc != PIE_ESTATE) OK(rc); if (!rc) { const int32_t back_s[2] = {12, 13}, back_d[2] = {3, 7}; OK(pie_elastic_move_blocks(ep, 2, back_s, back_d, cs)); } }
    OK(pie_elastic_step(ep, q, k, v, d_table, MB, d_ctx, B, out, cs, is, os));
    int32_t vis, tgt, mm; OK(pie_elastic_capacity(ep, &vis, &tgt, &mm));
    OK(pie_elastic_table(ep, tab.data()));
    if (step % 9 == 0) {
      OK(pie_elastic_settle_sync(ep, cs));
      for (int j = 0; j < N; ++j) { int32_t w, nc; void* ptr; OK(pie_elastic_layer(ep, j, &w, &nc, chunks.data(), &ptr)); }
    }
  }
  OK(pie_elastic_settle_sync(ep, cs));
  pie_layer_stats st; OK(pie_elastic_stats(ep, &st));
  uint32_t flags; OK(pie_check_errors_sync(p, &flags));
  if (flags) { printf("elastic part: device flags %u\n", flags); exit(4); }
  printf("elastic part ok: %lld swap-ins, %lld swap-outs\n", (long long)st.n_swap_in, (long long)st.n_swap_out); fflush(stdout);
  OK(pie_elastic_destroy(ep)); OK(pie_pool_destroy(p));
  hipFree(m.d); hipHostFree(hp); hipFree(dw); hipFree(d_table); hipFree(d_ctx); hipFree(q); hipFree(out); hipFree(k); hipFree(v);
}

int main() {
  HIP_OK(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
  HIP_OK(hipStreamCreateWithFlags(&is, hipStreamNonBlocking));
  HIP_OK(hipStreamCreateWithFlags(&os, hipStreamNonBlocking));
  part_step();
  part_layers();
  part_elastic();
  printf("gpu host check ok\n");
  return 0;
}
