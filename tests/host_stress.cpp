// Host-logic stress, meant to be built with the address and undefined-behaviour sanitizers on the host side
// (tests/test_host_sanitized.py does so): random call sequences, valid and invalid arguments alike, against the
// bookkeeping-only pool, the layer scheduler, the chunk book and the controller, with the invariants that must hold
// after every call.  No GPU call is made.  Prints "host stress ok" and exits 0.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <random>
#include <vector>
#include "pie.h"
static std::mt19937_64 rng(12345);
static long ok_count[4][12];
static int ri(int lo, int hi) { return lo + (int)(rng() % (uint64_t)(hi - lo + 1)); }
#define REQUIRE(c) do { if (!(c)) { printf("FAILED %s:%d %s\n", __FILE__, __LINE__, #c); exit(1); } } while (0)

static void stress_pool(int iters) {
  pie_config cfg; memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = ri(1, 5); cfg.n_q_heads = 8; cfg.n_kv_heads = 4; cfg.head_dim = 128; cfg.block_tokens = 16; cfg.dtype = PIE_DTYPE_F16;
  cfg.n_gpu_blocks = ri(1, 40); cfg.n_stage_blocks = ri(0, 10); cfg.n_host_blocks = ri(0, 40); cfg.max_batch = 8; cfg.max_blocks_per_seq = 16;
  pie_pool* p = nullptr;
  REQUIRE(pie_pool_init(&cfg, nullptr, 0, nullptr, 0, &p) == PIE_OK);
  const int H = cfg.n_gpu_blocks + cfg.n_host_blocks;
  std::vector<int32_t> buf(4 * H + 64), a(H + 8), b(H + 8);
  for (int it = 0; it < iters; ++it) {
    const int op = ri(0, 11);
    const int n = ri(-1, H + 2);
    if (ri(0, 3)) { std::vector<int32_t> perm(H); for (int i = 0; i < H; ++i) perm[i] = i; std::shuffle(perm.begin(), perm.end(), rng); std::copy(perm.begin(), perm.end(), buf.begin()); }
    else for (auto& x : buf) x = ri(-2, H + 1);
    int rc = 0;
    switch (op) {
      case 0: rc = pie_block_alloc(p, ri(-1, 2), n, buf.data()); break;
      case 1: rc = pie_block_free(p, n, buf.data()); break;
      case 2: rc = pie_block_where(p, std::min(n, H + 2), buf.data(), a.data(), b.data()); break;
      case 3: rc = pie_block_staged(p, ri(-1, 2), std::min(n, H + 2), buf.data(), a.data(), b.data()); break;
      case 4: { int32_t k; rc = pie_pool_free_count(p, ri(-1, 2), &k); if (!rc) REQUIRE(k >= 0 && k <= H); break; }
      case 5: rc = pie_migrate(p, n, buf.data(), ri(-1, 2), nullptr); break;
      case 6: { int32_t nh = -1; rc = pie_set_host_fraction(p, (float)ri(-1, 11) / 10.f, n, buf.data(), nullptr, &nh); break; }
      case 7: {
        const int batch = ri(0, 9), mb = ri(0, 17);
        std::vector<int32_t> table(batch * mb + 1), ctx(batch + 1), pf(batch * mb + 1), dirty(batch + 1);
        int32_t npf = -1, nd = -1;
        for (auto& x : table) x = ri(-1, H);
        for (auto& x : ctx) x = ri(-1, 16 * 16 + 1);
        rc = pie_prefetch_list(p, table.data(), mb, ctx.data(), batch, pf.data(), &npf, dirty.data(), &nd);
        if (!rc) REQUIRE(npf >= 0 && npf <= batch * mb && nd >= 0 && nd <= batch);
        break;
      }
      case 8: { pie_stats st; rc = pie_get_stats(p, &st); break; }
      case 9: { void* q = nullptr; rc = pie_block_address(p, ri(-1, 2), ri(-1, cfg.n_layers), ri(-1, H + 20), &q); break; }
      case 10: {                                  // the newer calls on a pool without device memory: refused, nothing touched
        int32_t tb[4] = {0, 1, 2, 3}, cx[1] = {20};
        char q[16];
        rc = pie_attn_decode_static(p, ri(-1, cfg.n_layers), q, tb, ri(-1, 4), cx, ri(-1, 1), q, nullptr);
        REQUIRE(rc == PIE_ESTATE || rc == PIE_EINVAL || rc == PIE_OK);
        REQUIRE(pie_set_async_submit(p, ri(0, 1)) == PIE_ESTATE);
        REQUIRE(pie_step_join_sync(p) == PIE_OK);
        break;
      }
      case 11: {
        rc = pie_set_attn_vector_alu(p, ri(0, 1));
        REQUIRE(rc == PIE_OK || rc == PIE_ESTATE);
        rc = pie_set_swap_workgroups(p, ri(-1, 1030));
        REQUIRE(rc == PIE_OK || rc == PIE_EINVAL);
        const int tokens = ri(-2, 5000);
        REQUIRE(pie_set_attn_partition(p, tokens) == (tokens < 0 ? PIE_EINVAL : PIE_OK));
        int32_t used = -7;
        REQUIRE(pie_get_attn_partition_sync(p, &used) == PIE_ESTATE && used == -7);   // no device: nothing planned
        REQUIRE(pie_get_attn_partition_sync(p, nullptr) == PIE_EINVAL);
        break;
      }
    }
    REQUIRE(rc <= 0 && rc >= -4);
    if (!rc) ++ok_count[0][op];
    int32_t fg, fh; REQUIRE(!pie_pool_free_count(p, 0, &fg) && !pie_pool_free_count(p, 1, &fh));
    REQUIRE(fg >= 0 && fg <= cfg.n_gpu_blocks && fh >= 0 && fh <= cfg.n_host_blocks);
  }
  REQUIRE(pie_pool_destroy(p) == PIE_OK);
}

static void stress_sched(int iters) {
  const int n = ri(2, 12), g = ri(1, n), m = n - g;
  std::vector<int32_t> on_host;
  for (int j = 0; j < m; ++j) on_host.push_back(n - 1 - j);
  pie_layer_sched* s = nullptr;
  int rc = pie_layer_sched_create(n, g, m + 2, m, on_host.data(), &s);
  if (rc) { REQUIRE(rc == PIE_ENOMEM || rc == PIE_EINVAL); return; }
  std::vector<pie_layer_entry> tab(n);
  int layer = 0;
  for (int it = 0; it < iters; ++it) {
    pie_layer_action a;
    const int op = ri(0, 9);
    if (op < 5) {                      // the regular order: presence, policy, maybe completions
      for (int guard = 0; guard < 8; ++guard) {
        rc = pie_layer_sched_present(s, layer, &a); REQUIRE(rc == 0);
        if (a.wait == PIE_LAYER_WAIT_NONE) break;
        REQUIRE(pie_layer_sched_complete(s, a.wait == PIE_LAYER_WAIT_IN ? 0 : 1) == 0);
      }
      REQUIRE(a.wait == PIE_LAYER_WAIT_NONE);
      rc = pie_layer_sched_policy(s, layer, &a); REQUIRE(rc == 0);
      layer = (layer + 1) % n;
    } else if (op < 8) {
      rc = pie_layer_sched_complete(s, ri(-1, 2)); REQUIRE(rc == 0 || rc == PIE_ESTATE || rc == PIE_EINVAL);
    } else if (op == 8) {
      rc = pie_layer_sched_set_gpu_slots(s, ri(-1, g + 1)); REQUIRE(rc == 0 || rc == PIE_EINVAL || rc == PIE_ESTATE);
    } else {
      rc = pie_layer_sched_policy(s, ri(-1, n), &a); REQUIRE(rc <= 0);
      rc = pie_layer_sched_present(s, ri(-1, n), &a); REQUIRE(rc <= 0);
      if (!rc && a.wait != PIE_LAYER_WAIT_NONE) REQUIRE(pie_layer_sched_complete(s, a.wait == PIE_LAYER_WAIT_IN ? 0 : 1) == 0);
    }
    REQUIRE(pie_layer_sched_table(s, tab.data()) == 0);
    std::vector<int> gs(n + 2, 0), hs(m + 4, 0);
    for (auto& e : tab) {
      REQUIRE(e.state >= 0 && e.state <= 3);
      if (e.gpu_slot >= 0) { REQUIRE(e.gpu_slot < g); REQUIRE(++gs[e.gpu_slot] == 1); }
      if (e.host_slot >= 0) { REQUIRE(e.host_slot < m + 2); REQUIRE(++hs[e.host_slot] == 1); }
      REQUIRE(e.gpu_slot >= 0 || e.host_slot >= 0);
    }
  }
  REQUIRE(pie_layer_sched_destroy(s) == 0);
}

static void stress_book(int iters) {
  const int n = ri(1, 10), k0 = ri(1, 6), cap = k0 + ri(0, 8);
  pie_chunk_book* b = nullptr;
  REQUIRE(pie_chunk_book_create(n, n * k0, cap, &b) == 0);
  std::vector<int32_t> chunks(cap + 1);
  for (int it = 0; it < iters; ++it) {
    const int op = ri(0, 3);
    int rc = 0;
    if (op == 0) rc = pie_chunk_book_set_layers_on_cpu(b, ri(-1, n), ri(-1, cap + 1));
    else if (op == 1) rc = pie_chunk_book_left_gpu(b, ri(-1, n), ri(-2, cap + 1));
    else if (op == 2) { int32_t nd; rc = pie_chunk_book_enters_gpu(b, ri(-1, n), &nd); if (!rc) REQUIRE(nd >= 0 && nd <= cap); }
    else { int32_t r, nd, nc; rc = pie_chunk_book_layer(b, ri(-1, n), &r, &nd, &nc, chunks.data()); if (!rc) REQUIRE(nc >= 0 && nc <= cap); }
    REQUIRE(rc <= 0 && rc >= -4);
    if (!rc) ++ok_count[2][op];
    int32_t vis, tgt, fr, m; REQUIRE(pie_chunk_book_capacity(b, &vis, &tgt, &fr, &m) == 0);
    REQUIRE(vis >= 0 && vis <= tgt && tgt <= cap && fr >= 0 && fr <= n * k0 && m >= 0 && m < n);
    int held = 0;
    std::vector<int> seen(n * k0, 0);
    for (int j = 0; j < n; ++j) {
      int32_t r, nd, nc; REQUIRE(pie_chunk_book_layer(b, j, &r, &nd, &nc, chunks.data()) == 0);
      for (int i = 0; i < nc; ++i) { REQUIRE(chunks[i] >= 0 && chunks[i] < n * k0); REQUIRE(++seen[chunks[i]] == 1); }
      held += nc;
      REQUIRE(r || nc == 0);
    }
    REQUIRE(held + fr == n * k0);
  }
  REQUIRE(pie_chunk_book_destroy(b) == 0);
}

static void stress_controller(int iters) {
  pie_controller* c = nullptr;
  const int units = ri(1, 64), kmax = ri(0, units);
  REQUIRE(pie_controller_create(units, kmax, &c) == 0);
  (void)pie_controller_config(c, 0.9, ri(1, 5), ri(1, 3), ri(1, 20), 0.01, 0.9, 0.01);
  const int L = ri(1, 8);
  std::vector<double> ta(L), ti(L), ts(L);
  for (int it = 0; it < iters; ++it) {
    for (int l = 0; l < L; ++l) { ta[l] = ri(0, 100) / 10.0; ti[l] = ri(0, 200) / 10.0; ts[l] = ri(0, 3) ? 0.0 : ri(0, 50) / 10.0; }
    int32_t lvl = -1, ceil_ = -2;
    int rc = pie_controller_observe(c, ri(0, 9) ? L : ri(-1, L), ta.data(), ti.data(), ts.data(), ri(0, 12) / 10.0, ri(0, 1000), &lvl);
    REQUIRE(rc == 0 || rc == PIE_EINVAL);
    REQUIRE(pie_controller_level(c, &lvl, &ceil_) == 0);
    REQUIRE(lvl >= 0 && lvl <= kmax && ceil_ >= -1 && ceil_ <= kmax);
  }
  REQUIRE(pie_controller_destroy(c) == 0);
}

int main() {
  for (int round = 0; round < 1500; ++round) {
    stress_pool(400);
    stress_sched(400);
    stress_book(400);
    stress_controller(200);
  }
  for (int k = 0; k < 4; ++k) { printf("ok[%d]:", k); for (int o = 0; o < 10; ++o) printf(" %ld", ok_count[k][o]); printf("\n"); }
  printf("host stress ok\n");
  return 0;
}
