/* The C boundary used from plain C, without Python or PyTorch: the program allocates device and pinned memory
 * itself (hipMalloc / hipHostMalloc), builds a pool through include/pie.h, decodes a short sequence token by
 * token with pie_step - some of its blocks homed in the host pool, so that prefetch, staged append and dirty
 * write-back all run - and checks the last token's attention output against the plain definition
 * (softmax(q K^T / sqrt(d)) V over the rows it appended) written out here in double precision.
 * Built by __graft_entry__.build(); run by tests/test_zy_gpu_c_abi.py.  Prints "c abi ok" and exits 0 on success. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "pie.h"

#define L 2
#define HQ 4
#define HKV 2
#define D 64
#define T 16
#define STEPS 40          /* tokens appended: three blocks, the last one ragged */
#define MAXB 4

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define PIE_OK_(x) do { int r_ = (x); if (r_ != PIE_OK) { fprintf(stderr, "%s: %s\n", #x, pie_strerror(r_)); return 3; } } while (0)

static uint32_t lcg_state = 12345u;
static float draw(void) {                      /* uniform in [-0.5, 0.5) */
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return (float)(lcg_state >> 8) / 16777216.0f - 0.5f;
}

int main(void) {
  pie_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = L; cfg.n_q_heads = HQ; cfg.n_kv_heads = HKV; cfg.head_dim = D; cfg.block_tokens = T;
  cfg.dtype = PIE_DTYPE_F32; cfg.n_gpu_blocks = 8; cfg.n_stage_blocks = 4; cfg.n_host_blocks = 4;
  cfg.max_batch = 1; cfg.max_blocks_per_seq = MAXB;
  size_t d_bytes = 0, h_bytes = 0;
  PIE_OK_(pie_pool_bytes_required(&cfg, &d_bytes, &h_bytes));
  void *d_base = NULL, *h_base = NULL;
  HIP_OK(hipMalloc(&d_base, d_bytes));
  HIP_OK(hipHostMalloc(&h_base, h_bytes, hipHostMallocDefault));
  HIP_OK(hipMemset(d_base, 0xff, d_bytes));    /* NaN patterns everywhere: unused rows must not matter */
  memset(h_base, 0xff, h_bytes);
  pie_pool* pool = NULL;
  PIE_OK_(pie_pool_init(&cfg, d_base, d_bytes, h_base, h_bytes, &pool));

  /* the sequence's first block in the GPU pool, its second and third (the tail from token 17 on) in the host pool */
  int32_t table[MAXB] = {-1, -1, -1, -1}, h;
  PIE_OK_(pie_block_alloc(pool, PIE_WHERE_GPU, 1, &h));  table[0] = h;
  PIE_OK_(pie_block_alloc(pool, PIE_WHERE_HOST, 1, &h)); table[1] = h;
  PIE_OK_(pie_block_alloc(pool, PIE_WHERE_HOST, 1, &h)); table[2] = h;

  hipStream_t cs, is, os;
  HIP_OK(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
  HIP_OK(hipStreamCreateWithFlags(&is, hipStreamNonBlocking));
  HIP_OK(hipStreamCreateWithFlags(&os, hipStreamNonBlocking));
  int32_t *d_table = NULL, *d_ctx = NULL;
  float *d_q = NULL, *d_k = NULL, *d_v = NULL, *d_out = NULL;
  HIP_OK(hipMalloc((void**)&d_table, sizeof table));
  HIP_OK(hipMalloc((void**)&d_ctx, sizeof(int32_t)));
  HIP_OK(hipMalloc((void**)&d_q, sizeof(float) * L * HQ * D));
  HIP_OK(hipMalloc((void**)&d_out, sizeof(float) * L * HQ * D));
  HIP_OK(hipMalloc((void**)&d_k, sizeof(float) * L * HKV * D));
  HIP_OK(hipMalloc((void**)&d_v, sizeof(float) * L * HKV * D));
  HIP_OK(hipMemcpy(d_table, table, sizeof table, hipMemcpyHostToDevice));

  static float K[L][STEPS][HKV][D], V[L][STEPS][HKV][D], q[L][HQ][D], out[L][HQ][D];
  for (int t = 0; t < STEPS; ++t) {
    float k_new[L][HKV][D], v_new[L][HKV][D];
    for (int l = 0; l < L; ++l)
      for (int g = 0; g < HKV; ++g)
        for (int c = 0; c < D; ++c) {
          K[l][t][g][c] = k_new[l][g][c] = draw();
          V[l][t][g][c] = v_new[l][g][c] = draw();
        }
    for (int l = 0; l < L; ++l)
      for (int hq = 0; hq < HQ; ++hq)
        for (int c = 0; c < D; ++c) q[l][hq][c] = 4.0f * draw();
    const int32_t ctx = t + 1;
    HIP_OK(hipMemcpy(d_ctx, &ctx, sizeof ctx, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_q, q, sizeof q, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_k, k_new, sizeof k_new, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_v, v_new, sizeof v_new, hipMemcpyHostToDevice));
    int32_t pf[MAXB], dirty[1], n_pf = 0, n_dirty = 0;
    PIE_OK_(pie_prefetch_list(pool, table, MAXB, &ctx, 1, pf, &n_pf, dirty, &n_dirty));
    PIE_OK_(pie_step(pool, d_q, d_k, d_v, d_table, MAXB, d_ctx, 1, n_pf, pf, n_dirty, dirty, d_out, cs, is, os));
    PIE_OK_(pie_pool_sync(pool));
  }
  uint32_t flags = 0;
  PIE_OK_(pie_check_errors_sync(pool, &flags));
  if (flags) { fprintf(stderr, "device error flags %u\n", flags); return 4; }
  HIP_OK(hipMemcpy(out, d_out, sizeof out, hipMemcpyDeviceToHost));

  /* the definition, for the last step's queries over all STEPS rows */
  double worst = 0.0;
  for (int l = 0; l < L; ++l)
    for (int hq = 0; hq < HQ; ++hq) {
      const int g = hq / (HQ / HKV);
      double s[STEPS], m = -1e300, z = 0.0, ref[D];
      for (int t = 0; t < STEPS; ++t) {
        double acc = 0.0;
        for (int c = 0; c < D; ++c) acc += (double)q[l][hq][c] * (double)K[l][t][g][c];
        s[t] = acc / sqrt((double)D);
        if (s[t] > m) m = s[t];
      }
      for (int t = 0; t < STEPS; ++t) { s[t] = exp(s[t] - m); z += s[t]; }
      double scale = 0.0;
      for (int c = 0; c < D; ++c) {
        ref[c] = 0.0;
        for (int t = 0; t < STEPS; ++t) ref[c] += s[t] / z * (double)V[l][t][g][c];
        if (fabs(ref[c]) > scale) scale = fabs(ref[c]);
      }
      for (int c = 0; c < D; ++c) {
        const double err = fabs((double)out[l][hq][c] - ref[c]) / scale;
        if (!(err <= worst)) worst = err;        /* also catches NaN */
      }
    }
  pie_stats st;
  PIE_OK_(pie_get_stats(pool, &st));
  printf("rows max relative error %.3g, host blocks %d, bytes in last step %llu\n", worst, st.host_blocks_in_use,
         (unsigned long long)st.bytes_in);
  if (!(worst <= 1e-5) || st.host_blocks_in_use != 2 || st.bytes_in == 0) { fprintf(stderr, "check failed\n"); return 5; }
  PIE_OK_(pie_pool_destroy(pool));
  hipFree(d_base); hipHostFree(h_base); hipFree(d_table); hipFree(d_ctx); hipFree(d_q); hipFree(d_out); hipFree(d_k); hipFree(d_v);
  printf("c abi ok\n");
  return 0;
}
