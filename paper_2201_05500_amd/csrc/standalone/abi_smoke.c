/*
 * abi_smoke.c - the C ABI used from plain C with nothing but the HIP runtime: no Python, no PyTorch.
 *
 * One table, one batch in which every key occurs a known number of times with a gradient of ones, one
 * pull + push, and the result checked against Algorithm 2's first step written out for that case:
 *   g = count, m = (1 - beta1) g, v = beta2 eps + (1 - beta2) g^2, x = x0 - lr m / sqrt(v)
 * where x0 is read back from the table after the pull (the initial value of a new row).  Then a
 * lookup-only pooling of the same batch must return, per segment, the sum of the updated rows.
 * Prints "abi_smoke ok" and returns 0, or says what failed and returns 1.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ctr_sparse.h"

#define CHECK_HIP(x)                                                             \
  do {                                                                           \
    hipError_t e_ = (x);                                                         \
    if (e_ != hipSuccess) {                                                      \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);      \
      return 1;                                                                  \
    }                                                                            \
  } while (0)
#define CHECK_CTR(x)                                          \
  do {                                                        \
    int s_ = (x);                                             \
    if (s_ != CTR_OK) {                                       \
      printf("ctr status %d at line %d\n", s_, __LINE__);     \
      return 1;                                               \
    }                                                         \
  } while (0)

enum { K = 37, D = 8, SEG = 5, G = 400, N = G * SEG };

int main(void) {
  ctr_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.capacity_rows = 1024;
  cfg.dim = D;
  cfg.load_factor = 0.5f;
  cfg.n_replicas = 1;
  cfg.lr = 1e-3f;
  cfg.beta1 = 0.9f;
  cfg.beta2 = 0.999f;
  cfg.eps = 1e-8f;
  cfg.init_seed = 42;
  cfg.init_std = 0.01f;
  cfg.flags = 0;

  const size_t table_bytes = ctr_table_bytes(&cfg);
  const size_t ws_bytes = ctr_workspace_bytes(&cfg, N, G);
  if (table_bytes == 0 || ws_bytes == 0) {
    printf("configuration rejected\n");
    return 1;
  }
  void *d_table = NULL, *d_ws = NULL;
  uint64_t* d_keys = NULL;
  uint32_t* d_off = NULL;
  float *d_pooled = NULL, *d_grad = NULL, *d_x = NULL, *d_m = NULL, *d_v = NULL;
  uint32_t* d_found = NULL;
  hipStream_t st;
  CHECK_HIP(hipStreamCreate(&st));
  CHECK_HIP(hipMalloc(&d_table, table_bytes));
  CHECK_HIP(hipMalloc(&d_ws, ws_bytes));
  CHECK_HIP(hipMalloc((void**)&d_keys, N * sizeof(uint64_t)));
  CHECK_HIP(hipMalloc((void**)&d_off, (G + 1) * sizeof(uint32_t)));
  CHECK_HIP(hipMalloc((void**)&d_pooled, (size_t)G * D * sizeof(float)));
  CHECK_HIP(hipMalloc((void**)&d_grad, (size_t)G * D * sizeof(float)));
  CHECK_HIP(hipMalloc((void**)&d_x, (size_t)K * D * sizeof(float)));
  CHECK_HIP(hipMalloc((void**)&d_m, (size_t)K * D * sizeof(float)));
  CHECK_HIP(hipMalloc((void**)&d_v, (size_t)K * D * sizeof(float)));
  CHECK_HIP(hipMalloc((void**)&d_found, K * sizeof(uint32_t)));

  static uint64_t keys[N], uniq[K];
  static uint32_t off[G + 1];
  static float grad[G * D], pooled[G * D], x0[K * D], x1[K * D], m1[K * D], v1[K * D];
  static uint32_t found[K];
  uint32_t count[K];
  memset(count, 0, sizeof count);
  for (int k = 0; k < K; ++k) uniq[k] = 0x9E3779B97F4A7C15ull * (uint64_t)(k + 1);
  for (int i = 0; i < N; ++i) {
    const int k = (int)(((uint64_t)i * 7u + (uint64_t)(i / 11)) % K);
    keys[i] = uniq[k];
    ++count[k];
  }
  for (int g = 0; g <= G; ++g) off[g] = (uint32_t)(g * SEG);
  for (int i = 0; i < G * D; ++i) grad[i] = 1.0f;
  CHECK_HIP(hipMemcpyAsync(d_keys, keys, sizeof keys, hipMemcpyHostToDevice, st));
  CHECK_HIP(hipMemcpyAsync(d_off, off, sizeof off, hipMemcpyHostToDevice, st));
  CHECK_HIP(hipMemcpyAsync(d_grad, grad, sizeof grad, hipMemcpyHostToDevice, st));

  ctr_table* t = NULL;
  ctr_batch* b = NULL;
  CHECK_CTR(ctr_table_create(&cfg, d_table, table_bytes, st, &t));
  CHECK_CTR(ctr_pull_pool(t, 0, d_keys, N, d_off, G, d_pooled, d_ws, ws_bytes, &b, st));
  /* the rows as the pull created them */
  uint64_t* d_uniq = NULL;
  CHECK_HIP(hipMalloc((void**)&d_uniq, sizeof uniq));
  CHECK_HIP(hipMemcpyAsync(d_uniq, uniq, sizeof uniq, hipMemcpyHostToDevice, st));
  CHECK_CTR(ctr_table_collect(t, 0, d_uniq, K, d_x, d_m, d_v, d_found, st));
  CHECK_HIP(hipMemcpyAsync(x0, d_x, sizeof x0, hipMemcpyDeviceToHost, st));
  CHECK_HIP(hipMemcpyAsync(found, d_found, sizeof found, hipMemcpyDeviceToHost, st));
  CHECK_CTR(ctr_push_adam(t, 0, b, d_grad, CTR_STEP_LOCAL, st));
  CHECK_CTR(ctr_table_collect(t, 0, d_uniq, K, d_x, d_m, d_v, d_found, st));
  CHECK_HIP(hipMemcpyAsync(x1, d_x, sizeof x1, hipMemcpyDeviceToHost, st));
  CHECK_HIP(hipMemcpyAsync(m1, d_m, sizeof m1, hipMemcpyDeviceToHost, st));
  CHECK_HIP(hipMemcpyAsync(v1, d_v, sizeof v1, hipMemcpyDeviceToHost, st));
  CHECK_CTR(ctr_lookup_pool(t, 0, d_keys, N, d_off, G, d_pooled, NULL, d_ws, ws_bytes, st));
  CHECK_HIP(hipMemcpyAsync(pooled, d_pooled, sizeof pooled, hipMemcpyDeviceToHost, st));
  CHECK_HIP(hipStreamSynchronize(st));
  CHECK_CTR(ctr_last_status(t, st));
  uint64_t n_rows = 0;
  CHECK_CTR(ctr_table_size(t, &n_rows, st));
  if (n_rows != K) {
    printf("rows in table: %llu, expected %d\n", (unsigned long long)n_rows, K);
    return 1;
  }

  const double b1 = (double)cfg.beta1, b2 = (double)cfg.beta2, eps = (double)cfg.eps, lr = (double)cfg.lr;
  int bad = 0;
  for (int k = 0; k < K && !bad; ++k) {
    if (!found[k]) bad = 1;
    const double g = (double)count[k];
    const float m = (float)((1.0 - b1) * g);
    const float v = (float)(b2 * eps + (1.0 - b2) * g * g);
    for (int d = 0; d < D && !bad; ++d) {
      const double x = (double)x0[k * D + d] - lr * (double)m / sqrt((double)v);
      if (fabs((double)m1[k * D + d] - (double)m) > 1e-6 + 1e-5 * fabs((double)m)) bad = 2;
      if (fabs((double)v1[k * D + d] - (double)v) > 1e-6 + 1e-5 * fabs((double)v)) bad = 3;
      if (fabs((double)x1[k * D + d] - x) > 1e-6 + 1e-5 * fabs(x)) bad = 4;
      if (fabs((double)x0[k * D + d]) > 0.1 || x0[k * D + d] == 0.0f) bad = 5; /* initial values: small, not zero */
    }
  }
  for (int g = 0; g < G && !bad; ++g)
    for (int d = 0; d < D && !bad; ++d) {
      double s = 0.0;
      for (int j = 0; j < SEG; ++j) {
        const int i = g * SEG + j;
        const int k = (int)(((uint64_t)i * 7u + (uint64_t)(i / 11)) % K);
        s += (double)x1[k * D + d];
      }
      if (fabs((double)pooled[g * D + d] - s) > SEG * (1e-6 + 1e-5 * 0.1)) bad = 6;
    }
  if (bad) {
    printf("abi_smoke FAILED (check %d)\n", bad);
    return 1;
  }
  CHECK_CTR(ctr_table_destroy(t));
  CHECK_HIP(hipFree(d_table));
  CHECK_HIP(hipFree(d_ws));
  printf("abi_smoke ok: %d keys, %d occurrences\n", K, N);
  return 0;
}
