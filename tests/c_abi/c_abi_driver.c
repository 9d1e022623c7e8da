/*
 * A plain C caller of the C ABI in include/emb_bag.h: no Python, no torch.  It builds a small
 * multi-table problem with a fixed linear congruential generator, runs emb_bag_forward and
 * emb_bag_validate through the shared library with memory from the HIP runtime API, and checks
 * the result against the obvious double-precision loop written out below (the operation of the
 * paper's Sec. 3.1: per bag, gather the named rows and add them).  Prints "C ABI OK" and returns 0
 * on success.  Built by paper_2410_22249_amd/build.py; run by tests/test_parity_gpu.py.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "emb_bag.h"

#define CHECK(x)                                                              \
  do {                                                                        \
    hipError_t e_ = (x);                                                      \
    if (e_ != hipSuccess) {                                                   \
      fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));          \
      return 2;                                                               \
    }                                                                         \
  } while (0)

static uint64_t lcg_state = 0x5EED0A00ull;
static uint32_t lcg(void) {
  lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(lcg_state >> 33);
}

int main(void) {
  enum { T = 3, B = 37, D = 128 };
  const int64_t rows[T] = {1000, 17, 333};
  int64_t toff[T + 1] = {0};
  for (int t = 0; t < T; ++t) toff[t + 1] = toff[t] + rows[t];
  const int64_t total_rows = toff[T];

  float* tab = (float*)malloc((size_t)total_rows * D * sizeof(float));
  for (int64_t i = 0; i < total_rows * D; ++i) tab[i] = ((int)(lcg() % 2001) - 1000) * 1e-4f;

  int64_t* off = (int64_t*)malloc((T * B + 1) * sizeof(int64_t));
  off[0] = 0;
  for (int g = 0; g < T * B; ++g) off[g + 1] = off[g] + (int64_t)(lcg() % 90);
  const int64_t nl = off[T * B];
  int64_t* idx = (int64_t*)malloc((size_t)(nl > 0 ? nl : 1) * sizeof(int64_t));
  for (int t = 0; t < T; ++t)
    for (int64_t j = off[t * B]; j < off[(t + 1) * B]; ++j) idx[j] = (int64_t)(lcg() % rows[t]);

  void *d_tab, *d_toff, *d_idx, *d_off, *d_out, *d_bad;
  CHECK(hipMalloc(&d_tab, (size_t)total_rows * D * sizeof(float)));
  CHECK(hipMalloc(&d_toff, sizeof toff));
  CHECK(hipMalloc(&d_idx, (size_t)(nl > 0 ? nl : 1) * sizeof(int64_t)));
  CHECK(hipMalloc(&d_off, (T * B + 1) * sizeof(int64_t)));
  CHECK(hipMalloc(&d_out, (size_t)B * T * D * sizeof(float)));
  CHECK(hipMalloc(&d_bad, sizeof(int64_t)));
  CHECK(hipMemcpy(d_tab, tab, (size_t)total_rows * D * sizeof(float), hipMemcpyHostToDevice));
  CHECK(hipMemcpy(d_toff, toff, sizeof toff, hipMemcpyHostToDevice));
  CHECK(hipMemcpy(d_idx, idx, (size_t)nl * sizeof(int64_t), hipMemcpyHostToDevice));
  CHECK(hipMemcpy(d_off, off, (T * B + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
  CHECK(hipMemset(d_bad, 0, sizeof(int64_t)));
  hipStream_t stream;
  CHECK(hipStreamCreate(&stream));

  float* out = (float*)malloc((size_t)B * T * D * sizeof(float));
  int failures = 0;
  for (int mode = EMB_SUM; mode <= EMB_MEAN; ++mode) {
    emb_bag_desc desc = {0};
    desc.num_tables = T;
    desc.dim = D;
    desc.table_dtype = EMB_F32;
    desc.mode = mode;
    desc.batch = B;
    desc.num_lookups = nl;
    desc.max_table_rows = 1000;
    int rc = emb_bag_forward(&desc, d_tab, (const int64_t*)d_toff, (const int64_t*)d_idx,
                             (const int64_t*)d_off, NULL, (float*)d_out, stream);
    if (rc != EMB_OK) {
      fprintf(stderr, "emb_bag_forward: %s\n", emb_bag_status_string(rc));
      return 3;
    }
    rc = emb_bag_validate(&desc, (const int64_t*)d_toff, (const int64_t*)d_idx,
                          (const int64_t*)d_off, (int64_t*)d_bad, stream);
    if (rc != EMB_OK) return 3;
    CHECK(hipStreamSynchronize(stream));
    CHECK(hipMemcpy(out, d_out, (size_t)B * T * D * sizeof(float), hipMemcpyDeviceToHost));
    for (int t = 0; t < T; ++t)
      for (int b = 0; b < B; ++b)
        for (int d = 0; d < D; ++d) {
          double acc = 0.0, mag = 0.0;
          const int64_t s = off[t * B + b], e = off[t * B + b + 1];
          for (int64_t j = s; j < e; ++j) {
            const double x = tab[(toff[t] + idx[j]) * D + d];
            acc += x;
            mag += fabs(x);
          }
          if (mode == EMB_MEAN && e > s) {
            acc /= (double)(e - s);
            mag /= (double)(e - s);
          }
          const double got = out[(size_t)b * T * D + t * D + d];
          if (fabs(got - acc) > 1e-5 * mag || (e == s && got != 0.0)) ++failures;
        }
  }
  int64_t bad = -1;
  CHECK(hipMemcpy(&bad, d_bad, sizeof bad, hipMemcpyDeviceToHost));
  if (bad != 0) ++failures;
  /* host-side argument errors come back as codes */
  {
    emb_bag_desc d2 = {0};
    d2.num_tables = 1; d2.dim = 6; d2.batch = 1;
    if (emb_bag_forward(&d2, d_tab, d_toff, d_idx, d_off, NULL, d_out, stream) != EMB_ERR_BAD_DIM)
      ++failures;
  }
  if (failures) {
    fprintf(stderr, "C ABI check FAILED: %d\n", failures);
    return 1;
  }
  printf("C ABI OK: version %d, %lld lookups, %d bags, sum and mean\n", emb_bag_version(),
         (long long)nl, T * B);
  hipFree(d_tab); hipFree(d_toff); hipFree(d_idx); hipFree(d_off); hipFree(d_out); hipFree(d_bad);
  free(tab); free(off); free(idx); free(out);
  return 0;
}
