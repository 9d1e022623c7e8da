/*
 * Host-path cost of emb_bag_forward, measured from plain C (no Python, no ctypes): at inference
 * batch sizes the kernel lasts a few microseconds and what the caller sees is the time the call
 * itself takes on the host plus the dispatch gap between back-to-back launches.
 *
 *   c_abi_latency [T R D B L [iterations]]      defaults: 8 100000 64 256 20 2000 (the smallest
 *                                               benchmark configuration: fp32, fixed pooling,
 *                                               uniform row ids, sum)
 *
 * Prints one JSON object:
 *   plan_us_per_call     host time of emb_bag_plan_forward (the planning a forward call does,
 *                        without the launch)
 *   host_us_per_call     host time inside emb_bag_forward, calls issued back to back
 *   eager_us_per_step    wall time per call of that loop including the final synchronise
 *   kernel_us            device time of one call between two events on the stream (median)
 * Table values and row ids come from a fixed linear congruential generator; results are not
 * checked here (c_abi_driver.c does that).  Built by paper_2410_22249_amd/build.py.
 */
#define _POSIX_C_SOURCE 199309L
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <time.h>

#include "emb_bag.h"

#define CHECK(x)                                                     \
  do {                                                               \
    hipError_t e_ = (x);                                             \
    if (e_ != hipSuccess) {                                          \
      fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_)); \
      return 2;                                                      \
    }                                                                \
  } while (0)

static double now_us(void) {
  struct timespec ts;
  clock_gettime(CLOCK_MONOTONIC, &ts);
  return (double)ts.tv_sec * 1e6 + (double)ts.tv_nsec * 1e-3;
}

static uint64_t lcg_state = 0x5EED0B00ull;
static uint32_t lcg(void) {
  lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(lcg_state >> 33);
}

static int cmp_float(const void* a, const void* b) {
  const float x = *(const float*)a, y = *(const float*)b;
  return x < y ? -1 : (x > y ? 1 : 0);
}

int main(int argc, char** argv) {
  const int64_t T = argc > 1 ? atoll(argv[1]) : 8;
  const int64_t R = argc > 2 ? atoll(argv[2]) : 100000;
  const int64_t D = argc > 3 ? atoll(argv[3]) : 64;
  const int64_t B = argc > 4 ? atoll(argv[4]) : 256;
  const int64_t L = argc > 5 ? atoll(argv[5]) : 20;
  const int iters = argc > 6 ? atoi(argv[6]) : 2000;
  if (T < 1 || R < 1 || D < 4 || D % 4 || B < 1 || L < 0 || iters < 1 || iters > 1000000 ||
      T * R * D > ((int64_t)1 << 31) || T * B * L > ((int64_t)1 << 28)) {
    fprintf(stderr, "bad shape\n");
    return 2;
  }
  const int64_t nl = T * B * L, bags = T * B;
  float* tab = (float*)malloc((size_t)(T * R * D) * sizeof(float));
  int64_t* toff = (int64_t*)malloc((size_t)(T + 1) * sizeof(int64_t));
  int64_t* off = (int64_t*)malloc((size_t)(bags + 1) * sizeof(int64_t));
  int64_t* idx = (int64_t*)malloc((size_t)(nl > 0 ? nl : 1) * sizeof(int64_t));
  if (!tab || !toff || !off || !idx) return 2;
  for (int64_t i = 0; i < T * R * D; ++i) tab[i] = ((int)(lcg() % 2001) - 1000) * 1e-4f;
  for (int64_t t = 0; t <= T; ++t) toff[t] = t * R;
  for (int64_t g = 0; g <= bags; ++g) off[g] = g * L;
  for (int64_t j = 0; j < nl; ++j) idx[j] = (int64_t)(lcg() % (uint32_t)R);

  void *d_tab, *d_toff, *d_idx, *d_off, *d_out;
  CHECK(hipMalloc(&d_tab, (size_t)(T * R * D) * sizeof(float)));
  CHECK(hipMalloc(&d_toff, (size_t)(T + 1) * sizeof(int64_t)));
  CHECK(hipMalloc(&d_idx, (size_t)(nl > 0 ? nl : 1) * sizeof(int64_t)));
  CHECK(hipMalloc(&d_off, (size_t)(bags + 1) * sizeof(int64_t)));
  CHECK(hipMalloc(&d_out, (size_t)(B * T * D) * sizeof(float)));
  CHECK(hipMemcpy(d_tab, tab, (size_t)(T * R * D) * sizeof(float), hipMemcpyHostToDevice));
  CHECK(hipMemcpy(d_toff, toff, (size_t)(T + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
  CHECK(hipMemcpy(d_idx, idx, (size_t)nl * sizeof(int64_t), hipMemcpyHostToDevice));
  CHECK(hipMemcpy(d_off, off, (size_t)(bags + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
  hipStream_t stream;
  CHECK(hipStreamCreate(&stream));

  emb_bag_desc desc = {0};
  desc.num_tables = (int32_t)T;
  desc.dim = (int32_t)D;
  desc.table_dtype = EMB_F32;
  desc.mode = EMB_SUM;
  desc.batch = B;
  desc.num_lookups = nl;
  desc.max_table_rows = R;

#define FORWARD()                                                                              \
  emb_bag_forward(&desc, d_tab, (const int64_t*)d_toff, (const int64_t*)d_idx,                 \
                  (const int64_t*)d_off, NULL, (float*)d_out, stream)

  for (int i = 0; i < 20; ++i)
    if (FORWARD() != EMB_OK) return 3;
  CHECK(hipStreamSynchronize(stream));

  /* planning alone (no launch, no HIP call) */
  emb_bag_plan plan;
  double t0 = now_us();
  for (int i = 0; i < iters; ++i)
    if (emb_bag_plan_forward(&desc, 0, 0, &plan, NULL) != EMB_OK) return 3;
  const double plan_us = (now_us() - t0) / iters;

  /* calls back to back: host time inside the calls, and wall time per step with the final wait */
  double in_calls = 0.0;
  t0 = now_us();
  for (int i = 0; i < iters; ++i) {
    const double a = now_us();
    if (FORWARD() != EMB_OK) return 3;
    in_calls += now_us() - a;
  }
  CHECK(hipStreamSynchronize(stream));
  const double eager_us = (now_us() - t0) / iters;
  const double host_us = in_calls / iters;

  /* device time of one call */
  enum { NK = 101 };
  float kern[NK];
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  for (int i = 0; i < NK; ++i) {
    CHECK(hipEventRecord(e0, stream));
    if (FORWARD() != EMB_OK) return 3;
    CHECK(hipEventRecord(e1, stream));
    CHECK(hipStreamSynchronize(stream));
    CHECK(hipEventElapsedTime(&kern[i], e0, e1));
  }
  qsort(kern, NK, sizeof(float), cmp_float);

  printf("{\"shape\": \"T=%lld R=%lld D=%lld B=%lld L=%lld fp32 sum\", \"iterations\": %d, "
         "\"plan_us_per_call\": %.3f, \"host_us_per_call\": %.3f, \"eager_us_per_step\": %.3f, "
         "\"kernel_us\": %.3f, \"kernel_us_min\": %.3f, \"launches\": %d, \"kernel\": %d}\n",
         (long long)T, (long long)R, (long long)D, (long long)B, (long long)L, iters, plan_us,
         host_us, eager_us, kern[NK / 2] * 1e3, kern[0] * 1e3, plan.num_launches, plan.kernel);
  hipFree(d_tab); hipFree(d_toff); hipFree(d_idx); hipFree(d_off); hipFree(d_out);
  free(tab); free(toff); free(off); free(idx);
  return 0;
}
