/*
 * Host-side planning of the library under AddressSanitizer / UndefinedBehaviorSanitizer: this
 * program is linked against a build of libembbag whose host code is instrumented, and drives
 * emb_bag_plan_forward / emb_bag_plan_forward_mixed (pure host code: no GPU is needed) through
 * table counts around the limits of the table list (1024) and of the 16-bit table numbers
 * (65535), every lanes-per-row class, every element type and mode, per-table bag lengths and
 * the tuning keys.  Any finding of a sanitizer ends the program with a non-zero status.
 * Built and run by tests/test_sanitizers.py.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "emb_bag.h"

static uint64_t state = 0x5EED5A17ull;
static uint32_t rnd(void) {
  state = state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(state >> 33);
}

static long calls = 0, ok_calls = 0;
static const emb_bag_tuning* desc_tuning = NULL; /* what the descriptors of a pass carry */

static void plan_uniform(int32_t T, int64_t B, int32_t D, int dtype, int mode, double avg,
                         const float* lens, int weights, int64_t max_rows, const void* hot) {
  emb_bag_desc d;
  memset(&d, 0, sizeof d);
  d.num_tables = T;
  d.dim = D;
  d.table_dtype = dtype;
  d.mode = mode;
  d.batch = B;
  d.num_lookups = (int64_t)((double)T * (double)B * avg);
  d.max_table_rows = max_rows;
  d.table_avg_len = lens;
  d.hot_rows = (const int64_t*)hot;
  d.tuning = desc_tuning;
  /* exactly min(T, 1024) entries: a write beyond them is an overflow the sanitizer sees */
  const int n = T < 1024 ? T : 1024;
  uint16_t* order = (uint16_t*)malloc((size_t)n * sizeof(uint16_t));
  emb_bag_plan p;
  int rc = emb_bag_plan_forward(&d, weights, 0, &p, order);
  ++calls;
  if (rc == EMB_OK) {
    ++ok_calls;
    for (int32_t w = 1; w < p.num_launches && w < 70000; w += (p.num_launches > 64 ? 997 : 1)) {
      emb_bag_plan q;
      rc = emb_bag_plan_forward(&d, weights, w, &q, order);
      ++calls;
      if (rc != EMB_OK) {
        fprintf(stderr, "launch %d of %d: status %d\n", w, p.num_launches, rc);
        exit(3);
      }
    }
    /* one past the last launch is an error code, not a crash */
    if (emb_bag_plan_forward(&d, weights, p.num_launches, &p, order) != EMB_ERR_BAD_SIZE) exit(4);
  }
  free(order);
}

static void plan_mixed(int32_t T, int64_t B, const int32_t* dims, int dtype, int mode, double avg,
                       const float* lens, int weights, int64_t max_bytes) {
  emb_bag_mixed_desc d;
  memset(&d, 0, sizeof d);
  d.num_tables = T;
  d.table_dtype = dtype;
  d.mode = mode;
  d.batch = B;
  d.num_lookups = (int64_t)((double)T * (double)B * avg);
  d.max_table_bytes = max_bytes;
  d.dims = dims;
  d.table_avg_len = lens;
  d.tuning = desc_tuning;
  const int n = T < 1024 ? T : 1024;
  uint16_t* order = (uint16_t*)malloc((size_t)n * sizeof(uint16_t));
  emb_bag_plan p;
  int rc = emb_bag_plan_forward_mixed(&d, weights, 0, &p, order);
  ++calls;
  if (rc == EMB_OK) {
    ++ok_calls;
    for (int32_t w = 1; w < p.num_launches; ++w) {
      emb_bag_plan q;
      if (emb_bag_plan_forward_mixed(&d, weights, w, &q, order) != EMB_OK) exit(5);
      ++calls;
    }
  }
  free(order);
}

int main(void) {
  static const int32_t tables[] = {1, 2, 7, 8, 60, 1023, 1024, 1025, 2600, 65535, 65536, 70000};
  static const int64_t batches[] = {1, 37, 4096, 1 << 20};
  static const double lengths[] = {0.4, 3.0, 30.0, 400.0};
  /* row sizes 16 B .. 64 KiB in fp32 elements: every lanes-per-row class, several slabs */
  static const int32_t dims_f32[] = {4, 8, 12, 16, 32, 64, 100, 128, 256, 260, 1024, 4096, 16384};
  static const char* keys[][2] = {{"depth", "0"}, {"depth", "1"}, {"depth", "16"}, {"stream", "1"},
                                  {"stream", "0"}, {"xcd_remap", "1"}, {"xcd_pieces", "8"},
                                  {"bags_per_group", "63"}, {"bags_per_wave", "32"},
                                  {"per_table_launch", "1"}, {"fuse", "0"}, {"addressing", "1"},
                                  {"hot_split", "1"}, {"station", "1"}};
  const int nkeys = (int)(sizeof keys / sizeof keys[0]);
  float* lens = (float*)malloc(70000 * sizeof(float));
  int32_t* dims = (int32_t*)malloc(70000 * sizeof(int32_t));
  int64_t fake_hot = 0; /* the plan only tests the pointer */
  /* the last pass: descriptors that carry their own tuning, in a heap block of its exact size */
  emb_bag_tuning* own = (emb_bag_tuning*)malloc(sizeof(emb_bag_tuning));
  if (emb_bag_tuning_defaults(own) != EMB_OK || emb_bag_tuning_defaults(NULL) != EMB_ERR_NULL_PTR)
    return 11;
  own->depth = 4;
  own->station = 1;
  own->xcd_pieces = 8;
  own->bags_per_wave = 32;
  own->blocks_per_cu = 2;
  for (int k = -1; k <= nkeys; ++k) {
    if (k == nkeys) desc_tuning = own;
    if (k >= 0 && k < nkeys && emb_bag_set_tuning(keys[k][0], atoll(keys[k][1])) != EMB_OK)
      return 6;
    for (size_t ti = 0; ti < sizeof tables / sizeof tables[0]; ++ti) {
      const int32_t T = tables[ti];
      /* one launch per table makes T launches of 2 KB each: the table counts around the list
         limit are enough for it, and the key sweeps stay below the 16-bit limit */
      if (k >= 0 && (T > 2600 || (k < nkeys && !strcmp(keys[k][0], "per_table_launch") && T > 1025)))
        continue;
      for (int i = 0; i < T; ++i) lens[i] = (rnd() % 4 == 0) ? (float)(rnd() % 200) : (float)(rnd() % 5);
      for (size_t bi = 0; bi < sizeof batches / sizeof batches[0]; ++bi) {
        const int64_t B = batches[bi];
        if ((double)T * (double)B > 3e9) continue;
        for (size_t li = 0; li < sizeof lengths / sizeof lengths[0]; ++li) {
          for (size_t di = 0; di < sizeof dims_f32 / sizeof dims_f32[0]; ++di) {
            if ((k >= 0 || T > 2600) && di % 3) continue; /* a thinner grid where calls are costly */
            const int32_t D = dims_f32[di];
            const int dtype = (int)(rnd() % 5), mode = (int)(rnd() % 3);
            const int32_t Dq = dtype >= 3 ? (D >= 1016 ? 1016 : D + 8 - (D % 16 ? D % 16 : 0) - 8 + 8) : D;
            plan_uniform(T, B, dtype >= 3 ? (Dq < 8 ? 8 : Dq) : D, dtype, mode, lengths[li],
                         rnd() % 2 ? lens : NULL, mode == EMB_SUM && rnd() % 2,
                         rnd() % 4 ? 4000000 : 0, rnd() % 3 == 0 ? &fake_hot : NULL);
          }
          /* tables of different widths (rows of at most 1 KiB) */
          const int dtype = (int)(rnd() % 3), mode = (int)(rnd() % 3);
          for (int i = 0; i < T; ++i) {
            const int32_t units = 1 + (int32_t)(rnd() % 64);  /* 16-byte units */
            dims[i] = dtype == 0 ? units * 4 : units * 8;
          }
          plan_mixed(T, B, dims, dtype, mode, lengths[li], rnd() % 2 ? lens : NULL,
                     mode == EMB_SUM && rnd() % 2, rnd() % 4 ? (int64_t)3 << 30 : 0);
        }
      }
    }
    if (k >= 0 && k < nkeys) {  /* back to the default */
      static const char* defaults[][2] = {{"depth", "0"}, {"stream", "-1"}, {"xcd_remap", "-1"},
                                          {"xcd_pieces", "0"}, {"bags_per_group", "0"},
                                          {"bags_per_wave", "0"}, {"per_table_launch", "0"},
                                          {"fuse", "1"}, {"addressing", "0"}, {"hot_split", "0"},
                                          {"station", "0"}};
      for (size_t i = 0; i < sizeof defaults / sizeof defaults[0]; ++i)
        if (emb_bag_set_tuning(defaults[i][0], atoll(defaults[i][1])) != EMB_OK) return 7;
    }
  }
  /* argument errors come back as codes */
  emb_bag_plan p;
  if (emb_bag_plan_forward(NULL, 0, 0, &p, NULL) != EMB_ERR_NULL_PTR) return 8;
  {
    emb_bag_desc d;
    memset(&d, 0, sizeof d);
    d.num_tables = 8;
    d.dim = 64;
    d.batch = 128;
    d.num_lookups = 8 * 128 * 100;
    d.max_table_rows = 100000; /* buffer addressing, which the LDS station needs */
    d.tuning = own;
    own->depth = 3; /* not a depth */
    if (emb_bag_plan_forward(&d, 0, 0, &p, NULL) != EMB_ERR_BAD_TUNING) return 12;
    own->depth = 8;
    if (emb_bag_plan_forward(&d, 0, 0, &p, NULL) != EMB_OK || p.depth != 8 || p.station != 1)
      return 13;
  }
  free(own);
  if (emb_bag_set_tuning("no such key", 1) != EMB_ERR_BAD_TUNING) return 9;
  printf("sanitized planning: %ld calls, %ld accepted\n", calls, ok_calls);
  free(lens);
  free(dims);
  return ok_calls > 1000 ? 0 : 10;
}
