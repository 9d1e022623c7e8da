/*
 * CPU oracle for the multi-table EmbeddingBag forward.  TEST INFRASTRUCTURE ONLY.
 *
 * This is the plain definition of what the embedding stage computes, written out slowly and
 * obviously: only tests, the smoke check and the benchmark's cpu_baseline leg may use it.  It
 * shares no code, header, table or helper with the HIP library or with the input generator.
 *
 * What is computed (paper Sec. 3.1, Algorithm 1 and the per-thread description that follows
 * it): for every table t and every sample b of the batch, the bag (t, b) owns the lookups
 * indices[offsets[t*B+b] .. offsets[t*B+b+1]); each lookup names a row of table t; the bag's
 * output is the element-wise sum of those rows (a "gather" then a "reduce"), one vector of
 * length ED per (sample, table).  The output of table t is the [BS, ED] block at columns
 * t*D .. t*D+D of the [B, out_ld] result.
 *
 * Readings taken where the paper is silent or garbled:
 *   - Algorithm 1 prints the accumulator load/store inside the lookup loop; the accumulator is
 *     taken to start at zero once per (sample, element) and to be stored once after the last
 *     lookup, which is what "one [BS, ED] output per table" requires.
 *   - "mean" appears only in the name of the kernel the paper studies: mean = sum / bag length,
 *     and an empty bag gives 0.
 *   - per-sample weights are not in the paper: out = sum_j w_j * row_j, sum mode only.
 *   - max pooling is not in the paper either (its kernel is the sum/mean one): out = max_j row_j
 *     element by element, 0 for an empty bag; the maximum is an element of the table, so no
 *     rounding is involved except in the dequantisation of quantised rows.
 *   - summation order is not fixed by the paper: this oracle adds in index order, in fp64.
 *
 * Arithmetic: every table element is widened exactly (fp32, IEEE half or bfloat16 -> fp64; a
 * quantised element is scale * code + bias evaluated in fp64, the code being an unsigned byte or an
 * E4M3 8-bit float) and accumulated in fp64.  Alongside each output element the oracle returns bound = sum_j |w_j *
 * x_j| (divided by the bag length in mean mode), the scale of the rounding-error tolerance.
 *
 * Parity pins (tests/test_oracle_pins.py): exact rational brute force on tiny inputs, index
 * histograms through identity tables, the one-item case, mean = sum / len, permutation and
 * linearity invariants on integer tables, and agreement with a sparse-matrix product and with
 * torch's CPU embedding_bag as second opinions.  The paper prints no output value of the
 * operator, so beyond those pins the numbers rest on the definition above.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_OFFSETS (-2)
#define ORACLE_ERR_INDEX (-3)

/* IEEE 754 binary16 bit pattern -> double, exactly (subnormals, infinities, NaN included). */
static double half_bits_to_double(uint16_t h) {
  const int sign = (h >> 15) & 1;
  const int expo = (h >> 10) & 0x1F;
  const int frac = h & 0x3FF;
  double v;
  if (expo == 0)
    v = ldexp((double)frac, -24); /* subnormal: frac * 2^-10 * 2^-14 */
  else if (expo == 31)
    v = frac ? NAN : INFINITY;
  else
    v = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
  return sign ? -v : v;
}

/* bfloat16 bit pattern -> double, exactly: a bfloat16 is the upper 16 bits of an IEEE binary32. */
static double bf16_bits_to_double(uint16_t h) {
  const uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/*
 * OCP 8-bit floating point, format E4M3 (1 sign, 4 exponent bits with bias 7, 3 fraction bits; no
 * infinities; S.1111.111 is NaN; largest finite value 448) -> double, exactly.
 */
static double e4m3_bits_to_double(uint8_t c) {
  const int sign = (c >> 7) & 1;
  const int expo = (c >> 3) & 0xF;
  const int frac = c & 0x7;
  double v;
  if (expo == 0)
    v = ldexp((double)frac, -9); /* subnormal: frac/8 * 2^-6 */
  else if (expo == 15 && frac == 7)
    v = NAN;
  else
    v = ldexp((double)(8 + frac), expo - 10); /* (1 + frac/8) * 2^(expo-7) */
  return sign ? -v : v;
}

/*
 * Element d of an arena row as a double, and the magnitude the error bound charges for it.
 * dtype 3 and 4 are row-wise quantised tables: a row is D 8-bit codes followed by an fp32 scale
 * and an fp32 bias (row stride D + 8 bytes), and element d is scale * value(code_d) + bias, where
 * value() is the unsigned integer (dtype 3) or the E4M3 number (dtype 4) the code stands for; its
 * magnitude for the bound is |scale * value| + |bias|, the two terms an implementation adds.
 */
static double table_elem(const void* tables, int dtype, int64_t arena_row, int64_t D, int64_t d,
                         double* magnitude) {
  double x;
  if (dtype == 3 || dtype == 4) {
    const uint8_t* row = (const uint8_t*)tables + arena_row * (D + 8);
    float scale, bias;
    memcpy(&scale, row + D, sizeof scale);
    memcpy(&bias, row + D + 4, sizeof bias);
    const double code = dtype == 3 ? (double)row[d] : e4m3_bits_to_double(row[d]);
    const double sc = (double)scale * code;
    *magnitude = fabs(sc) + fabs((double)bias);
    return sc + (double)bias;
  }
  if (dtype == 1)
    x = half_bits_to_double(((const uint16_t*)tables)[arena_row * D + d]);
  else if (dtype == 2)
    x = bf16_bits_to_double(((const uint16_t*)tables)[arena_row * D + d]);
  else
    x = (double)((const float*)tables)[arena_row * D + d];
  *magnitude = fabs(x);
  return x;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/*
 * All pointers are HOST pointers.
 *   T, B, D        tables, batch, embedding dimension
 *   dtype          0 = fp32 tables, 1 = fp16 tables (raw half bit patterns),
 *                  2 = bfloat16 tables (raw bit patterns),
 *                  3 = row-wise quantised tables: D uint8 codes + fp32 scale + fp32 bias per row
 *                  4 = the same with E4M3 8-bit floating-point codes
 *   mode           0 = sum, 1 = mean, 2 = max (bound = magnitude of the element that is the max)
 *   tables         arena [sum_t R_t, D], row-major ([sum_t R_t, D + 8] bytes for dtype 3)
 *   table_offsets  [T+1] first arena row of each table (so R_t = table_offsets[t+1]-table_offsets[t])
 *   indices        [NL] table-local row ids
 *   offsets        [T*B+1] CSR over bags in (t, b) order
 *   weights        [NL] or NULL (sum mode only)
 *   out_ld         leading dimension of ref / bound in elements (>= T*D)
 *   ref, bound     [B, out_ld] fp64 outputs; only columns [0, T*D) are written
 *   strict         [B, out_ld] fp64 output or NULL: the sum of |w * element| with the element taken
 *                  as one number (for quantised rows |scale * value + bias|, which is at most
 *                  what `bound` charges; the same as `bound` for the other element types)
 * Returns ORACLE_OK or a negative code (bad argument, non-monotone offsets, index out of range).
 */
int oracle_emb_bag(int32_t T, int64_t B, int32_t D, int32_t dtype, int32_t mode,
                   const void* tables, const int64_t* table_offsets, const int64_t* indices,
                   const int64_t* offsets, const float* weights, int64_t out_ld, double* ref,
                   double* bound, double* strict) {
  if (T < 1 || B < 0 || D < 1 || (dtype < 0 || dtype > 4) || (mode < 0 || mode > 2))
    return ORACLE_ERR_ARG;
  if (out_ld < (int64_t)T * D) return ORACLE_ERR_ARG;
  if (weights && mode != 0) return ORACLE_ERR_ARG;
  if (B == 0) return ORACLE_OK;
  if (!tables || !table_offsets || !offsets || !ref || !bound) return ORACLE_ERR_ARG;

  const int64_t nbags = (int64_t)T * B;
  if (offsets[0] != 0) return ORACLE_ERR_OFFSETS;
  for (int64_t g = 0; g < nbags; ++g)
    if (offsets[g + 1] < offsets[g]) return ORACLE_ERR_OFFSETS;
  if (offsets[nbags] > 0 && !indices) return ORACLE_ERR_ARG;

  int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t g = 0; g < nbags; ++g) {
    const int64_t t = g / B;
    const int64_t b = g % B;
    const int64_t R = table_offsets[t + 1] - table_offsets[t];
    const int64_t s = offsets[g];
    const int64_t e = offsets[g + 1];
    int bad = 0;
    for (int64_t j = s; j < e; ++j)
      if (indices[j] < 0 || indices[j] >= R) bad = 1;
    if (bad) {
#pragma omp atomic write
      status = ORACLE_ERR_INDEX;
      continue;
    }
    for (int64_t d = 0; d < D; ++d) {
      double acc = 0.0;
      double mag = 0.0;
      double smag = 0.0;
      for (int64_t j = s; j < e; ++j) {
        double ax;
        const double x = table_elem(tables, dtype, table_offsets[t] + indices[j], D, d, &ax);
        if (mode == 2) {
          if (j == s || x > acc) {
            acc = x;
            mag = ax;
            smag = fabs(x);
          }
          continue;
        }
        const double w = weights ? (double)weights[j] : 1.0;
        acc += w * x;
        mag += fabs(w) * ax;
        smag += fabs(w * x);
      }
      if (mode == 1) {
        if (e > s) {
          acc /= (double)(e - s);
          mag /= (double)(e - s);
          smag /= (double)(e - s);
        } else {
          acc = 0.0;
          mag = 0.0;
          smag = 0.0;
        }
      }
      ref[b * out_ld + t * D + d] = acc;
      bound[b * out_ld + t * D + d] = mag;
      if (strict) strict[b * out_ld + t * D + d] = smag;
    }
  }
  return status;
}
