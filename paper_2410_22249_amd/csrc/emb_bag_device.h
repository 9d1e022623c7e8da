// Device-side building blocks shared by the embedding-bag kernels (gfx950, wave64): constants,
// launch parameters, cross-lane helpers, the per-segment accumulate and the gather of one bag.
// Included by the kernel sources only; nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/emb_bag.h"
#include "emb_bag_params.h"

namespace embbag {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int64_t uniform64(int64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ int64_t shfl64(int64_t v, int src) {
  const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)(uint64_t)v, src);
  const uint32_t hi = (uint32_t)__shfl((int)(uint32_t)((uint64_t)v >> 32), src);
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ float as_float(uint32_t u) { return __builtin_bit_cast(float, u); }

// Row-wise quantised element types: D one-byte codes, then an fp32 scale and an fp32 bias.
template <int ELEM>
struct IsQuant {
  static constexpr bool value = ELEM == EMB_U8ROW || ELEM == EMB_FP8ROW;
};

// Elements of the output a lane owns (its 16-byte segment of the row): 4 fp32 elements, 8 fp16 /
// bf16 elements, or 16 one-byte codes.
template <int ELEM>
struct OutCount {
  static constexpr int value = ELEM == EMB_F32 ? 4 : (IsQuant<ELEM>::value ? 16 : 8);
};

// fp32 accumulators a lane keeps: one per element, plus one more for quantised rows (the sum of
// the row biases) or for max pooling (the number of valid lookups seen).
template <int ELEM, int OP = kOpSum>
struct AccCount {
  static constexpr int value = OutCount<ELEM>::value + ((IsQuant<ELEM>::value || OP == kOpMax) ? 1 : 0);
};

template <int ELEM, int OP>
__device__ __forceinline__ void init_acc(float* acc) {
  constexpr int NOUT = OutCount<ELEM>::value;
#pragma unroll
  for (int i = 0; i < AccCount<ELEM, OP>::value; ++i)
    acc[i] = (OP == kOpMax && i < NOUT) ? -__builtin_inff() : 0.0f;
}

// One 16-byte segment of a row into the accumulators: 4 fp32 elements, 8 fp16 / bf16 elements
// widened exactly to fp32, or 16 codes (unsigned bytes or E4M3 numbers, both exact in fp32) of a
// row-wise quantised row.  For the latter the row's
// scale and bias sit in the last 8 bytes of the row, i.e. in words z and w of lane `meta_lane`'s
// segment.
//   kOpSum / kOpWeighted: acc += w * element; for quantised rows acc[i] collects w * scale *
//     code_i and acc[16] collects w * bias, added to every element at the end of the bag (a
//     lookup that fetched nothing has scale = bias = 0).
//   kOpMax: acc = max(acc, element) where w != 0 marks a valid lookup (an invalid one fetched
//     zeros, which must not take part); the last accumulator counts the valid lookups.
template <int ELEM, int OP>
__device__ __forceinline__ void accumulate(float* acc, u32x4 r, float w, int meta_lane) {
  constexpr bool WEIGHTED = OP == kOpWeighted;
  constexpr bool MAXP = OP == kOpMax;
  constexpr int NOUT = OutCount<ELEM>::value;
  const float skip = -__builtin_inff();
  if constexpr (IsQuant<ELEM>::value) {
    float scale = as_float((uint32_t)__shfl((int)r.z, meta_lane));
    float bias = as_float((uint32_t)__shfl((int)r.w, meta_lane));
    if constexpr (WEIGHTED) {
      scale *= w;
      bias *= w;
    }
    const uint32_t u[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float codes[4];
      if constexpr (ELEM == EMB_FP8ROW) {  // two E4M3 codes per conversion instruction
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)u[i], false);
        const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)u[i], true);
        codes[0] = lo.x;
        codes[1] = lo.y;
        codes[2] = hi.x;
        codes[3] = hi.y;
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) codes[k] = (float)((u[i] >> (8 * k)) & 0xFFu);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float code = codes[k];
        if constexpr (MAXP) {
          const float v = __builtin_fmaf(scale, code, bias);
          acc[4 * i + k] = __builtin_fmaxf(acc[4 * i + k], w != 0.0f ? v : skip);
        } else {
          acc[4 * i + k] = __builtin_fmaf(scale, code, acc[4 * i + k]);
        }
      }
    }
    acc[16] += MAXP ? w : bias;
  } else if constexpr (ELEM == EMB_F16 && !MAXP) {
    // acc += w * half, one instruction per element: the mixed-precision FMA reads the half
    // straight from its half of the register (the product of a half and a float is exact in
    // the FMA, so the result equals widening first and adding, or multiplying, afterwards)
    const uint32_t u[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if constexpr (WEIGHTED) {
        asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[0,0,0] op_sel_hi:[1,0,0]"
            : "+v"(acc[2 * i]) : "v"(u[i]), "v"(w));
        asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[1,0,0] op_sel_hi:[1,0,0]"
            : "+v"(acc[2 * i + 1]) : "v"(u[i]), "v"(w));
      } else {
        asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel:[0,0,0] op_sel_hi:[1,0,0]"
            : "+v"(acc[2 * i]) : "v"(u[i]));
        asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel:[1,0,0] op_sel_hi:[1,0,0]"
            : "+v"(acc[2 * i + 1]) : "v"(u[i]));
      }
    }
  } else if constexpr (ELEM != EMB_F32) {
    const uint32_t u[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float lo, hi;
      if constexpr (ELEM == EMB_F16) {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        const h2 h = __builtin_bit_cast(h2, u[i]);
        lo = (float)h.x;
        hi = (float)h.y;
      } else {  // bfloat16 is the upper half of a binary32: widening is a shift
        lo = as_float(u[i] << 16);
        hi = as_float(u[i] & 0xFFFF0000u);
      }
      if constexpr (MAXP) {
        acc[2 * i] = __builtin_fmaxf(acc[2 * i], w != 0.0f ? lo : skip);
        acc[2 * i + 1] = __builtin_fmaxf(acc[2 * i + 1], w != 0.0f ? hi : skip);
      } else if constexpr (WEIGHTED) {
        acc[2 * i] = __builtin_fmaf(w, lo, acc[2 * i]);
        acc[2 * i + 1] = __builtin_fmaf(w, hi, acc[2 * i + 1]);
      } else {
        acc[2 * i] += lo;
        acc[2 * i + 1] += hi;
      }
    }
    if constexpr (MAXP) acc[NOUT] += w;
  } else {
    const float x[4] = {as_float(r.x), as_float(r.y), as_float(r.z), as_float(r.w)};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if constexpr (MAXP)
        acc[i] = __builtin_fmaxf(acc[i], w != 0.0f ? x[i] : skip);
      else if constexpr (WEIGHTED)
        acc[i] = __builtin_fmaf(w, x[i], acc[i]);
      else
        acc[i] += x[i];
    }
    if constexpr (MAXP) acc[NOUT] += w;
  }
}

// What lane i holds for lookup i of a chunk of up to 64 lookups: where the row starts inside its
// table (a 32-bit byte offset for buffer addressing, kBufSentinel = no row; or a 64-bit byte
// offset, -1 = no row) and the lookup's weight.
template <bool BUF>
struct ChunkLookups {
  uint32_t voff;
  int64_t roff;
  float w;
};

// Request lookup `lane` of the chunk that starts at position c of `indices` (n lookups, n <= 64):
// one coalesced non-temporal load of the row ids (and one of the weights).
template <bool WEIGHTED>
__device__ __forceinline__ void load_chunk(const int64_t* __restrict__ indices,
                                           const float* __restrict__ weights, int64_t c, int n,
                                           int lane, int64_t* idx, float* w) {
  *idx = -1;
  *w = 0.0f;
  if (lane < n) {
    *idx = __builtin_nontemporal_load(indices + c + lane);
    if constexpr (WEIGHTED) *w = __builtin_nontemporal_load(weights + c + lane);
  }
}

// Row id -> byte offset of the row, once per lookup.  A row id outside [0, R) names no row.
template <bool BUF>
__device__ __forceinline__ ChunkLookups<BUF> chunk_offsets(int64_t idx, float w, int64_t R,
                                                           uint32_t row_bytes) {
  ChunkLookups<BUF> q;
  const bool idx_ok = (uint64_t)idx < (uint64_t)R;
  q.voff = kBufSentinel;
  q.roff = -1;
  q.w = w;
  if constexpr (BUF) {
    if (idx_ok) q.voff = (uint32_t)idx * row_bytes;
  } else {
    if (idx_ok) q.roff = idx * (int64_t)row_bytes;
  }
  return q;
}

// Gather the lookups that sit in slots [j_lo, j_hi) of a chunk (slot = lane that holds the
// lookup) and add their rows into acc.  LPR is the number of lanes per row (0: decided per table
// at run time); 2^gl rows share one load instruction, group g of the wavefront taking slot
// (step << gl) + g; DEPTH load instructions are issued back to back before the first is
// consumed.  NT selects the non-temporal cache policy for the row loads (rows that are not
// re-used within a batch), the default policy otherwise.  A slot outside the range, a lane
// beyond the row's end and a lookup without a row fetch nothing: their offset fails the
// buffer's range check (zeros, no memory traffic), or the load is skipped (64-bit addressing).
//
// The two per-load tests are compiled in only where they can fire.  RANGE: slots outside
// [j_lo, j_hi) may hold a lookup (the hot / cold split), or a batch of DEPTH steps can run past
// slot 63 and wrap (DEPTH steps cover more than 64 slots); without it j_lo is 0 and the slots
// from j_hi on hold "no row" already, as load_chunk and chunk_offsets leave them.  PARTIAL:
// the row does not fill its lane group (lane_ok is false for some lanes).
// The LDS station (LDS = true; buffer addressing, sum pooling): the DEPTH row loads of a batch
// bypass the registers (buffer load to LDS, 16 bytes per lane: load d of the wavefront fills the
// d-th 1-KiB slot of the wavefront's DEPTH KiB of dynamic LDS) and each lane reads its segment
// back when the load has landed.  This is the shared-memory prefetch station of paper Sec. 4.2.
// The compiler does not track such a load in its wait-count insertion, so the wait is placed
// here: loads complete in the order issued, stores (of an earlier bag) in theirs, so once at
// most DEPTH - 1 - d vector memory operations are outstanding, load d and everything issued
// before the batch have completed, whatever else is in flight.
template <int D, int DEPTH, int ELEM, int OP>
__device__ __forceinline__ void consume_lds_slots(float* acc, const u32x4* mine, int meta_lane) {
  if constexpr (D < DEPTH) {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (DEPTH - 1 - D));  // vmcnt alone; the others at their maximum
    asm volatile("" ::: "memory");
    const u32x4 v = *(const volatile u32x4*)(mine + D * kWaveSize);
    accumulate<ELEM, OP>(acc, v, 1.0f, meta_lane);
    consume_lds_slots<D + 1, DEPTH, ELEM, OP>(acc, mine, meta_lane);
  }
}

template <int LPR, int ELEM, int DEPTH, int OP, bool BUF, bool NT, bool RANGE = true,
          bool PARTIAL = true, bool LDS = false>
__device__ __forceinline__ void gather_slots(float* acc, int j_lo, int j_hi,
                                             const ChunkLookups<BUF>& q, const char* tbase,
                                             __amdgpu_buffer_rsrc_t rsrc, int g, uint32_t col,
                                             bool lane_ok, int meta_lane, int gl) {
  constexpr bool WEIGHTED = OP == kOpWeighted;
  constexpr int kAux = NT ? 2 : 0;  // gfx94x/gfx950 cache-policy bits: 1 = sc0, 2 = nt, 16 = sc1
  const int k_lo = RANGE ? j_lo >> gl : 0;
  const int k_hi = (j_hi + (1 << gl) - 1) >> gl;
  if constexpr (LDS) {
    static_assert(BUF && OP == kOpSum && DEPTH <= 8, "the LDS station: buffer addressing, sum");
    extern __shared__ u32x4 emb_stage[];  // kWavesPerBlock * DEPTH slots of 64 segments
    u32x4* slots = emb_stage + (threadIdx.x >> 6) * (DEPTH * kWaveSize);
    for (int k0 = k_lo; k0 < k_hi; k0 += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        const int j = ((k0 + d) << gl) + g;
        const int src = RANGE ? (j & (kWaveSize - 1)) : j;
        const bool take = (!RANGE || (j >= j_lo && j < j_hi)) && (!PARTIAL || lane_ok);
        uint32_t vo = (uint32_t)__builtin_amdgcn_ds_bpermute(src << 2, (int)q.voff);
        if constexpr (RANGE || PARTIAL) vo = take ? vo : kBufSentinel;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc, (__attribute__((address_space(3))) void*)(slots + d * kWaveSize), 16,
            (int)(vo + col), 0, 0, kAux);
      }
      consume_lds_slots<0, DEPTH, ELEM, OP>(acc, slots + (threadIdx.x & (kWaveSize - 1)),
                                            meta_lane);
      asm volatile("" ::: "memory");  // the slots are refilled only after they have been read
    }
    return;
  }
  for (int k0 = k_lo; k0 < k_hi; k0 += DEPTH) {
    u32x4 r[DEPTH];
    float wj[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int j = ((k0 + d) << gl) + g;  // slot served by this lane's group in this step
      const int src = RANGE ? (j & (kWaveSize - 1)) : j;  // (no wrap without RANGE)
      const bool in = !RANGE || (j >= j_lo && j < j_hi);
      const bool take = in && (!PARTIAL || lane_ok);
      bool valid;  // this lane fetches a segment of a row that exists
      if constexpr (BUF) {
        uint32_t vo = (uint32_t)__builtin_amdgcn_ds_bpermute(src << 2, (int)q.voff);
        if constexpr (RANGE || PARTIAL) vo = take ? vo : kBufSentinel;
        valid = vo != kBufSentinel;
        r[d] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(vo + col), 0, kAux);
      } else {
        const int64_t ro = shfl64(q.roff, src);
        u32x4 v = {0u, 0u, 0u, 0u};
        valid = take && ro >= 0;
        if (valid) {
          const u32x4* srcp = reinterpret_cast<const u32x4*>(tbase + ro + col);
          v = NT ? __builtin_nontemporal_load(srcp) : *srcp;
        }
        r[d] = v;
      }
      if constexpr (WEIGHTED) {
        // (a slot without a lookup holds weight 0 and fetched zeros)
        const float ws = __builtin_bit_cast(
            float, __builtin_amdgcn_ds_bpermute(src << 2, __builtin_bit_cast(int, q.w)));
        wj[d] = in ? ws : 0.0f;
      } else if constexpr (OP == kOpMax) {
        wj[d] = valid ? 1.0f : 0.0f;
      } else {
        wj[d] = 1.0f;
      }
    }
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) accumulate<ELEM, OP>(acc, r[d], wj[d], meta_lane);
  }
}

// A chunk whose table has a hot head (rows [0, hot) of the table are the frequently looked-up
// ones, the outcome of the offline profiling of paper Sec. 4.3): the lookups are regrouped, hot
// ones to the low slots and the others to the high slots, each kind keeping its order, and the
// two kinds are gathered one after the other - the hot rows with the default cache policy, so
// that they stay in L2, the others non-temporally, so that they do not push hot rows out.
// `hot_mask` has bit i set if lookup i names a hot row, `n` is the number of lookups.
template <int LPR, int ELEM, int DEPTH, int OP, bool COLD_NT>
__device__ __forceinline__ void gather_hot_cold(float* acc, int n, uint64_t hot_mask,
                                                const ChunkLookups<true>& q, const char* tbase,
                                                __amdgpu_buffer_rsrc_t rsrc, int lane, int g,
                                                uint32_t col, bool lane_ok, int meta_lane,
                                                int gl) {
  const uint64_t present = n >= kWaveSize ? ~0ull : ((1ull << n) - 1ull);
  const uint64_t cold_mask = present & ~hot_mask;
  const uint64_t below = (1ull << lane) - 1ull;
  const int nh = __builtin_popcountll(hot_mask), nc = __builtin_popcountll(cold_mask);
  const bool is_hot = (hot_mask >> lane) & 1ull, is_cold = (cold_mask >> lane) & 1ull;
  // a bijection of the 64 slots: hot lookups to [0, nh), lanes without a lookup to the middle,
  // other lookups to [64 - nc, 64)
  const int dest = is_hot ? __builtin_popcountll(hot_mask & below)
                          : (is_cold ? kWaveSize - nc + __builtin_popcountll(cold_mask & below)
                                     : nh + __builtin_popcountll(~present & below));
  ChunkLookups<true> s;
  s.voff = (uint32_t)__builtin_amdgcn_ds_permute(dest << 2, (int)q.voff);
  s.roff = -1;
  s.w = q.w;
  if constexpr (OP == kOpWeighted)
    s.w = __builtin_bit_cast(float, __builtin_amdgcn_ds_permute(
                                        dest << 2, __builtin_bit_cast(int, q.w)));
  gather_slots<LPR, ELEM, DEPTH, OP, true, false>(acc, 0, nh, s, tbase, rsrc, g, col, lane_ok,
                                                  meta_lane, gl);
  gather_slots<LPR, ELEM, DEPTH, OP, true, COLD_NT>(acc, kWaveSize - nc, kWaveSize, s, tbase,
                                                    rsrc, g, col, lane_ok, meta_lane, gl);
}

// The gather of one bag (one column slab of it) by a whole wavefront: walk the bag's lookups
// [s, e) in chunks of 64 and add the rows into acc.
template <int LPR, int ELEM, int DEPTH, int OP, bool BUF, bool NT>
__device__ __forceinline__ void gather_bag(float* acc, const int64_t* __restrict__ indices,
                                           const float* __restrict__ weights, int64_t s,
                                           int64_t e, int64_t R, uint32_t row_bytes,
                                           const char* tbase, __amdgpu_buffer_rsrc_t rsrc,
                                           int lane, int g, uint32_t col, bool lane_ok,
                                           int meta_lane, int glog2) {
  // log2 of the rows per wave load: a constant for a fixed LPR, a wave-uniform value for LPR == 0
  const int gl = LPR ? __builtin_ctz((unsigned)(kWaveSize / (LPR ? LPR : 1))) : glog2;
  for (int64_t c = s; c < e; c += kWaveSize) {
    const int64_t left = e - c;
    const int n = left < kWaveSize ? (int)left : kWaveSize;  // lookups in this chunk (uniform)
    int64_t idx;
    float w;
    load_chunk<OP == kOpWeighted>(indices, weights, c, n, lane, &idx, &w);
    const ChunkLookups<BUF> q = chunk_offsets<BUF>(idx, w, R, row_bytes);
    gather_slots<LPR, ELEM, DEPTH, OP, BUF, NT>(acc, 0, n, q, tbase, rsrc, g, col, lane_ok,
                                                meta_lane, gl);
  }
}

// Which piece of work this wavefront owns: position `tpos` in the launch's table list and
// wavefront `w_in_table` of that table (0 .. wpt-1), or false if it has none.  Workgroups are
// dealt round-robin to the 8 XCDs, so blockIdx % 8 names the XCD (and its L2); the XCD-affine
// order turns that into (position, piece) as described at KParams.  `block` is the workgroup's
// index within the launch (or within its block range of a fused launch, which starts at a
// multiple of 8 so that block % 8 still names the XCD).
__device__ __forceinline__ bool decode_work(const KParams& p, uint32_t block, uint32_t wave,
                                            uint32_t* tpos, uint32_t* w_in_table) {
  if (p.xcd_bpp) {
    const uint32_t xcd = block & 7u, slot = block >> 3;
    const uint32_t ul = slot / p.xcd_bpp;
    const uint32_t unit = ul * 8u + xcd;
    const uint32_t w_in_piece = (slot - ul * p.xcd_bpp) * kWavesPerBlock + wave;
    const uint32_t w = (unit & ((1u << p.xcd_pshift) - 1u)) * p.xcd_wpp + w_in_piece;
    if (w_in_piece >= p.xcd_wpp || w >= p.wpt || unit >= p.xcd_units) return false;
    *tpos = unit >> p.xcd_pshift;
    *w_in_table = w;
    return true;
  }
  const uint64_t work64 = (uint64_t)block * kWavesPerBlock + wave;
  if (work64 >= p.num_work) return false;
  const uint32_t q = (uint32_t)work64 / p.wpt;
  *tpos = q;
  *w_in_table = (uint32_t)work64 - q * p.wpt;
  return true;
}

// The end of a bag that all 64 lanes gathered together (gather_bag): combine the G = 64/lpr row
// groups with a fixed xor butterfly (every lane ends with the same bits), add the summed biases
// of quantised rows, divide by the bag length for the mean (or, for max pooling, give 0 to a bag
// without a valid lookup), and store the lane's elements of bag row `b` at output column
// `out_col` with 16-byte non-temporal stores.
template <int LPR, int ELEM, int OP>
__device__ __forceinline__ void finish_bag(float* acc, int lpr, int lane, bool lane_ok,
                                           uint32_t col, uint32_t D_t, int64_t len, bool mean,
                                           float* __restrict__ out, int64_t out_ld, uint32_t b,
                                           int64_t out_col) {
  constexpr bool HALF = ELEM == EMB_F16 || ELEM == EMB_BF16;
  constexpr bool QUANT = IsQuant<ELEM>::value;
  constexpr bool MAXP = OP == kOpMax;
  constexpr int NOUT = OutCount<ELEM>::value;
  if constexpr (QUANT && !MAXP) {
#pragma unroll
    for (int i = 0; i < NOUT; ++i) acc[i] += acc[16];
  }
#pragma unroll
  for (int m = kWaveSize / 2; m >= 4; m >>= 1) {
    if (m >= lpr) {  // wave-uniform; a compile-time constant unless LPR == 0
#pragma unroll
      for (int i = 0; i < NOUT; ++i) {
        const float other = __shfl_xor(acc[i], m);
        acc[i] = MAXP ? __builtin_fmaxf(acc[i], other) : acc[i] + other;
      }
      if constexpr (MAXP) acc[NOUT] += __shfl_xor(acc[NOUT], m);
    }
  }
  if constexpr (MAXP) {
    const bool none = acc[NOUT] == 0.0f;  // empty bag, or no lookup named an existing row
#pragma unroll
    for (int i = 0; i < NOUT; ++i) acc[i] = none ? 0.0f : acc[i];
  } else if (mean && len > 0) {
    const float fl = (float)len;
#pragma unroll
    for (int i = 0; i < NOUT; ++i) acc[i] = acc[i] / fl;
  }
  if (lane < lpr && lane_ok) {
    // col counts bytes of the table row; the output is fp32.  A quantised row ends with 8 codes
    // and 8 bytes of scale and bias, so its last lane stores 8 elements instead of 16.
    const uint32_t elem0 = QUANT ? col : (HALF ? col / 2 : col / 4);
    f32x4* dst = reinterpret_cast<f32x4*>(out + (int64_t)b * out_ld + out_col + elem0);
#pragma unroll
    for (int q = 0; q < NOUT / 4; ++q) {
      if (!QUANT || elem0 + 4 * q < D_t) {
        const f32x4 v = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        __builtin_nontemporal_store(v, dst + q);
      }
    }
  }
}

}  // namespace embbag
