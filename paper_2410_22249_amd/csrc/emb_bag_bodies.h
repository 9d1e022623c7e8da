// The bodies of the forward kernels as device functions, so that a kernel per body
// (emb_bag_wave.hip, emb_bag_stream.hip) and a fused kernel that runs several bodies over
// consecutive block ranges of one launch (emb_bag_fused.hip) share them.  `block` is the
// workgroup's index within its launch or block range; `order_base` is where the tables of that
// range start in the table list.  Included by the kernel sources only.
#pragma once

#include "emb_bag_device.h"

namespace embbag {

// Position q of a launch's table list.  The list arrives in the kernel-argument segment; read as
// an aligned 32-bit word at a wave-uniform position it is a scalar load, not a vector one.
__device__ __forceinline__ uint32_t listed_table(const TableOrder& order, uint32_t q) {
  q = __builtin_amdgcn_readfirstlane(q);
  const uint32_t word = reinterpret_cast<const uint32_t*>(order.t)[q >> 1];
  return (word >> ((q & 1u) * 16u)) & 0xFFFFu;
}

// ---------------------------------------------------------------------------------------------
// wave body
// ---------------------------------------------------------------------------------------------

// One wavefront per (bag, column slab), or per p.bags_per_wave consecutive bags of one table when
// rows fit one slab.  LPR = lanes per row (power of two, 4..64), or 0 for tables of different
// widths: then table t is described by table_offsets[t] (its BYTE offset in the arena) and
// out_offsets[t] (its first output column; its width is the difference to the next entry), the
// lanes per row are chosen per wavefront, and rows are at most 1 KiB.
//
// The per-bag chain bounds -> row ids -> rows (paper Sec. 3.1) is taken apart across the bags of
// a wavefront: the bounds of all its bags arrive with one load (lane l holds bound l), and the
// row ids of the next bag's first chunk are requested before the rows of the current bag, so
// that they are there when the current bag has been stored (the index prefetch of Sec. 4.2,
// which is always accurate because the ids are known ahead; here it runs across bags).
//
// HOT (buffer addressing only): hot_rows[t] leading rows of table t are its hot head; lookups
// are regrouped per chunk, hot ones first (gather_hot_cold).  HOT == 1: the other rows are read
// non-temporally, and the hot head replaces the per-table hint (0 rows = a streaming table);
// HOT == 2: both kinds are read with the default policy.
// LDS (buffer addressing, sum pooling, no hot / cold split): the row loads go through the LDS
// station of gather_slots; the launch then provides kWavesPerBlock * DEPTH KiB of dynamic LDS.
template <int LPR, int ELEM, int DEPTH, int OP, bool BUF, int HOT = 0, bool LDS = false>
__device__ __forceinline__ void wave_body(
    const char* __restrict__ tables, const int64_t* __restrict__ table_offsets,
    const int64_t* __restrict__ indices, const int64_t* __restrict__ offsets,
    const float* __restrict__ weights, const uint8_t* __restrict__ table_hints,
    const int64_t* __restrict__ hot_rows, const int64_t* __restrict__ out_offsets,
    float* __restrict__ out, const KParams& p, const TableOrder& order, uint32_t order_base,
    uint32_t block) {
  static_assert(!HOT || BUF, "the hot / cold split is built for buffer addressing");
  static_assert(!LDS || (BUF && !HOT), "the LDS station is built for buffer addressing");
  constexpr bool MIXED = LPR == 0;
  constexpr bool HALF = ELEM == EMB_F16 || ELEM == EMB_BF16;  // 2-byte elements
  constexpr bool QUANT = IsQuant<ELEM>::value;                // 1-byte codes + scale, bias
  constexpr bool WEIGHTED = OP == kOpWeighted;
  constexpr int NACC = AccCount<ELEM, OP>::value;             // fp32 accumulators per lane

  const int lane = threadIdx.x & (kWaveSize - 1);
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint32_t tpos, w_in_table;
  if (!decode_work(p, block, wave, &tpos, &w_in_table)) return;
  const uint32_t t = p.listed ? listed_table(order, order_base + tpos) : tpos;
  // the wavefront's bags b0 .. b0 + nb - 1 (one bag, one slab of it, when rows span slabs)
  uint32_t b0 = w_in_table * p.bags_per_wave, slab = 0, nb = p.bags_per_wave;
  if (p.slabs > 1) {
    b0 = w_in_table / p.slabs;
    slab = w_in_table - b0 * p.slabs;
    nb = 1;
  }
  if (nb > p.B - b0) nb = p.B - b0;  // b0 < B: the grid holds ceil(B / bags_per_wave) per table

  // Everything the wavefront needs to know before it can ask for row ids is requested at once
  // and waited for once: the bag bounds (lane l holds bound l of the wavefront's bags), the
  // table's cache hint or hot-head size, and the table's geometry.
  int64_t o = 0;
  if ((uint32_t)lane <= nb) o = offsets[(uint64_t)t * p.B + b0 + (uint32_t)lane];
  int hint_raw = 0;
  int64_t hot_raw = 0;
  if constexpr (HOT) {
    hot_raw = hot_rows[t];
  } else {
    if (p.has_hints) hint_raw = table_hints[t];
  }

  // per-table geometry
  uint32_t D_t = p.D, row_bytes = p.row_bytes;
  int64_t out_col = (int64_t)t * p.D;
  int lpr = LPR ? LPR : 4;
  const char* tbase;
  int64_t R;
  if constexpr (MIXED) {
    out_col = uniform64(out_offsets[t]);
    const int64_t out_next = uniform64(out_offsets[t + 1]);
    const int64_t byte0 = uniform64(table_offsets[t]);
    int64_t bytes = uniform64(table_offsets[t + 1]) - byte0;
    const int64_t d64 = out_next - out_col;
    const int64_t rb64 = QUANT ? d64 + 8 : d64 * (HALF ? 2 : 4);
    // a malformed table description writes nothing (the host checked its own copy of the widths)
    if (d64 <= 0 || rb64 > kSlabBytes || (rb64 & 15) || out_col < 0 || (out_col & 3) ||
        out_next > p.out_ld)
      return;
    D_t = (uint32_t)d64;
    row_bytes = (uint32_t)rb64;
    while ((uint32_t)lpr * 16u < row_bytes) lpr <<= 1;
    if (bytes < 0) bytes = 0;
    if (BUF && bytes > (int64_t)kBufMaxBytes) bytes = (int64_t)kBufMaxBytes;
    R = bytes / row_bytes;
    tbase = tables + byte0;
  } else {
    const int64_t row0 = uniform64(table_offsets[t]);
    R = uniform64(table_offsets[t + 1]) - row0;
    if (R < 0) R = 0;
    if (BUF && R > p.max_rows) R = p.max_rows;
    tbase = tables + row0 * (int64_t)p.row_bytes;
  }
  const int lpr_log2 = __builtin_ctz((unsigned)lpr);
  const int gl = 6 - lpr_log2;  // log2 of the rows per load instruction

  const int g = lane >> lpr_log2;
  const uint32_t col = slab * kSlabBytes + (uint32_t)(lane & (lpr - 1)) * 16u;
  const bool lane_ok = col < row_bytes;

  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(tbase), 0, BUF ? (uint32_t)((uint64_t)R * row_bytes) : 0u, kBufWord3);

  // quantised rows: the lane of this lane's group whose segment ends with the row's scale and bias
  const int meta_lane = (lane & ~(lpr - 1)) + (int)(D_t >> 4);

  // bag bounds are clamped to [0, NL] so that no index read can leave [0, NL); a decreasing pair
  // makes an empty bag
  o = o < 0 ? 0 : (o > p.num_lookups ? p.num_lookups : o);
  const bool streaming = !HOT && (__builtin_amdgcn_readfirstlane(hint_raw) & 1);
  const int64_t hot = HOT ? uniform64(hot_raw) : 0;

  // Rows that fill their lane groups exactly (every benchmark shape) with a batch of DEPTH
  // steps inside the 64 slots of a chunk need neither of gather_slots' per-load tests.
  constexpr bool kNoWrap = LPR != 0 && DEPTH <= (LPR ? LPR : 1);
  const bool lean = row_bytes % ((uint32_t)lpr * 16u) == 0;

  // the first bag's first chunk; from then on a bag's first chunk is requested one bag ahead
  int64_t s = uniform64(o), e = uniform64(shfl64(o, 1));
  e = e < s ? s : e;
  int n = e - s < kWaveSize ? (int)(e - s) : kWaveSize;
  int64_t idx;
  float w;
  load_chunk<WEIGHTED>(indices, weights, s, n, lane, &idx, &w);
  ChunkLookups<BUF> q = chunk_offsets<BUF>(idx, w, R, row_bytes);
  uint64_t hot_mask = HOT ? __builtin_amdgcn_ballot_w64((uint64_t)idx < (uint64_t)hot &&
                                                        q.voff != kBufSentinel) : 0ull;

  for (uint32_t i = 0; i < nb; ++i) {
    // the next bag's first chunk is on its way while this bag's rows are gathered (bag i spans
    // [bound i, max(bound i + 1, bound i)): a decreasing pair makes an empty bag)
    int64_t s2 = 0, e2 = 0;
    if (i + 1 < nb) {
      s2 = uniform64(shfl64(o, (int)i + 1));
      e2 = uniform64(shfl64(o, (int)i + 2));
      e2 = e2 < s2 ? s2 : e2;
    }
    const int n2 = e2 - s2 < kWaveSize ? (int)(e2 - s2) : kWaveSize;
    int64_t idx2;
    float w2;
    load_chunk<WEIGHTED>(indices, weights, s2, n2, lane, &idx2, &w2);

    float acc[NACC];
    init_acc<ELEM, OP>(acc);
    for (int64_t c = s; c < e; c += kWaveSize) {
      if (c != s) {  // chunks after the first are requested here
        const int64_t left = e - c;
        n = left < kWaveSize ? (int)left : kWaveSize;
        load_chunk<WEIGHTED>(indices, weights, c, n, lane, &idx, &w);
        q = chunk_offsets<BUF>(idx, w, R, row_bytes);
        if constexpr (HOT)
          hot_mask = __builtin_amdgcn_ballot_w64((uint64_t)idx < (uint64_t)hot &&
                                                 q.voff != kBufSentinel);
      }
      bool gathered = false;
      if constexpr (HOT) {
        gather_hot_cold<LPR, ELEM, DEPTH, OP, HOT == 1>(acc, n, hot_mask, q, tbase, rsrc, lane, g,
                                                        col, lane_ok, meta_lane, gl);
        gathered = true;
      } else if constexpr (kNoWrap && BUF) {
        if (lean) {  // no per-load tests: see gather_slots
          if (streaming)
            gather_slots<LPR, ELEM, DEPTH, OP, true, true, false, false, LDS>(
                acc, 0, n, q, tbase, rsrc, g, col, lane_ok, meta_lane, gl);
          else
            gather_slots<LPR, ELEM, DEPTH, OP, true, false, false, false, LDS>(
                acc, 0, n, q, tbase, rsrc, g, col, lane_ok, meta_lane, gl);
          gathered = true;
        }
      }
      if (!gathered) {
        if (streaming)
          gather_slots<LPR, ELEM, DEPTH, OP, BUF, true, true, true, LDS>(
              acc, 0, n, q, tbase, rsrc, g, col, lane_ok, meta_lane, gl);
        else
          gather_slots<LPR, ELEM, DEPTH, OP, BUF, false, true, true, LDS>(
              acc, 0, n, q, tbase, rsrc, g, col, lane_ok, meta_lane, gl);
      }
    }
    // the next bag's row offsets before this bag's stores: its ids arrived ahead of the rows
    // just consumed, so nothing is waited for here, and the stores are not waited for there
    const ChunkLookups<BUF> q2 = chunk_offsets<BUF>(idx2, w2, R, row_bytes);
    uint64_t hot_mask2 = 0ull;
    if constexpr (HOT)
      hot_mask2 = __builtin_amdgcn_ballot_w64((uint64_t)idx2 < (uint64_t)hot &&
                                              q2.voff != kBufSentinel);
    finish_bag<LPR, ELEM, OP>(acc, lpr, lane, lane_ok, col, D_t, e - s, p.mean != 0, out,
                              p.out_ld, b0 + i, out_col);
    q = q2;
    hot_mask = hot_mask2;
    s = s2;
    e = e2;
    n = n2;
  }
}

// ---------------------------------------------------------------------------------------------
// stream body
// ---------------------------------------------------------------------------------------------

constexpr uint32_t kNoBag = 0xFFFFFFFFu;       // packed (end, bag) of "no further bag"
constexpr uint32_t kMaxGroupLookups = 1u << 25;  // a group's range must stay below this

__device__ __forceinline__ bool any_lane(bool c) { return __builtin_amdgcn_ballot_w64(c) != 0; }

// The stream of one wavefront.  Per lane: `glen` lookups of its group start at gi (indices) and
// gw (weights); `pk` holds, in lane r of the group, (relative end << 6 | bag number within the
// group) of the group's r-th non-empty bag, kNoBag beyond; out_rsrc covers the wavefront's
// output rows and `store0` is the byte offset of this lane's elements in its group's first bag.
template <int LPR, int ELEM, int DEPTH, int OP, bool NT, bool BUF>
__device__ __forceinline__ void stream_groups(const int64_t* __restrict__ gi,
                                              const float* __restrict__ gw, uint32_t glen,
                                              uint32_t pk, int64_t R, uint32_t row_bytes,
                                              const char* tbase, __amdgpu_buffer_rsrc_t rsrc,
                                              __amdgpu_buffer_rsrc_t out_rsrc, uint32_t store0,
                                              uint32_t out_ld_bytes, uint32_t D, bool mean,
                                              int lane, uint32_t col, bool lane_ok,
                                              int meta_lane) {
  constexpr bool WEIGHTED = OP == kOpWeighted;
  constexpr bool MAXP = OP == kOpMax;
  constexpr bool HALF = ELEM == EMB_F16 || ELEM == EMB_BF16;
  constexpr bool QUANT = IsQuant<ELEM>::value;
  constexpr int NACC = AccCount<ELEM, OP>::value;
  constexpr int NOUT = OutCount<ELEM>::value;
  constexpr int kAux = NT ? 2 : 0;  // cache-policy bits of the row loads: 2 = nt
  const int l = lane & (LPR - 1);
  const int group_base = lane & ~(LPR - 1);
  const uint32_t elem0 = QUANT ? col : (HALF ? col / 2 : col / 4);

  float acc[NACC], acc0[NACC];  // (acc0: what a bag starts from)
  init_acc<ELEM, OP>(acc0);
#pragma unroll
  for (int i = 0; i < NACC; ++i) acc[i] = acc0[i];

  // the group's current (non-empty) bag: rank among the non-empty ones, relative bounds, number
  uint32_t rank = 0, bag_start = 0;
  uint32_t cur = (uint32_t)__shfl((int)pk, group_base);
  uint32_t next_end = cur >> 6, bag_local = cur & 63u;

  int64_t idx = -1;
  float wt = 0.0f;
  if ((uint32_t)l < glen) {
    idx = __builtin_nontemporal_load(gi + l);
    if constexpr (WEIGHTED) wt = __builtin_nontemporal_load(gw + l);
  }

  for (uint32_t qbase = 0; any_lane(qbase < glen); qbase += LPR) {
    // the next chunk of indices is on its way while this chunk's rows are gathered
    int64_t idx_next = -1;
    float wt_next = 0.0f;
    const uint32_t qn = qbase + LPR + (uint32_t)l;
    if (qn < glen) {
      idx_next = __builtin_nontemporal_load(gi + qn);
      if constexpr (WEIGHTED) wt_next = __builtin_nontemporal_load(gw + qn);
    }
    // a lookup past the group's range has idx = -1: out of range like any invalid row id
    const ChunkLookups<BUF> q = chunk_offsets<BUF>(idx, wt, R, row_bytes);

#pragma unroll 1
    for (int k0 = 0; k0 < LPR; k0 += DEPTH) {
      if (k0 > 0 && !any_lane(qbase + k0 < glen)) break;
      u32x4 r[DEPTH];
      float wj[DEPTH];
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        bool row_exists;
        if constexpr (BUF) {
          uint32_t vo = (uint32_t)__shfl((int)q.voff, group_base + k0 + d);
          row_exists = vo != kBufSentinel;
          vo = lane_ok ? vo : kBufSentinel;
          r[d] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(vo + col), 0, kAux);
        } else {  // 64-bit addressing: the load is skipped where the buffer would return zeros
          const int64_t ro = shfl64(q.roff, group_base + k0 + d);
          row_exists = ro >= 0;
          u32x4 v = {0u, 0u, 0u, 0u};
          if (row_exists && lane_ok) {
            const u32x4* srcp = reinterpret_cast<const u32x4*>(tbase + ro + col);
            v = NT ? __builtin_nontemporal_load(srcp) : *srcp;
          }
          r[d] = v;
        }
        if constexpr (WEIGHTED)
          wj[d] = __shfl(wt, group_base + k0 + d);
        else if constexpr (MAXP)
          wj[d] = row_exists ? 1.0f : 0.0f;  // marks a lookup of a row that exists
        else
          wj[d] = 1.0f;
      }
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        accumulate<ELEM, OP>(acc, r[d], wj[d], meta_lane);
        const bool flush = qbase + (uint32_t)(k0 + d) + 1u == next_end;  // this lookup ends a bag
        float v[NOUT];
#pragma unroll
        for (int i = 0; i < NOUT; ++i) {
          if constexpr (MAXP)  // the last accumulator counts the bag's valid lookups
            v[i] = acc[NOUT] > 0.0f ? acc[i] : 0.0f;
          else
            v[i] = QUANT ? acc[i] + acc[16] : acc[i];
        }
        if (!MAXP && mean && any_lane(flush)) {
          const float fl = (float)(next_end - bag_start);  // > 0: the bag is not empty
#pragma unroll
          for (int i = 0; i < NOUT; ++i) v[i] = v[i] / fl;
        }
        const uint32_t so = (flush && lane_ok) ? store0 + bag_local * out_ld_bytes : kBufSentinel;
#pragma unroll
        for (int q = 0; q < NOUT / 4; ++q) {
          const bool in_row = !QUANT || elem0 + 4u * q < D;
          const u32x4 bits = {__builtin_bit_cast(uint32_t, v[4 * q]),
                              __builtin_bit_cast(uint32_t, v[4 * q + 1]),
                              __builtin_bit_cast(uint32_t, v[4 * q + 2]),
                              __builtin_bit_cast(uint32_t, v[4 * q + 3])};
          __builtin_amdgcn_raw_buffer_store_b128(bits, out_rsrc,
                                                 (int)(in_row ? so + 16u * q : kBufSentinel), 0, 2);
        }
#pragma unroll
        for (int i = 0; i < NACC; ++i) acc[i] = flush ? acc0[i] : acc[i];
        if (any_lane(flush)) {  // move the groups that stored to their next non-empty bag
          rank += flush ? 1u : 0u;
          bag_start = flush ? next_end : bag_start;
          cur = (uint32_t)__shfl((int)pk, group_base + (int)rank);
          next_end = cur >> 6;
          bag_local = cur & 63u;
        }
      }
    }
    idx = idx_next;
    wt = wt_next;
  }
}

// One wavefront per G * M consecutive bags of one table (see the head of this file).  MIXED: the launch covers tables of
// different widths that share LPR lanes per row; table t is then described by table_offsets[t]
// (its BYTE offset in the arena) and out_offsets[t] (its first output column; its width is the
// difference to the next entry), as for the wave kernel.
template <int LPR, int ELEM, int DEPTH, int OP, bool MIXED, bool BUF = true>
__device__ __forceinline__ void stream_body(
    const char* __restrict__ tables, const int64_t* __restrict__ table_offsets,
    const int64_t* __restrict__ indices, const int64_t* __restrict__ offsets,
    const float* __restrict__ weights, const uint8_t* __restrict__ table_hints,
    const int64_t* __restrict__ /*hot_rows*/, const int64_t* __restrict__ out_offsets,
    float* __restrict__ out, const KParams& p, const TableOrder& order, uint32_t order_base,
    uint32_t block) {
  constexpr int G = kWaveSize / LPR;
  constexpr int GL = __builtin_ctz((unsigned)G);
  constexpr bool HALF = ELEM == EMB_F16 || ELEM == EMB_BF16;
  constexpr bool QUANT = IsQuant<ELEM>::value;
  constexpr bool WEIGHTED = OP == kOpWeighted;
  constexpr int NACC = AccCount<ELEM, OP>::value;
  constexpr int NOUT = OutCount<ELEM>::value;

  const int lane = threadIdx.x & (kWaveSize - 1);
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint32_t tpos, w_in_table;
  if (!decode_work(p, block, wave, &tpos, &w_in_table)) return;
  const uint32_t t = p.listed ? listed_table(order, order_base + tpos) : tpos;
  const uint32_t M = p.bags_per_group;                   // 1 .. LPR - 1
  const uint32_t b0 = w_in_table * (uint32_t)G * M;      // first bag of the wavefront, < B
  const uint32_t nbw = p.B - b0 < (uint32_t)G * M ? p.B - b0 : (uint32_t)G * M;  // its bags

  const int g = lane >> __builtin_ctz((unsigned)LPR);
  const int l = lane & (LPR - 1);
  const int group_base = lane & ~(LPR - 1);
  const uint32_t gb0 = (uint32_t)g * M;                            // group's first bag, wave-relative
  const uint32_t m = gb0 < nbw ? (nbw - gb0 < M ? nbw - gb0 : M) : 0u;  // group's bags

  // table geometry
  uint32_t D_t = p.D, row_bytes = p.row_bytes;
  int64_t out_col = (int64_t)t * p.D;
  const char* tbase;
  int64_t R;
  if constexpr (MIXED) {
    out_col = uniform64(out_offsets[t]);
    const int64_t out_next = uniform64(out_offsets[t + 1]);
    const int64_t d64 = out_next - out_col;
    const int64_t rb64 = QUANT ? d64 + 8 : d64 * (HALF ? 2 : 4);
    // a table description that does not fit this launch writes nothing (the host chose LPR from
    // its own copy of the widths)
    if (d64 <= 0 || rb64 > (int64_t)LPR * 16 || (rb64 & 15) || out_col < 0 || (out_col & 3) ||
        out_next > p.out_ld)
      return;
    D_t = (uint32_t)d64;
    row_bytes = (uint32_t)rb64;
    const int64_t byte0 = uniform64(table_offsets[t]);
    int64_t bytes = uniform64(table_offsets[t + 1]) - byte0;
    if (bytes < 0) bytes = 0;
    if (BUF && bytes > (int64_t)kBufMaxBytes) bytes = (int64_t)kBufMaxBytes;
    R = bytes / row_bytes;
    tbase = tables + byte0;
  } else {
    const int64_t row0 = uniform64(table_offsets[t]);
    R = uniform64(table_offsets[t + 1]) - row0;
    if (R < 0) R = 0;
    if (BUF && R > p.max_rows) R = p.max_rows;
    tbase = tables + row0 * (int64_t)row_bytes;
  }
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(tbase), 0, BUF ? (uint32_t)((uint64_t)R * row_bytes) : 0u, kBufWord3);
  const uint32_t col = (uint32_t)l * 16u;
  const bool lane_ok = col < row_bytes;
  const int meta_lane = group_base + (int)(D_t >> 4);
  const bool streaming = p.has_hints && (__builtin_amdgcn_readfirstlane((int)table_hints[t]) & 1);

  // bag bounds: lane l of a group holds bound min(l, m) of the group, clamped to [0, NL]
  const int64_t* obase = offsets + (uint64_t)t * p.B + b0;
  int64_t o = 0;
  if (m > 0) {
    o = obase[gb0 + ((uint32_t)l < m ? (uint32_t)l : m)];
    o = o < 0 ? 0 : (o > p.num_lookups ? p.num_lookups : o);
  }
  const int64_t o_next = shfl64(o, lane + 1 < kWaveSize ? lane + 1 : lane);
  const bool mine = (uint32_t)l < m;                     // this lane stands for bag l of its group
  const int64_t len = mine ? o_next - o : 0;
  const int64_t S = shfl64(o, group_base);               // the group's first lookup
  const int64_t E = shfl64(o, group_base + (int)m);      // one past its last
  const bool malformed = (mine && len < 0) || E - S >= (int64_t)kMaxGroupLookups;

  if (any_lane(malformed)) {
    // bag by bag with the whole wavefront, exactly as the wave kernel treats a bag
    for (uint32_t i = 0; i < nbw; ++i) {
      int64_t s = uniform64(obase[i]);
      int64_t e = uniform64(obase[i + 1]);
      s = s < 0 ? 0 : (s > p.num_lookups ? p.num_lookups : s);
      e = e < s ? s : (e > p.num_lookups ? p.num_lookups : e);
      float acc[NACC];
      init_acc<ELEM, OP>(acc);
      gather_bag<LPR, ELEM, 2, OP, BUF, false>(acc, indices, weights, s, e, R, row_bytes, tbase,
                                               rsrc, lane, g, col, lane_ok, meta_lane, GL);
      finish_bag<LPR, ELEM, OP>(acc, LPR, lane, lane_ok, col, D_t, e - s, p.mean != 0, out,
                                p.out_ld, b0 + i, out_col);
    }
    return;
  }

  // output rows of this wavefront as a buffer: a store with an out-of-range offset is dropped
  const uint32_t out_ld_bytes = (uint32_t)p.out_ld * 4u;
  float* obuf = out + (int64_t)b0 * p.out_ld + out_col;
  const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      obuf, 0, (nbw - 1u) * out_ld_bytes + D_t * 4u, kBufWord3);
  const uint32_t elem0 = QUANT ? col : (HALF ? col / 2 : col / 4);
  const uint32_t store0 = gb0 * out_ld_bytes + elem0 * 4u;

  // empty bags get zeros now: the stream only ever stores bags that end at a lookup
  const bool empty = mine && len == 0;
  if (any_lane(empty)) {
    for (uint32_t i = 0; i < M; ++i) {
      const bool e_i = __shfl((int)empty, group_base + (int)i) != 0;
      const uint32_t so = (e_i && lane_ok) ? store0 + i * out_ld_bytes : kBufSentinel;
      const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int q = 0; q < NOUT / 4; ++q) {
        const bool in_row = !QUANT || elem0 + 4u * q < D_t;
        __builtin_amdgcn_raw_buffer_store_b128(zero, out_rsrc,
                                               (int)(in_row ? so + 16u * q : kBufSentinel), 0, 2);
      }
    }
  }

  // Lane r of a group gets (relative end << 6 | bag) of the group's r-th non-empty bag: a stable
  // partition of the group's lanes, non-empty bags first, sent with one forward permute.
  const uint64_t ballot = __builtin_amdgcn_ballot_w64(mine && len > 0);
  const uint64_t gmask = LPR == 64 ? ballot : (ballot >> group_base) & ((1ull << (LPR & 63)) - 1ull);
  const uint32_t before = (uint32_t)__builtin_popcountll(gmask & ((1ull << l) - 1ull));
  const uint32_t total = (uint32_t)__builtin_popcountll(gmask);
  const bool nonempty = mine && len > 0;
  const uint32_t dest = nonempty ? before : total + ((uint32_t)l - before);
  const uint32_t send = nonempty ? ((uint32_t)(o_next - S) << 6) | (uint32_t)l : kNoBag;
  const uint32_t pk =
      (uint32_t)__builtin_amdgcn_ds_permute((group_base + (int)dest) << 2, (int)send);

  const uint32_t glen = (uint32_t)(E - S);
  const int64_t* gi = indices + S;
  const float* gw = WEIGHTED ? weights + S : nullptr;
  if (streaming)
    stream_groups<LPR, ELEM, DEPTH, OP, true, BUF>(gi, gw, glen, pk, R, row_bytes, tbase, rsrc,
                                                   out_rsrc, store0, out_ld_bytes, D_t,
                                                   p.mean != 0, lane, col, lane_ok, meta_lane);
  else
    stream_groups<LPR, ELEM, DEPTH, OP, false, BUF>(gi, gw, glen, pk, R, row_bytes, tbase, rsrc,
                                                    out_rsrc, store0, out_ld_bytes, D_t,
                                                    p.mean != 0, lane, col, lane_ok, meta_lane);
}

}  // namespace embbag
