// EmbeddingBag forward for MI355X (gfx950): the wave kernel, one wavefront per bag (per 1-KiB
// column slab of it).
//
// What is computed is the embedding stage of the paper (Sec. 3.1, Algorithm 1): per bag (t, b)
// follow offsets -> indices -> table rows, add the rows, store one vector of length D.
//
// How it is mapped to the machine (this is not the paper's A100 kernel, which gives one CUDA
// thread to one output element and walks the bag with dependent loads, Sec. 3.1):
//   * one 64-lane wavefront owns one bag (or one 1-KiB column slab of it when rows are longer
//     than 1 KiB); all tables of the batch share one launch;
//   * a row is read as 16-byte lane segments, so one load instruction of the wavefront moves
//     1 KiB: G = 64/LPR different rows of the same bag at once, LPR lanes per row
//     (512-byte rows: 2 rows per instruction, 256-byte rows: 4);
//   * the bag's indices are contiguous: the wavefront fetches up to 64 of them with one
//     coalesced load (lane i holds lookup i), turns them into row byte offsets once, and hands
//     offset j to the lanes that need it with a cross-lane permute - no dependent index load
//     in front of every row load as in the paper's base kernel;
//   * DEPTH row loads are issued back to back before the first is consumed (the register
//     prefetch of Sec. 4.2, with the distance as a tuning knob, Sec. 7 step vi), and the many
//     resident wavefronts per SIMD (the kernels need few VGPRs) supply the rest of the
//     memory-level parallelism (the multithreading fix of Sec. 3.3);
//   * rows are addressed through a per-table buffer resource with 32-bit offsets when the table
//     is below 3.5 GiB: the hardware range check turns an invalid row into zeros instead of a
//     fault, and address arithmetic stays 32-bit.  Larger tables use 64-bit global addressing
//     with an explicit check;
//   * a table that the caller marks as streaming (rows not re-used within a batch; the outcome of
//     the access-pattern profiling the paper does offline, Sec. 4.3 and Sec. 7) has its rows read
//     with the non-temporal policy, a re-used table with the default policy;
//   * rows may be fp32, fp16, bf16 (widened exactly) or row-wise quantised 8-bit codes;
//   * partial sums of the G row groups are combined with a fixed xor butterfly (deterministic),
//     the mean is one division per element per bag, and the result leaves with 16-byte
//     non-temporal stores so that it does not displace table rows in L2 / MALL.
// No MFMA: this is a gather-reduce, not a contraction; the bound is HBM bandwidth.
//
// This file is compiled once per lanes-per-row class (-DEMB_LPR=0, 4, 8, 16, 32, 64; 0 = tables
// of different widths, lanes per row chosen per wavefront) so that the classes build side by
// side; each build exports pick_wave_kernel_lpr<EMB_LPR>.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/emb_bag.h"
#include "emb_bag_device.h"

#ifndef EMB_LPR
#error "compile with -DEMB_LPR=<lanes per row: 0, 4, 8, 16, 32 or 64>"
#endif

namespace {

using namespace embbag;

// One wavefront per (bag, column slab).  LPR = lanes per row (power of two, 4..64), or 0 for
// tables of different widths: then table t is described by table_offsets[t] (its BYTE offset in
// the arena) and out_offsets[t] (its first output column; its width is the difference to the next
// entry), the lanes per row are chosen per wavefront, and rows are at most 1 KiB.
template <int LPR, int ELEM, int DEPTH, int OP, bool BUF>
__global__ void __launch_bounds__(kBlock)
emb_bag_wave_kernel(const char* __restrict__ tables, const int64_t* __restrict__ table_offsets,
                    const int64_t* __restrict__ indices, const int64_t* __restrict__ offsets,
                    const float* __restrict__ weights, const uint8_t* __restrict__ table_hints,
                    const int64_t* __restrict__ out_offsets, float* __restrict__ out, KParams p,
                    TableOrder order) {
  constexpr bool MIXED = LPR == 0;
  constexpr bool HALF = ELEM == EMB_F16 || ELEM == EMB_BF16;  // 2-byte elements
  constexpr bool QUANT = IsQuant<ELEM>::value;                // 1-byte codes + scale, bias
  constexpr int NACC = AccCount<ELEM, OP>::value;             // fp32 accumulators per lane

  const int lane = threadIdx.x & (kWaveSize - 1);
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint32_t tpos, w_in_table;
  if (!decode_work(p, wave, &tpos, &w_in_table)) return;
  const uint32_t t = p.listed ? order.t[tpos] : tpos;
  uint32_t b = w_in_table, slab = 0;
  if (p.slabs > 1) {
    b = w_in_table / p.slabs;
    slab = w_in_table - b * p.slabs;
  }
  const uint32_t bag = t * p.B + b;

  // bag bounds, clamped so that no index read can leave [0, NL)
  int64_t s = uniform64(offsets[bag]);
  int64_t e = uniform64(offsets[bag + 1]);
  s = s < 0 ? 0 : (s > p.num_lookups ? p.num_lookups : s);
  e = e < s ? s : (e > p.num_lookups ? p.num_lookups : e);

  // per-table geometry
  uint32_t D_t = p.D, row_bytes = p.row_bytes;
  int64_t out_col = (int64_t)t * p.D;
  int lpr = LPR ? LPR : 4;
  const char* tbase;
  int64_t R;
  if constexpr (MIXED) {
    out_col = uniform64(out_offsets[t]);
    const int64_t out_next = uniform64(out_offsets[t + 1]);
    const int64_t d64 = out_next - out_col;
    const int64_t rb64 = QUANT ? d64 + 8 : d64 * (HALF ? 2 : 4);
    // a malformed table description writes nothing (the host checked its own copy of the widths)
    if (d64 <= 0 || rb64 > kSlabBytes || (rb64 & 15) || out_col < 0 || (out_col & 3) ||
        out_next > p.out_ld)
      return;
    D_t = (uint32_t)d64;
    row_bytes = (uint32_t)rb64;
    while ((uint32_t)lpr * 16u < row_bytes) lpr <<= 1;
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
    tbase = tables + row0 * (int64_t)p.row_bytes;
  }
  const int lpr_log2 = __builtin_ctz((unsigned)lpr);

  const int g = lane >> lpr_log2;
  const uint32_t col = slab * kSlabBytes + (uint32_t)(lane & (lpr - 1)) * 16u;
  const bool lane_ok = col < row_bytes;

  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(tbase), 0, BUF ? (uint32_t)((uint64_t)R * row_bytes) : 0u, kBufWord3);

  float acc[NACC];
  init_acc<ELEM, OP>(acc);
  // quantised rows: the lane of this lane's group whose segment ends with the row's scale and bias
  const int meta_lane = (lane & ~(lpr - 1)) + (int)(D_t >> 4);

  const bool streaming = p.has_hints && (__builtin_amdgcn_readfirstlane((int)table_hints[t]) & 1);
  if (streaming)
    gather_bag<LPR, ELEM, DEPTH, OP, BUF, true>(acc, indices, weights, s, e, R, row_bytes,
                                                     tbase, rsrc, lane, g, col, lane_ok,
                                                     meta_lane, 6 - lpr_log2);
  else
    gather_bag<LPR, ELEM, DEPTH, OP, BUF, false>(acc, indices, weights, s, e, R, row_bytes,
                                                      tbase, rsrc, lane, g, col, lane_ok,
                                                      meta_lane, 6 - lpr_log2);

  finish_bag<LPR, ELEM, OP>(acc, lpr, lane, lane_ok, col, D_t, e - s, p.mean != 0, out, p.out_ld, b,
                        out_col);
}

template <int LPR, int ELEM, int DEPTH>
KernelFn pick_op(int op, bool buf) {
  if (op == kOpWeighted)
    return buf ? emb_bag_wave_kernel<LPR, ELEM, DEPTH, kOpWeighted, true>
               : emb_bag_wave_kernel<LPR, ELEM, DEPTH, kOpWeighted, false>;
  if (op == kOpMax) {
    if constexpr (DEPTH == 4 || DEPTH == 8)  // max pooling: two depths are enough
      return buf ? emb_bag_wave_kernel<LPR, ELEM, DEPTH, kOpMax, true>
                 : emb_bag_wave_kernel<LPR, ELEM, DEPTH, kOpMax, false>;
    else
      return nullptr;
  }
  return buf ? emb_bag_wave_kernel<LPR, ELEM, DEPTH, kOpSum, true>
             : emb_bag_wave_kernel<LPR, ELEM, DEPTH, kOpSum, false>;
}

template <int LPR, int ELEM>
KernelFn pick_depth(int depth, int op, bool buf) {
  if (LPR == 0 || op == kOpMax)  // tables of different widths, max pooling: depth 4 or 8
    return depth <= 4 ? pick_op<LPR, ELEM, 4>(op, buf) : pick_op<LPR, ELEM, 8>(op, buf);
  if constexpr (LPR != 0) {
    switch (depth) {
      case 1: return pick_op<LPR, ELEM, 1>(op, buf);
      case 2: return pick_op<LPR, ELEM, 2>(op, buf);
      case 4: return pick_op<LPR, ELEM, 4>(op, buf);
      case 8: return pick_op<LPR, ELEM, 8>(op, buf);
      case 16: return pick_op<LPR, ELEM, 16>(op, buf);
      default: return nullptr;
    }
  }
  return nullptr;
}

template <int LPR>
KernelFn pick_dtype(int elem, int depth, int op, bool buf) {
  switch (elem) {
    case EMB_F32: return pick_depth<LPR, EMB_F32>(depth, op, buf);
    case EMB_F16: return pick_depth<LPR, EMB_F16>(depth, op, buf);
    case EMB_BF16: return pick_depth<LPR, EMB_BF16>(depth, op, buf);
    case EMB_U8ROW: return pick_depth<LPR, EMB_U8ROW>(depth, op, buf);
    case EMB_FP8ROW: return pick_depth<LPR, EMB_FP8ROW>(depth, op, buf);
    default: return nullptr;
  }
}

}  // namespace

namespace embbag {

KernelFn EMB_PASTE(pick_wave_kernel_lpr, EMB_LPR)(int elem, int depth, int op, bool buf) {
  return pick_dtype<EMB_LPR>(elem, depth, op, buf);
}

}  // namespace embbag
