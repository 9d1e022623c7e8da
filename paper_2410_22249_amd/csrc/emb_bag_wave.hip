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
//     memory-level parallelism (the multithreading fix of Sec. 3.3); a variant lets the loads
//     land in LDS instead (the shared-memory station of Sec. 4.2; opt-in, never faster here);
//   * a wavefront may own several consecutive bags of a table: their bounds arrive with one
//     load and the next bag's row ids are requested before the current bag's rows, so the
//     offsets -> indices -> rows chain of Sec. 3.1 is paid once per wavefront, not per bag;
//   * tables laid out with their most frequently used rows first (the offline hot-index
//     profiling of Sec. 4.3) can have a bag's lookups regrouped hot rows first, the hot head
//     read with the default cache policy and the rest non-temporally (opt-in);
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
#include "emb_bag_bodies.h"

#ifndef EMB_LPR
#error "compile with -DEMB_LPR=<lanes per row: 0, 4, 8, 16, 32 or 64>"
#endif

namespace {

using namespace embbag;

// The kernel proper is embbag::wave_body (emb_bag_bodies.h), shared with the fused launch.
template <int LPR, int ELEM, int DEPTH, int OP, bool BUF, int HOT, bool LDS = false>
__global__ void __launch_bounds__(kBlock)
emb_bag_wave_kernel(const char* __restrict__ tables, const int64_t* __restrict__ table_offsets,
                    const int64_t* __restrict__ indices, const int64_t* __restrict__ offsets,
                    const float* __restrict__ weights, const uint8_t* __restrict__ table_hints,
                    const int64_t* __restrict__ hot_rows,
                    const int64_t* __restrict__ out_offsets, float* __restrict__ out, KParams p,
                    TableOrder order) {
  wave_body<LPR, ELEM, DEPTH, OP, BUF, HOT, LDS>(tables, table_offsets, indices, offsets,
                                                 weights, table_hints, hot_rows, out_offsets, out,
                                                 p, order, 0u, blockIdx.x);
}

// buffer or 64-bit addressing.  `variant` selects among the kernels built for buffer addressing,
// tables of one width and depths 4 and 8: kVariantHotNt / kVariantHot = the hot / cold split
// (tables with a hot head), kVariantLds = row loads through the LDS station (sum pooling).
template <int LPR, int ELEM, int DEPTH, int OP>
KernelFn pick_addr(bool buf, int variant) {
  if (variant != kVariantPlain) {
    if constexpr (LPR != 0 && (DEPTH == 4 || DEPTH == 8)) {
      if (!buf) return nullptr;
      if (variant == kVariantLds) {
        if constexpr (OP == kOpSum)
          return emb_bag_wave_kernel<LPR, ELEM, DEPTH, OP, true, 0, true>;
        else
          return nullptr;
      }
      return variant == kVariantHotNt ? emb_bag_wave_kernel<LPR, ELEM, DEPTH, OP, true, 1>
                                      : emb_bag_wave_kernel<LPR, ELEM, DEPTH, OP, true, 2>;
    } else {
      return nullptr;
    }
  }
  return buf ? emb_bag_wave_kernel<LPR, ELEM, DEPTH, OP, true, 0>
             : emb_bag_wave_kernel<LPR, ELEM, DEPTH, OP, false, 0>;
}

template <int LPR, int ELEM, int DEPTH>
KernelFn pick_op(int op, bool buf, int hot) {
  if (op == kOpWeighted) return pick_addr<LPR, ELEM, DEPTH, kOpWeighted>(buf, hot);
  if (op == kOpMax) {
    if constexpr (DEPTH == 4 || DEPTH == 8)  // max pooling: two depths are enough
      return pick_addr<LPR, ELEM, DEPTH, kOpMax>(buf, hot);
    else
      return nullptr;
  }
  return pick_addr<LPR, ELEM, DEPTH, kOpSum>(buf, hot);
}

template <int LPR, int ELEM>
KernelFn pick_depth(int depth, int op, bool buf, int hot) {
  if (LPR == 0 || op == kOpMax)  // tables of different widths, max pooling: depth 4 or 8
    return depth <= 4 ? pick_op<LPR, ELEM, 4>(op, buf, hot) : pick_op<LPR, ELEM, 8>(op, buf, hot);
  if constexpr (LPR != 0) {
    switch (depth) {
      case 1: return pick_op<LPR, ELEM, 1>(op, buf, hot);
      case 2: return pick_op<LPR, ELEM, 2>(op, buf, hot);
      case 4: return pick_op<LPR, ELEM, 4>(op, buf, hot);
      case 8: return pick_op<LPR, ELEM, 8>(op, buf, hot);
      case 16: return pick_op<LPR, ELEM, 16>(op, buf, hot);
      default: return nullptr;
    }
  }
  return nullptr;
}

template <int LPR>
KernelFn pick_dtype(int elem, int depth, int op, bool buf, int hot) {
  switch (elem) {
    case EMB_F32: return pick_depth<LPR, EMB_F32>(depth, op, buf, hot);
    case EMB_F16: return pick_depth<LPR, EMB_F16>(depth, op, buf, hot);
    case EMB_BF16: return pick_depth<LPR, EMB_BF16>(depth, op, buf, hot);
    case EMB_U8ROW: return pick_depth<LPR, EMB_U8ROW>(depth, op, buf, hot);
    case EMB_FP8ROW: return pick_depth<LPR, EMB_FP8ROW>(depth, op, buf, hot);
    default: return nullptr;
  }
}

}  // namespace

namespace embbag {

// nullptr if there is no such instantiation
KernelFn EMB_PASTE(pick_wave_kernel_lpr, EMB_LPR)(int elem, int depth, int op, bool buf,
                                                  int hot) {
  return pick_dtype<EMB_LPR>(elem, depth, op, buf, hot);
}

}  // namespace embbag
