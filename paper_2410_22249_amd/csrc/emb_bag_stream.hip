// EmbeddingBag forward for SHORT bags on MI355X (gfx950): the stream kernel.
//
// With one wavefront per bag, a bag of a few lookups is a chain of three dependent memory round
// trips (bag bounds -> indices -> rows) with little to overlap inside the wavefront: the
// latency-bound regime of the paper (Sec. 3.1), which it attacks by prefetching further ahead
// (Sec. 4.2).  Here the prefetch runs across bag boundaries:
//   * a wavefront owns G * M consecutive bags of one table, G = 64/LPR lane groups with M
//     consecutive bags each.  Consecutive bags are consecutive in `indices`, so a group's lookups
//     are ONE contiguous range, which the group streams without regard to where its bags end;
//   * the M + 1 bag bounds of a group are fetched with one load (lane l holds bound l), the
//     indices LPR at a time with one coalesced load per group, the next chunk of indices is
//     requested before the rows of the current chunk, and DEPTH row loads per group (G * DEPTH
//     per wavefront) are in flight; every load instruction fetches one row for each group;
//   * a group adds rows into its accumulator and, at the lookup that ends a bag, stores the
//     accumulator to that bag's output and clears it.  The store is a buffer store whose offset
//     is out of range for lanes that have nothing to store, so the row pipeline has no branches
//     around memory instructions;
//   * rows are read through the table's buffer resource, or - tables that are beyond a
//     buffer's reach or have no size bound - with 64-bit addresses, the load skipped where the
//     range check would have returned zeros; sum, mean, weighted sum and max pooling;
//   * empty bags are zero-filled before the stream starts; a wavefront whose bag bounds are not
//     monotone (malformed input) or whose group covers 2^25 lookups or more handles its bags one
//     after the other with the whole wavefront instead, with the semantics of the wave kernel.
// A bag is summed by one group in the order of its lookups (the wave kernel keeps G partial sums
// and combines them at the end), so the two kernels agree to rounding, not to the bit, while
// this kernel's result does not depend on G, M or DEPTH.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/emb_bag.h"
#include "emb_bag_device.h"
#include "emb_bag_bodies.h"

// Compiled once per lanes-per-row class (-DEMB_LPR=4, 8, 16, 32, 64) so that the classes build
// side by side; each build exports pick_stream_kernel_lpr<EMB_LPR>.
#ifndef EMB_LPR
#error "compile with -DEMB_LPR=<lanes per row: 4, 8, 16, 32 or 64>"
#endif

namespace {

using namespace embbag;

// The kernel proper is embbag::stream_body (emb_bag_bodies.h), shared with the fused launch.
template <int LPR, int ELEM, int DEPTH, int OP, bool MIXED, bool BUF>
__global__ void __launch_bounds__(kBlock)
emb_bag_stream_kernel(const char* __restrict__ tables, const int64_t* __restrict__ table_offsets,
                      const int64_t* __restrict__ indices, const int64_t* __restrict__ offsets,
                      const float* __restrict__ weights, const uint8_t* __restrict__ table_hints,
                      const int64_t* __restrict__ hot_rows,
                      const int64_t* __restrict__ out_offsets, float* __restrict__ out,
                      KParams p, TableOrder order) {
  stream_body<LPR, ELEM, DEPTH, OP, MIXED, BUF>(tables, table_offsets, indices, offsets, weights,
                                           table_hints, hot_rows, out_offsets, out, p, order, 0u,
                                           blockIdx.x);
}

// rows through a buffer resource, or with 64-bit addresses
template <int LPR, int ELEM, int DEPTH, int OP, bool MIXED>
KernelFn pick_addr(bool buf) {
  return buf ? emb_bag_stream_kernel<LPR, ELEM, DEPTH, OP, MIXED, true>
             : emb_bag_stream_kernel<LPR, ELEM, DEPTH, OP, MIXED, false>;
}

template <int LPR, int ELEM, int DEPTH, bool MIXED>
KernelFn pick_op(int op, bool buf) {
  switch (op) {
    case kOpSum: return pick_addr<LPR, ELEM, DEPTH, kOpSum, MIXED>(buf);
    case kOpWeighted: return pick_addr<LPR, ELEM, DEPTH, kOpWeighted, MIXED>(buf);
    case kOpMax: return pick_addr<LPR, ELEM, DEPTH, kOpMax, MIXED>(buf);
    default: return nullptr;
  }
}

template <int LPR, int ELEM, bool MIXED>
KernelFn pick_d(int depth, int op, bool buf) {
  constexpr int D8 = LPR >= 8 ? 8 : 4;  // a group holds LPR lookups per chunk: DEPTH <= LPR
  return depth <= 4 ? pick_op<LPR, ELEM, 4, MIXED>(op, buf) : pick_op<LPR, ELEM, D8, MIXED>(op, buf);
}

template <int LPR, bool MIXED>
KernelFn pick_e(int elem, int depth, int op, bool buf) {
  switch (elem) {
    case EMB_F32: return pick_d<LPR, EMB_F32, MIXED>(depth, op, buf);
    case EMB_F16: return pick_d<LPR, EMB_F16, MIXED>(depth, op, buf);
    case EMB_BF16: return pick_d<LPR, EMB_BF16, MIXED>(depth, op, buf);
    case EMB_U8ROW: return pick_d<LPR, EMB_U8ROW, MIXED>(depth, op, buf);
    case EMB_FP8ROW: return pick_d<LPR, EMB_FP8ROW, MIXED>(depth, op, buf);
    default: return nullptr;
  }
}

}  // namespace

namespace embbag {

KernelFn EMB_PASTE(pick_stream_kernel_lpr, EMB_LPR)(int elem, int depth, int op, bool mixed,
                                                     bool buf) {
  return mixed ? pick_e<EMB_LPR, true>(elem, depth, op, buf)
               : pick_e<EMB_LPR, false>(elem, depth, op, buf);
}

}  // namespace embbag
