// EmbeddingBag forward for tables of different widths whose call would otherwise split into
// several launches (one stream-kernel launch per lanes-per-row class with short bags, one
// wave-kernel launch for the other tables): the fused kernel.
//
// Launches on one HIP stream run one after the other, each with its own ramp and drain; at the
// batch sizes of inference (the paper's 2048 samples, Sec. 5) a launch of one row class lasts a
// few microseconds and four to six of them in a row cost several times the work they hold.  The
// launches of such a call touch disjoint tables and disjoint output columns, so nothing orders
// them: here they are consecutive ranges of the workgroups of ONE launch, each range running the
// body it would have run as a launch of its own (emb_bag_bodies.h), with the parameters and the
// table list of that launch.  Results are bit-identical to the separate launches.
//
// Compiled once per element type (-DEMB_ELEM=0 .. 4); each build exports
// pick_fused_kernel_elem<EMB_ELEM>.  Sum and mean pooling with buffer addressing only (what
// the stream body supports); a call with max pooling or 64-bit addressing never splits.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/emb_bag.h"
#include "emb_bag_device.h"
#include "emb_bag_bodies.h"

#ifndef EMB_ELEM
#error "compile with -DEMB_ELEM=<element type: 0 .. 4>"
#endif

namespace {

using namespace embbag;

// DEPTH (4 or 8) is the row loads in flight of the wave body and of the stream bodies with 8 or
// more lanes per row; with 4 lanes per row a group holds 4 lookups per chunk, hence depth 4.
template <int ELEM, int DEPTH, bool WEIGHTED>
__global__ void __launch_bounds__(kBlock)
emb_bag_fused_kernel(const char* __restrict__ tables, const int64_t* __restrict__ table_offsets,
                     const int64_t* __restrict__ indices, const int64_t* __restrict__ offsets,
                     const float* __restrict__ weights, const uint8_t* __restrict__ table_hints,
                     const int64_t* __restrict__ hot_rows,
                     const int64_t* __restrict__ out_offsets, float* __restrict__ out,
                     FusedParams f, TableOrder order) {
  constexpr int OP = WEIGHTED ? kOpWeighted : kOpSum;
  const uint32_t blk = blockIdx.x;
#define EMB_ARGS tables, table_offsets, indices, offsets, weights, table_hints, hot_rows, out_offsets, out
  if (blk < f.end_block[0])
    wave_body<0, ELEM, DEPTH, OP, true>(EMB_ARGS, f.seg[0], order, f.order_base[0], blk);
  else if (blk < f.end_block[1])
    stream_body<4, ELEM, 4, OP, true>(EMB_ARGS, f.seg[1], order, f.order_base[1],
                                            blk - f.end_block[0]);
  else if (blk < f.end_block[2])
    stream_body<8, ELEM, DEPTH, OP, true>(EMB_ARGS, f.seg[2], order, f.order_base[2],
                                                blk - f.end_block[1]);
  else if (blk < f.end_block[3])
    stream_body<16, ELEM, DEPTH, OP, true>(EMB_ARGS, f.seg[3], order, f.order_base[3],
                                                 blk - f.end_block[2]);
  else if (blk < f.end_block[4])
    stream_body<32, ELEM, DEPTH, OP, true>(EMB_ARGS, f.seg[4], order, f.order_base[4],
                                                 blk - f.end_block[3]);
  else if (blk < f.end_block[5])
    stream_body<64, ELEM, DEPTH, OP, true>(EMB_ARGS, f.seg[5], order, f.order_base[5],
                                                 blk - f.end_block[4]);
#undef EMB_ARGS
}

}  // namespace

namespace embbag {

FusedFn EMB_PASTE(pick_fused_kernel_elem, EMB_ELEM)(int depth, bool weighted) {
  if (depth <= 4)
    return weighted ? emb_bag_fused_kernel<EMB_ELEM, 4, true>
                    : emb_bag_fused_kernel<EMB_ELEM, 4, false>;
  return weighted ? emb_bag_fused_kernel<EMB_ELEM, 8, true>
                  : emb_bag_fused_kernel<EMB_ELEM, 8, false>;
}

}  // namespace embbag
