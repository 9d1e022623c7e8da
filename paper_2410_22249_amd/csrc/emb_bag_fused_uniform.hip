// EmbeddingBag forward for tables of ONE width whose call desc->table_avg_len splits in two
// (short-bag tables to the stream body, the others to the wave body): both as consecutive
// workgroup ranges of one launch, for the reason given in emb_bag_fused.hip - at inference batch
// sizes two launches in a row cost more in ramp and drain than the work they hold.  Results are
// bit-identical to the two separate launches.
//
// Compiled once per lanes-per-row class (-DEMB_LPR=4 .. 64, rows of at most 1 KiB); each build
// exports pick_fused_uniform_kernel_lpr<EMB_LPR>.  Sum and mean pooling, buffer addressing, wave
// depth 4 or 8 (other depths keep the two launches).

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/emb_bag.h"
#include "emb_bag_device.h"
#include "emb_bag_bodies.h"

#ifndef EMB_LPR
#error "compile with -DEMB_LPR=<lanes per row: 4, 8, 16, 32 or 64>"
#endif

namespace {

using namespace embbag;

template <int LPR, int ELEM, int DEPTH, bool WEIGHTED>
__global__ void __launch_bounds__(kBlock)
emb_bag_fused_uniform_kernel(const char* __restrict__ tables,
                             const int64_t* __restrict__ table_offsets,
                             const int64_t* __restrict__ indices,
                             const int64_t* __restrict__ offsets,
                             const float* __restrict__ weights,
                             const uint8_t* __restrict__ table_hints,
                             const int64_t* __restrict__ hot_rows,
                             const int64_t* __restrict__ out_offsets, float* __restrict__ out,
                             FusedParams f, TableOrder order) {
  constexpr int OP = WEIGHTED ? kOpWeighted : kOpSum;
  constexpr int STREAM_DEPTH = (DEPTH <= 4 || LPR < 8) ? 4 : 8;  // as for its own launch
  const uint32_t blk = blockIdx.x;
  if (blk < f.end_block[0])
    wave_body<LPR, ELEM, DEPTH, OP, true>(tables, table_offsets, indices, offsets, weights,
                                          table_hints, hot_rows, out_offsets, out, f.seg[0], order,
                                          f.order_base[0], blk);
  else if (blk < f.end_block[1])
    stream_body<LPR, ELEM, STREAM_DEPTH, OP, false>(tables, table_offsets, indices, offsets,
                                                          weights, table_hints, hot_rows, out_offsets, out,
                                                          f.seg[1], order, f.order_base[1],
                                                          blk - f.end_block[0]);
}

template <int LPR, int ELEM>
FusedFn pick_w(int depth, bool weighted) {
  if (depth == 4)
    return weighted ? emb_bag_fused_uniform_kernel<LPR, ELEM, 4, true>
                    : emb_bag_fused_uniform_kernel<LPR, ELEM, 4, false>;
  if (depth == 8)
    return weighted ? emb_bag_fused_uniform_kernel<LPR, ELEM, 8, true>
                    : emb_bag_fused_uniform_kernel<LPR, ELEM, 8, false>;
  return nullptr;
}

}  // namespace

namespace embbag {

FusedFn EMB_PASTE(pick_fused_uniform_kernel_lpr, EMB_LPR)(int elem, int depth, bool weighted) {
  switch (elem) {
    case EMB_F32: return pick_w<EMB_LPR, EMB_F32>(depth, weighted);
    case EMB_F16: return pick_w<EMB_LPR, EMB_F16>(depth, weighted);
    case EMB_BF16: return pick_w<EMB_LPR, EMB_BF16>(depth, weighted);
    case EMB_U8ROW: return pick_w<EMB_LPR, EMB_U8ROW>(depth, weighted);
    case EMB_FP8ROW: return pick_w<EMB_LPR, EMB_FP8ROW>(depth, weighted);
    default: return nullptr;
  }
}

}  // namespace embbag
