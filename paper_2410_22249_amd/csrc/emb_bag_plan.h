// Host-side planning of a forward call: everything decided before a launch (kernel
// instantiation, prefetch depth, grid, block order, table lists, fusing) and the process-wide
// tuning it follows.  Plain C++ without HIP calls or device pointers being read: the same code
// is built for the CPU under sanitizers by the tests.  Not part of the C ABI.
#pragma once

#include <stdint.h>

#include <vector>

#include "../../include/emb_bag.h"
#include "emb_bag_params.h"

namespace embbag {
namespace host {

struct Tuning {
  int64_t depth = 0;
  int64_t addressing = 0;
  int64_t blocks_per_cu = 0;
  int64_t xcd_remap = -1;
  int64_t use_hints = 1;
  int64_t stream = -1;          // short-bag kernel: -1 = by average bag length, 0 = never, 1 = when possible
  int64_t bags_per_group = 0;   // its consecutive bags per lane group: 0 = automatic
  int64_t xcd_pieces = 0;       // pieces per table in XCD-affine order: 0 = automatic, 1, 2, 4, 8
  int64_t per_table_launch = 0; // 1 = one launch per table, as the paper's system does (Sec. 3.1)
  int64_t fuse = 1;             // 1 = the launches of a split call become one launch
  int64_t bags_per_wave = 0;    // wave kernel: consecutive bags per wavefront, 0 = automatic
  int64_t hot_split = 0;        // desc->hot_rows: 0 = not used, 1 = regroup + cold rows nt, 2 = regroup
  int64_t station = 0;          // where row loads land: 0 = registers, 1 = LDS (paper Sec. 4.2)
};
extern Tuning g_tuning;

// A dispatch counts its work-items in 32 bits, so a launch of 256-thread workgroups holds at most
// 2^24 - 1 of them (67,108,860 wavefronts).  Larger calls are refused, not split.
constexpr uint64_t kMaxBlocks = 0xFFFFFFull;

// Everything a forward call decides on the host before it launches: the kernel instantiation,
// its parameters, the grid and the table order.  Filled by plan_uniform / plan_mixed, launched
// by emb_bag.hip, reported by emb_bag_plan_forward*.
struct Launch {
  KernelFn fn = nullptr;
  KParams p = {};
  TableOrder order = {};  // table at each position of the launch; read only when p.listed is set
  int64_t tables = 0;     // positions of the launch
  uint32_t blocks = 0;
  int kernel = EMB_KERNEL_WAVE;
  int lpr = 0;
  int depth = 0;
  bool buf = false;
  int op = kOpSum;        // pooling of the call: kOpSum (sum and mean), kOpWeighted, kOpMax
  bool hot = false;       // the kernel splits a table's lookups into hot-head and other rows
  uint32_t lds_bytes = 0; // dynamic LDS the kernel uses (the LDS station), else 0
  Tuning tuning;          // what the call was planned from (the descriptor's, or process-wide)
};

// The launches of a split call as ONE launch: consecutive ranges of its workgroups run what
// would have been the separate launches (emb_bag_fused.hip, emb_bag_fused_uniform.hip).
struct FusedLaunch {
  FusedFn fn = nullptr;
  FusedParams f;
  TableOrder order;
  uint32_t blocks = 0;
  int64_t blocks_per_cu = 0;  // occupancy cap of the call (tuning key), 0 = none
};

int check_desc(const emb_bag_desc* d, uint32_t* row_bytes_out);
int precheck_uniform(const emb_bag_desc* desc, bool weighted, uint32_t* row_bytes, int64_t* out_ld);
int precheck_mixed(const emb_bag_mixed_desc* desc, bool weighted, uint32_t* max_row_bytes,
                   int64_t* out_ld);
int plan_uniform(const emb_bag_desc* desc, bool weighted, uint32_t row_bytes, int64_t out_ld,
                 std::vector<Launch>* launches);
int plan_mixed(const emb_bag_mixed_desc* desc, bool weighted, uint32_t max_row_bytes,
               int64_t out_ld, std::vector<Launch>* launches);
bool plan_fused(const std::vector<Launch>& segs, bool mixed, int table_dtype, bool weighted,
                FusedLaunch* F);
int check_grids(const std::vector<Launch>& launches);

}  // namespace host
}  // namespace embbag
