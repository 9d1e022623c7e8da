// Launch parameters, limits and kernel-picker declarations shared by the host-side planning
// (emb_bag_plan.cpp, plain C++: it is also built for the CPU with sanitizers) and the device code
// (emb_bag_device.h).  Nothing here needs the HIP headers; nothing here is part of the C ABI.
#pragma once

#include <stdint.h>

#include "../../include/emb_bag.h"

namespace embbag {

constexpr int kWaveSize = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWaveSize * kWavesPerBlock;
constexpr int kSlabBytes = 1024;                   // bytes of one row a wavefront covers per pass
constexpr uint32_t kBufSentinel = 0xF0000000u;     // offset that is out of range for any table
constexpr uint64_t kBufMaxBytes = 0xE0000000ull;   // largest table addressed through a buffer
constexpr uint32_t kBufWord3 = 0x00020000u;        // gfx9 buffer resource: 32-bit data format

// What a lookup does to the accumulator: plain sum, sum with per-sample weights, or maximum.
constexpr int kOpSum = 0, kOpWeighted = 1, kOpMax = 2;
// variants of the wave kernel (buffer addressing, tables of one width, depth 4 or 8): the hot /
// cold split with the other rows read non-temporally or with the default policy, and the LDS
// station (sum pooling)
constexpr int kVariantPlain = 0, kVariantHotNt = 1, kVariantHot = 2, kVariantLds = 3;

struct KParams {
  int64_t num_lookups;   // NL
  int64_t out_ld;        // floats
  int64_t max_rows;      // clamp on R_t in buffer mode (host guarantees max_rows*row_bytes fits)
  uint32_t B;            // bags per table
  uint32_t num_work;     // wavefronts with work: T * wpt
  uint32_t wpt;          // wavefronts per table
  uint32_t slabs;        // ceil(row_bytes / 1024)
  uint32_t row_bytes;
  uint32_t D;
  uint32_t mean;         // 1 = divide by bag length
  uint32_t has_hints;    // 1 = table_hints points to T bytes
  // XCD-affine block order (xcd_bpp = 0: natural order).  Every table is cut into 2^xcd_pshift
  // pieces of xcd_wpp wavefronts (xcd_bpp workgroups); piece u = t * 2^xcd_pshift + k runs on
  // XCD u % 8, and an XCD takes its pieces in increasing u.
  uint32_t xcd_bpp;
  uint32_t xcd_wpp;
  uint32_t xcd_pshift;
  uint32_t xcd_units;    // positions * pieces: units at or beyond this have no work
  uint32_t listed;       // 1 = position q of the launch holds table TableOrder::t[q], 0 = table q
  uint32_t bags_per_group;  // stream kernel: consecutive bags owned by one lane group
  uint32_t bags_per_wave;   // wave kernel: consecutive bags owned by one wavefront (1 if slabs > 1)
};

// A launch over tables of different widths may cover a subset of the tables (one lanes-per-row
// class for the stream kernel) and may take them in another order than the caller's: dealt out
// in their own order, tables of different widths load the XCDs unevenly (a wavefront's work
// grows with the row width), so the host deals them by width.  Either way the kernel receives
// the table at each position of the launch by value, in the kernel-argument segment.
constexpr int kMaxOrdered = 1024;
struct alignas(8) TableOrder {  // (aligned: the kernels read it in 32-bit words)
  uint16_t t[kMaxOrdered];
};

// Every forward kernel takes the same arguments: tables, table_offsets, indices, offsets,
// weights, table_hints, hot_rows (kernels with the hot / cold split only), out_offsets
// (different widths only), out, parameters, table order.
using KernelFn = void (*)(const char*, const int64_t*, const int64_t*, const int64_t*,
                          const float*, const uint8_t*, const int64_t*, const int64_t*, float*,
                          KParams, TableOrder);

// A fused launch runs several bodies over consecutive ranges of its workgroups.  Tables of
// different widths: segment 0 is the wave body, segments 1 .. 5 the stream body with 4, 8, 16,
// 32, 64 lanes per row.  Tables of one width: segment 0 the wave body, segment 1 the stream body.  Segment k owns workgroups [end_block[k-1], end_block[k]) (from 0 for k = 0; an
// unused segment is empty), every boundary a multiple of 8 so that a workgroup's index within
// its segment still names its XCD; its tables are TableOrder::t[order_base[k] ...].
constexpr int kFusedSegments = 6;
struct FusedParams {
  uint32_t end_block[kFusedSegments];
  uint32_t order_base[kFusedSegments];
  KParams seg[kFusedSegments];
};
using FusedFn = void (*)(const char*, const int64_t*, const int64_t*, const int64_t*,
                         const float*, const uint8_t*, const int64_t*, const int64_t*, float*,
                         FusedParams, TableOrder);
// emb_bag_fused.hip, one translation unit per element type; depth 4 or 8
#define EMB_DECLARE_FUSED(n) \
  __attribute__((visibility("hidden"))) FusedFn pick_fused_kernel_elem##n(int depth, bool weighted);
EMB_DECLARE_FUSED(0)
EMB_DECLARE_FUSED(1)
EMB_DECLARE_FUSED(2)
EMB_DECLARE_FUSED(3)
EMB_DECLARE_FUSED(4)
#undef EMB_DECLARE_FUSED

// emb_bag_fused_uniform.hip (tables of one width: segment 0 the wave body, segment 1 the stream
// body, both with the call's lanes per row), one translation unit per class; depth 4 or 8
#define EMB_DECLARE_FUSED_UNIFORM(n)                                                    \
  __attribute__((visibility("hidden"))) FusedFn pick_fused_uniform_kernel_lpr##n(int elem, \
                                                                                int depth, \
                                                                                bool weighted);
EMB_DECLARE_FUSED_UNIFORM(4)
EMB_DECLARE_FUSED_UNIFORM(8)
EMB_DECLARE_FUSED_UNIFORM(16)
EMB_DECLARE_FUSED_UNIFORM(32)
EMB_DECLARE_FUSED_UNIFORM(64)
#undef EMB_DECLARE_FUSED_UNIFORM

// The forward kernels are built one lanes-per-row class per translation unit; each unit exports
// one function that picks an instantiation (nullptr if there is none):
//   wave kernel (emb_bag_wave.hip):     lanes per row 0 (different widths), 4 .. 64
//   stream kernel (emb_bag_stream.hip): lanes per row 4 .. 64, rows of at most 1 KiB; `mixed`:
//     tables of different widths within the class
#define EMB_PASTE_(a, b) a##b
#define EMB_PASTE(a, b) EMB_PASTE_(a, b)
#define EMB_DECLARE_PICKERS(n)                                                                  \
  __attribute__((visibility("hidden"))) KernelFn pick_wave_kernel_lpr##n(                       \
      int elem, int depth, int op, bool buf, int variant);                                      \
  __attribute__((visibility("hidden"))) KernelFn pick_stream_kernel_lpr##n(                     \
      int elem, int depth, int op, bool mixed, bool buf);
EMB_DECLARE_PICKERS(0)  // (there is no stream kernel for class 0; the declaration is unused)
EMB_DECLARE_PICKERS(4)
EMB_DECLARE_PICKERS(8)
EMB_DECLARE_PICKERS(16)
EMB_DECLARE_PICKERS(32)
EMB_DECLARE_PICKERS(64)
#undef EMB_DECLARE_PICKERS

}  // namespace embbag
