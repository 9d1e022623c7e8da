// Multi-table EmbeddingBag forward for MI355X (gfx950, CDNA4): the C-ABI entry points that enqueue
// work (emb_bag_forward, emb_bag_forward_mixed, emb_bag_validate, emb_bag_profile_reuse), the
// validator and the reuse profiler kernels (the offline profiling of paper Sec. 4.3, on the
// device).  What a forward call launches is decided in emb_bag_plan.cpp (plain C++); the forward
// kernels live in emb_bag_wave.hip (one wavefront per bag), emb_bag_stream.hip (short bags) and
// the fused variants, shared device code in emb_bag_device.h.

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <vector>

#include "../../include/emb_bag.h"
#include "emb_bag_device.h"
#include "emb_bag_plan.h"

namespace {

using namespace embbag;
using namespace embbag::host;

// One wavefront per bag: count bad bounds and bad indices.
__global__ void __launch_bounds__(kBlock)
emb_bag_validate_kernel(const int64_t* __restrict__ table_offsets,
                        const int64_t* __restrict__ indices, const int64_t* __restrict__ offsets,
                        unsigned long long* __restrict__ num_bad, int64_t num_lookups, uint32_t B,
                        uint32_t num_bags) {
  const int lane = threadIdx.x & (kWaveSize - 1);
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t bag64 = (uint64_t)blockIdx.x * kWavesPerBlock + wave;
  if (bag64 >= num_bags) return;
  const uint32_t bag = (uint32_t)bag64;
  const uint32_t t = bag / B;
  int64_t s = uniform64(offsets[bag]);
  int64_t e = uniform64(offsets[bag + 1]);
  unsigned long long bad = 0;
  if (lane == 0) {
    if (s < 0 || e < s || e > num_lookups) bad += 1;
    if (bag == 0 && s != 0) bad += 1;
    if (bag == num_bags - 1 && e != num_lookups) bad += 1;
  }
  s = s < 0 ? 0 : (s > num_lookups ? num_lookups : s);
  e = e < s ? s : (e > num_lookups ? num_lookups : e);
  const int64_t R = uniform64(table_offsets[t + 1]) - uniform64(table_offsets[t]);
  for (int64_t j = s + lane; j < e; j += kWaveSize) {
    const int64_t idx = indices[j];
    if (idx < 0 || idx >= R) bad += 1;
  }
#pragma unroll
  for (int m = kWaveSize / 2; m >= 1; m >>= 1) bad += __shfl_xor(bad, m);
  if (lane == 0 && bad) atomicAdd(num_bad, bad);
}

// One workgroup per table: insert the first `window` lookups of the table into an open-addressing
// hash set in LDS (32-bit compare-and-swap, linear probing) and count the inserts that find their
// row id already present.  A slot holds the position of a lookup inside the window, not its row
// id (the id is read back from `indices` to compare), so 16,384 lookups fit in 96 KiB.  The count
// does not depend on the order of the inserts.
constexpr int kProfileThreads = 1024;
constexpr int kProfileMaxWindow = 16384;
constexpr int kProfileDefaultPermille = 75;
constexpr int kProfileMaxPermille = 1000000;  // keeps threshold * window^2 * 128 inside 64 bits
// d repeats among n draws put the rows in use at n^2 / 2d; they outgrow the last-level
// (memory-side) cache of 256 MiB = 2^28 bytes when n^2 * row_bytes > d * 2^29.  Rows narrower
// than a 128-byte line share it with 128 / row_bytes others, which makes a line that much more
// likely to be asked for again before it leaves, and the bar that much higher:
// n^2 * row_bytes * min(row_bytes, 128) > d * 2^36.
constexpr int kProfileCacheShift = 36;

inline uint32_t profile_slots(int32_t window) {  // load factor <= 2/3: every probe sequence ends
  return (uint32_t)window + (uint32_t)window / 2u + 2u;
}

__global__ void __launch_bounds__(kProfileThreads)
emb_bag_profile_kernel(const int64_t* __restrict__ indices, const int64_t* __restrict__ offsets,
                       int32_t* __restrict__ dup_count, int32_t* __restrict__ window_used,
                       uint8_t* __restrict__ hints, int64_t num_lookups, uint32_t B,
                       int32_t window, int32_t threshold_permille, uint32_t row_bytes,
                       uint32_t num_slots) {
  extern __shared__ uint32_t slots[];
  __shared__ int dups;
  constexpr uint32_t kEmpty = ~0u;
  const uint32_t t = blockIdx.x;
  for (uint32_t i = threadIdx.x; i < num_slots; i += kProfileThreads) slots[i] = kEmpty;
  if (threadIdx.x == 0) dups = 0;
  __syncthreads();

  int64_t s = offsets[(uint64_t)t * B];
  int64_t e = offsets[(uint64_t)(t + 1) * B];
  s = s < 0 ? 0 : (s > num_lookups ? num_lookups : s);
  e = e < s ? s : (e > num_lookups ? num_lookups : e);
  const int64_t n64 = e - s;
  const int n = n64 < window ? (int)n64 : window;

  int mine = 0;
  for (int i = threadIdx.x; i < n; i += kProfileThreads) {
    const unsigned long long key = (unsigned long long)indices[s + i];
    uint32_t slot = (uint32_t)((key * 0x9E3779B97F4A7C15ull) >> 40) % num_slots;
    for (uint32_t probe = 0; probe < num_slots; ++probe) {
      const uint32_t old = atomicCAS(&slots[slot], kEmpty, (uint32_t)i);
      if (old == kEmpty) break;
      if ((unsigned long long)indices[s + old] == key) {
        ++mine;
        break;
      }
      slot = slot + 1 == num_slots ? 0 : slot + 1;
    }
  }
  if (mine) atomicAdd(&dups, mine);
  __syncthreads();
  if (threadIdx.x == 0) {
    const int64_t d = dups;
    if (dup_count) dup_count[t] = (int32_t)d;
    if (window_used) window_used[t] = n;
    // d repeats among n draws put the rows in use at about n^2 / 2d.  Streaming: those rows do
    // not fit the last-level cache, or few of the table's n64 lookups of the whole batch find
    // their cache line already fetched (n64 draws over n^2 / 2d rows repeat a row in about
    // n64 * d / n^2 of cases, and a 128-byte line holds 128 / row_bytes rows), or nothing was
    // examined.  The share test is n64 * d * 1000 * 128 < threshold * n^2 * min(row_bytes, 128),
    // taken without overflow.
    const int64_t n2 = (int64_t)n * n;
    const int64_t line_rows = row_bytes < 128u ? row_bytes : 128u;  // 128 / rows per line
    const int64_t bar = (int64_t)threshold_permille * n2 * line_rows;
    const bool beyond_cache = n2 * (int64_t)row_bytes * line_rows > (d << kProfileCacheShift);
    const bool few_repeats = bar > 0 && n64 * d <= ((bar - 1) / 1000) / 128;
    if (hints) hints[t] = (n == 0 || beyond_cache || few_repeats) ? EMB_HINT_STREAMING
                                                                  : EMB_HINT_DEFAULT;
  }
}

// A cap on resident workgroups per CU is imposed through a dynamic LDS request that the kernel
// never touches: k workgroups fit when each asks for 1/k of the CU's LDS.
int occupancy_cap_lds(const void* fn, int64_t blocks_per_cu, uint32_t* lds) {
  *lds = 0;
  if (blocks_per_cu <= 0) return EMB_OK;
  int dev = 0, lds_per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&lds_per_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor,
                            dev) != hipSuccess || lds_per_cu <= 0)
    return EMB_ERR_LAUNCH;
  *lds = ((uint32_t)lds_per_cu / (uint32_t)blocks_per_cu) & ~1023u;
  if (*lds > 65536u &&
      hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)*lds) != hipSuccess)
    return EMB_ERR_LAUNCH;
  return EMB_OK;
}

// Apply the occupancy cap and launch what was planned.
int launch(const Launch& L, const void* tables, const int64_t* table_offsets,
           const int64_t* indices, const int64_t* offsets, const float* weights,
           const uint8_t* table_hints, const int64_t* hot_rows, const int64_t* out_offsets,
           float* out, void* stream) {
  uint32_t lds = 0;
  const int rc = occupancy_cap_lds(reinterpret_cast<const void*>(L.fn), L.tuning.blocks_per_cu,
                                   &lds);
  if (rc != EMB_OK) return rc;
  if (lds < L.lds_bytes) lds = L.lds_bytes;  // the LDS station's slots (at most 32 KiB)
  hipLaunchKernelGGL(L.fn, dim3(L.blocks), dim3(kBlock), lds, static_cast<hipStream_t>(stream),
                     static_cast<const char*>(tables), table_offsets, indices, offsets, weights,
                     table_hints, L.hot ? hot_rows : nullptr, out_offsets, out, L.p, L.order);
  return hipGetLastError() == hipSuccess ? EMB_OK : EMB_ERR_LAUNCH;
}

int launch_fused(const FusedLaunch& F, const void* tables, const int64_t* table_offsets,
                 const int64_t* indices, const int64_t* offsets, const float* weights,
                 const uint8_t* table_hints, const int64_t* out_offsets, float* out,
                 void* stream) {
  uint32_t lds = 0;
  const int rc = occupancy_cap_lds(reinterpret_cast<const void*>(F.fn), F.blocks_per_cu, &lds);
  if (rc != EMB_OK) return rc;
  hipLaunchKernelGGL(F.fn, dim3(F.blocks), dim3(kBlock), lds, static_cast<hipStream_t>(stream),
                     static_cast<const char*>(tables), table_offsets, indices, offsets, weights,
                     table_hints, static_cast<const int64_t*>(nullptr), out_offsets, out, F.f,
                     F.order);
  return hipGetLastError() == hipSuccess ? EMB_OK : EMB_ERR_LAUNCH;
}

}  // namespace

extern "C" {


int emb_bag_forward(const emb_bag_desc* desc, const void* tables, const int64_t* table_offsets,
                    const int64_t* indices, const int64_t* offsets,
                    const float* per_sample_weights, float* out, void* stream) {
  uint32_t row_bytes = 0;
  int64_t out_ld = 0;
  int rc = precheck_uniform(desc, per_sample_weights != nullptr, &row_bytes, &out_ld);
  if (rc != EMB_OK) return rc;
  if (desc->batch == 0) return EMB_OK;
  if (!tables || !table_offsets || !offsets || !out) return EMB_ERR_NULL_PTR;
  if (desc->num_lookups > 0 && !indices) return EMB_ERR_NULL_PTR;
  if ((reinterpret_cast<uintptr_t>(tables) | reinterpret_cast<uintptr_t>(out)) & 15)
    return EMB_ERR_ALIGNMENT;
  std::vector<Launch> launches;
  rc = plan_uniform(desc, per_sample_weights != nullptr, row_bytes, out_ld, &launches);
  if (rc == EMB_OK) rc = check_grids(launches);
  if (rc != EMB_OK) return rc;
  FusedLaunch fused;
  if (plan_fused(launches, false, desc->table_dtype, per_sample_weights != nullptr, &fused))
    return launch_fused(fused, tables, table_offsets, indices, offsets, per_sample_weights,
                        desc->table_hints, nullptr, out, stream);
  for (const Launch& L : launches) {  // disjoint tables: the launches are independent
    rc = launch(L, tables, table_offsets, indices, offsets, per_sample_weights, desc->table_hints,
                desc->hot_rows, nullptr, out, stream);
    if (rc != EMB_OK) return rc;
  }
  return EMB_OK;
}

int emb_bag_forward_mixed(const emb_bag_mixed_desc* desc, const void* tables,
                          const int64_t* table_byte_offsets, const int64_t* out_offsets,
                          const int64_t* indices, const int64_t* offsets,
                          const float* per_sample_weights, float* out, void* stream) {
  uint32_t max_row_bytes = 0;
  int64_t out_ld = 0;
  int rc = precheck_mixed(desc, per_sample_weights != nullptr, &max_row_bytes, &out_ld);
  if (rc != EMB_OK) return rc;
  if (desc->batch == 0) return EMB_OK;
  if (!tables || !table_byte_offsets || !out_offsets || !offsets || !out) return EMB_ERR_NULL_PTR;
  if (desc->num_lookups > 0 && !indices) return EMB_ERR_NULL_PTR;
  if ((reinterpret_cast<uintptr_t>(tables) | reinterpret_cast<uintptr_t>(out)) & 15)
    return EMB_ERR_ALIGNMENT;
  std::vector<Launch> launches;
  rc = plan_mixed(desc, per_sample_weights != nullptr, max_row_bytes, out_ld, &launches);
  if (rc == EMB_OK) rc = check_grids(launches);
  if (rc != EMB_OK) return rc;
  FusedLaunch fused;
  if (plan_fused(launches, true, desc->table_dtype, per_sample_weights != nullptr, &fused))
    return launch_fused(fused, tables, table_byte_offsets, indices, offsets, per_sample_weights,
                        desc->table_hints, out_offsets, out, stream);
  for (const Launch& L : launches) {  // disjoint tables: the launches are independent
    rc = launch(L, tables, table_byte_offsets, indices, offsets, per_sample_weights,
                desc->table_hints, nullptr, out_offsets, out, stream);
    if (rc != EMB_OK) return rc;
  }
  return EMB_OK;
}

int emb_bag_validate(const emb_bag_desc* desc, const int64_t* table_offsets,
                     const int64_t* indices, const int64_t* offsets, int64_t* num_bad,
                     void* stream) {
  uint32_t row_bytes = 0;
  const int rc = check_desc(desc, &row_bytes);
  if (rc != EMB_OK) return rc;
  const int64_t T = desc->num_tables, B = desc->batch;
  if (B == 0) return EMB_OK;
  if (!table_offsets || !offsets || !num_bad) return EMB_ERR_NULL_PTR;
  if (desc->num_lookups > 0 && !indices) return EMB_ERR_NULL_PTR;
  if (B > 0x7FFFFFFF || T * B > 0x7FFFFFFF) return EMB_ERR_BAD_SIZE;
  const uint32_t num_bags = (uint32_t)(T * B);
  const uint32_t blocks = (num_bags + kWavesPerBlock - 1) / kWavesPerBlock;
  if (blocks > kMaxBlocks) return EMB_ERR_BAD_SIZE;
  hipLaunchKernelGGL(emb_bag_validate_kernel, dim3(blocks), dim3(kBlock), 0,
                     static_cast<hipStream_t>(stream), table_offsets, indices, offsets,
                     reinterpret_cast<unsigned long long*>(num_bad), desc->num_lookups,
                     (uint32_t)B, num_bags);
  return hipGetLastError() == hipSuccess ? EMB_OK : EMB_ERR_LAUNCH;
}

int emb_bag_profile_reuse(const emb_bag_desc* desc, const int64_t* indices,
                          const int64_t* offsets, int32_t window, int32_t threshold_permille,
                          int32_t* dup_count, int32_t* window_used, uint8_t* hints,
                          void* stream) {
  uint32_t row_bytes = 0;
  const int rc = check_desc(desc, &row_bytes);
  if (rc != EMB_OK) return rc;
  const int64_t T = desc->num_tables, B = desc->batch;
  if (B == 0) return EMB_OK;
  if (!offsets) return EMB_ERR_NULL_PTR;
  if (desc->num_lookups > 0 && !indices) return EMB_ERR_NULL_PTR;
  if (B > 0x7FFFFFFF || T * B > 0x7FFFFFFF) return EMB_ERR_BAD_SIZE;
  if (window < 1) window = 1;
  if (window > kProfileMaxWindow) window = kProfileMaxWindow;
  if (threshold_permille < 0) threshold_permille = kProfileDefaultPermille;
  if (threshold_permille > kProfileMaxPermille) threshold_permille = kProfileMaxPermille;
  const uint32_t num_slots = profile_slots(window);
  const uint32_t lds = num_slots * 4u;
  if (lds > 65536u &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(emb_bag_profile_kernel),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
    return EMB_ERR_LAUNCH;
  hipLaunchKernelGGL(emb_bag_profile_kernel, dim3((uint32_t)T), dim3(kProfileThreads), lds,
                     static_cast<hipStream_t>(stream), indices, offsets, dup_count, window_used,
                     hints, desc->num_lookups, (uint32_t)B, window, threshold_permille, row_bytes,
                     num_slots);
  return hipGetLastError() == hipSuccess ? EMB_OK : EMB_ERR_LAUNCH;
}
}  // extern "C"
