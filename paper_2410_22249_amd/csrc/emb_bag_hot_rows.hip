// The hot-row profile: which rows of each table a batch looks up most often.  The paper finds the
// top 60K indices of every table by profiling offline and keeps their rows in L2 (Sec. 4.3,
// "What, When, and How to Pin?"); this is that profiling step on the device, from a sample
// batch: per table, the k most frequently named row ids and how often each was named.  What the
// caller does with them (lay the table out hot rows first and pass emb_bag_desc.hot_rows) is its
// own, offline, step.
//
// One 1024-thread workgroup per table, working in that table's own part of a scratch buffer (so
// workgroup barriers are the only synchronisation needed):
//   1. an open-addressing hash table of 64-bit slots, (row id + 1) << 24 | count, is cleared and
//      the table's first `window` lookups are inserted with compare-and-swap / add atomics;
//   2. every occupied slot stands for one key  count << 40 | (2^40 - 1 - id): larger = named more
//      often, ties to the smaller id.  The k-th largest key is found by a radix select over the
//      slots, eight bits per pass from the top (a 256-bin histogram in LDS per pass);
//   3. the slots at or above that key are copied to a second part of the scratch buffer, padded
//      with zeros to a power of two, sorted there in descending order (bitonic, one workgroup),
//      and written out as ids and counts.
// All keys are distinct, so the result is unique and can be checked bit for bit.
//
// The scratch buffer is either the caller's workspace or, for callers that cannot allocate, a
// fixed array in device memory that belongs to the library (emb_bag_profile_hot_rows_noalloc).

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/emb_bag.h"

// Scratch memory of emb_bag_profile_hot_rows_noalloc: 16 MiB of device memory that every GPU the
// library runs on holds from the moment the library is loaded until the process ends.  In host
// code this name is only a handle; the array's device address comes from hipGetSymbolAddress
// (once per device, see scratch_on_current_device) and is what kernels and copies are given.
constexpr uint64_t kScratchWords = 2ull << 20;
static __device__ __align__(256) unsigned long long scratch[kScratchWords];

namespace {

constexpr int kThreads = 1024;
constexpr int kIdBits = 40;                      // row ids below 2^40 - 1 are counted
constexpr int kCountBits = 24;                   // at most 2^24 - 1 lookups per table examined
constexpr uint64_t kIdMask = (1ull << kIdBits) - 1ull;
constexpr int64_t kMaxWindow = (1ll << kCountBits) - 1;
constexpr int64_t kMaxK = 1 << 16;

// Words (8 bytes each) a table needs: its hash slots, then its sort buffer.
struct Layout {
  uint64_t slots;  // power of two, >= 2 * window
  uint64_t kpad;   // power of two, >= k
};

bool make_layout(int64_t window, int64_t k, Layout* L) {
  if (window < 1 || window > kMaxWindow || k < 1 || k > kMaxK) return false;
  uint64_t s = 64;
  while (s < 2ull * (uint64_t)window) s <<= 1;
  uint64_t kp = 2;
  while (kp < (uint64_t)k) kp <<= 1;
  L->slots = s;
  L->kpad = kp;
  return true;
}

__device__ __forceinline__ uint64_t slot_load(const uint64_t* p) {
  // slots are written by atomics (performed in L2): read them past the L1 as well
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// key of an occupied slot: count << 40 | (2^40 - 1 - id); 0 for an empty slot
__device__ __forceinline__ uint64_t slot_key(uint64_t slot) {
  if (slot == 0) return 0;
  const uint64_t id = (slot >> kCountBits) - 1ull;
  const uint64_t count = slot & ((1ull << kCountBits) - 1ull);
  return (count << kIdBits) | (kIdMask - id);
}

__global__ void __launch_bounds__(kThreads)
emb_bag_hot_rows_kernel(const int64_t* __restrict__ indices, const int64_t* __restrict__ offsets,
                        int64_t* __restrict__ hot_ids, int32_t* __restrict__ hot_counts,
                        int32_t* __restrict__ num_hot, uint64_t* __restrict__ scratch,
                        int64_t num_lookups, uint32_t B, int64_t window, uint32_t k,
                        uint64_t num_slots, uint64_t kpad) {
  __shared__ uint32_t hist[256];
  __shared__ uint64_t sh_prefix;
  __shared__ uint32_t sh_need, sh_count;
  const uint32_t t = blockIdx.x;
  const uint32_t tid = threadIdx.x;
  uint64_t* slots = scratch + (uint64_t)t * (num_slots + kpad);
  uint64_t* sorted = slots + num_slots;

  for (uint64_t i = tid; i < num_slots; i += kThreads) slots[i] = 0;
  __threadfence();
  __syncthreads();

  // 1. count the row ids of the table's first `window` lookups
  int64_t s = offsets[(uint64_t)t * B];
  int64_t e = offsets[(uint64_t)(t + 1) * B];
  s = s < 0 ? 0 : (s > num_lookups ? num_lookups : s);
  e = e < s ? s : (e > num_lookups ? num_lookups : e);
  const int64_t n = e - s < window ? e - s : window;
  const uint64_t mask = num_slots - 1;
  for (int64_t i = tid; i < n; i += kThreads) {
    const int64_t id = indices[s + i];
    if (id < 0 || (uint64_t)id >= kIdMask) continue;  // not a countable row id
    const uint64_t tag = (uint64_t)id + 1ull;
    uint64_t h = (((uint64_t)id * 0x9E3779B97F4A7C15ull) >> 20) & mask;
    for (uint64_t probe = 0; probe < num_slots; ++probe) {  // load factor <= 1/2: ends early
      uint64_t cur = slot_load(slots + h);
      if (cur == 0) {
        cur = atomicCAS(reinterpret_cast<unsigned long long*>(slots + h), 0ull,
                        (unsigned long long)((tag << kCountBits) | 1ull));
        if (cur == 0) break;  // this lookup opened the slot with count 1
      }
      if ((cur >> kCountBits) == tag) {
        atomicAdd(reinterpret_cast<unsigned long long*>(slots + h), 1ull);
        break;
      }
      h = (h + 1) & mask;
    }
  }
  __threadfence();
  __syncthreads();

  // 2. radix select: the k-th largest key among the occupied slots (0 if there are fewer than k)
  if (tid == 0) {
    sh_prefix = 0;
    sh_need = k;
  }
  for (int shift = 56; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const uint64_t prefix = sh_prefix;
    const uint64_t high_mask = shift == 56 ? 0ull : ~0ull << (shift + 8);
    for (uint64_t i = tid; i < num_slots; i += kThreads) {
      const uint64_t key = slot_key(slot_load(slots + i));
      if (key != 0 && (key & high_mask) == prefix) atomicAdd(&hist[(key >> shift) & 0xFFu], 1u);
    }
    __syncthreads();
    if (tid == 0) {
      uint32_t need = sh_need, digit = 0;
      bool found = false;
      for (int d = 255; d >= 0; --d) {
        if (hist[d] >= need) {
          digit = (uint32_t)d;
          found = true;
          break;
        }
        need -= hist[d];
      }
      if (found) {
        sh_prefix = prefix | ((uint64_t)digit << shift);
        sh_need = need;
      } else {  // fewer than k keys share this prefix (only at the top: fewer than k keys at all)
        sh_prefix = 0;
        sh_need = 0;
        shift = -8;  // (thread 0's copy; the others learn from sh_need below)
      }
    }
    __syncthreads();
    if (sh_need == 0) break;
  }
  const uint64_t kth = sh_need == 0 ? 1ull : sh_prefix;  // keys >= kth are the answer (all keys if few)

  // 3. copy them out, pad, sort descending, write
  if (tid == 0) sh_count = 0;
  __syncthreads();
  for (uint64_t i = tid; i < num_slots; i += kThreads) {
    const uint64_t key = slot_key(slot_load(slots + i));
    if (key != 0 && key >= kth) {
      const uint32_t pos = atomicAdd(&sh_count, 1u);
      if (pos < kpad) sorted[pos] = key;
    }
  }
  __syncthreads();
  const uint32_t found = sh_count < k ? sh_count : k;
  for (uint64_t i = found + tid; i < kpad; i += kThreads) sorted[i] = 0;
  __syncthreads();
  for (uint64_t size = 2; size <= kpad; size <<= 1) {
    for (uint64_t stride = size >> 1; stride > 0; stride >>= 1) {
      for (uint64_t i = tid; i < kpad / 2; i += kThreads) {
        const uint64_t lo = 2 * i - (i & (stride - 1));  // partner pairs (lo, lo + stride)
        const uint64_t hi = lo + stride;
        const bool descending = (lo & size) == 0;
        const uint64_t a = sorted[lo], b = sorted[hi];
        if (descending ? a < b : a > b) {
          sorted[lo] = b;
          sorted[hi] = a;
        }
      }
      __syncthreads();
    }
  }
  for (uint32_t r = tid; r < k; r += kThreads) {
    const uint64_t key = r < found ? sorted[r] : 0;
    hot_ids[(uint64_t)t * k + r] = key ? (int64_t)(kIdMask - (key & kIdMask)) : -1;
    hot_counts[(uint64_t)t * k + r] = (int32_t)(key >> kIdBits);
  }
  if (tid == 0 && num_hot) num_hot[t] = (int32_t)found;
}

int check_and_launch(const emb_bag_desc* desc, const int64_t* indices, const int64_t* offsets,
                     int64_t window, int64_t k, int64_t* hot_ids, int32_t* hot_counts,
                     int32_t* num_hot, uint64_t* scratch, uint64_t scratch_words, void* stream) {
  if (!desc) return EMB_ERR_NULL_PTR;
  if (desc->num_tables < 1) return EMB_ERR_BAD_DIM;
  if (desc->batch < 0 || desc->num_lookups < 0) return EMB_ERR_BAD_SIZE;
  Layout L;
  if (!make_layout(window, k, &L)) return EMB_ERR_BAD_SIZE;
  const int64_t T = desc->num_tables, B = desc->batch;
  if (B == 0) return EMB_OK;
  if (!offsets || !hot_ids || !hot_counts || !scratch) return EMB_ERR_NULL_PTR;
  if (desc->num_lookups > 0 && !indices) return EMB_ERR_NULL_PTR;
  if (B > 0x7FFFFFFF || T * B > 0x7FFFFFFF) return EMB_ERR_BAD_SIZE;
  if ((uint64_t)T * (L.slots + L.kpad) > scratch_words) return EMB_ERR_BAD_SIZE;
  hipLaunchKernelGGL(emb_bag_hot_rows_kernel, dim3((uint32_t)T), dim3(kThreads), 0,
                     static_cast<hipStream_t>(stream), indices, offsets, hot_ids, hot_counts,
                     num_hot, scratch, desc->num_lookups, (uint32_t)B, window, (uint32_t)k, L.slots,
                     L.kpad);
  return hipGetLastError() == hipSuccess ? EMB_OK : EMB_ERR_LAUNCH;
}

// The device address of `scratch` on the current device: asked for once per device, then kept
// (every GPU has its own copy of the array at its own address).
constexpr int kMaxDevices = 64;
uint64_t* g_scratch_ptr[kMaxDevices];

int scratch_on_current_device(uint64_t** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return EMB_ERR_LAUNCH;
  uint64_t* p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym)
      return EMB_ERR_LAUNCH;
    p = static_cast<uint64_t*>(sym);
    __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);  // (a racing thread stores the same)
  }
  *ptr = p;
  return EMB_OK;
}

}  // namespace

extern "C" {

int emb_bag_profile_hot_rows_noalloc(const emb_bag_desc* desc, const int64_t* indices,
                                     const int64_t* offsets, int64_t window, int64_t k,
                                     int64_t* hot_ids, int32_t* hot_counts, int32_t* num_hot,
                                     void* stream) {
  uint64_t* ptr = nullptr;
  const int rc = scratch_on_current_device(&ptr);
  if (rc != EMB_OK) return rc;
  return check_and_launch(desc, indices, offsets, window, k, hot_ids, hot_counts, num_hot, ptr,
                          kScratchWords, stream);
}

int64_t emb_bag_profile_hot_rows_workspace(int32_t num_tables, int64_t window, int64_t k) {
  Layout L;
  if (num_tables < 1 || !make_layout(window, k, &L)) return EMB_ERR_BAD_SIZE;
  return (int64_t)num_tables * (int64_t)(L.slots + L.kpad) * 8;
}

int emb_bag_profile_hot_rows(const emb_bag_desc* desc, const int64_t* indices,
                             const int64_t* offsets, int64_t window, int64_t k, int64_t* hot_ids,
                             int32_t* hot_counts, int32_t* num_hot, void* workspace,
                             int64_t workspace_bytes, void* stream) {
  if (workspace_bytes < 0 || (reinterpret_cast<uintptr_t>(workspace) & 7))
    return workspace_bytes < 0 ? EMB_ERR_BAD_SIZE : EMB_ERR_ALIGNMENT;
  return check_and_launch(desc, indices, offsets, window, k, hot_ids, hot_counts, num_hot,
                          static_cast<uint64_t*>(workspace), (uint64_t)workspace_bytes / 8, stream);
}

}  // extern "C"
