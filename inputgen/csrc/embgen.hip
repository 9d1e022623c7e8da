// Seeded synthetic-input generator, device side (gfx950).
//
// This file belongs to the input generator, not to the embedding-bag library and not to the
// CPU oracle: it holds none of the gather/pool arithmetic.  It provides
//   * gen_fill_table  - fill a row-major [nrows, D] slab of an embedding-table arena with
//                       procedural values that the host generator reproduces bit for bit, so
//                       100+ GB arenas never need a host copy;
//   * gen_alloc_arena / gen_free_arena - arena memory, optionally physically contiguous;
//   * gen_copy_bytes  - a plain device-to-device copy kernel of known size, used to calibrate
//                       the HBM byte counters of the profiler;
//   * gen_read_bytes  - a read-only streaming kernel: the measured read-bandwidth ceiling;
//   * gen_scrub_cache - stream over a scratch buffer to push earlier data out of L2 / MALL.
//
// Value function (shared, by construction, with inputgen/gen.py::table_values):
//   z  = seed + arena_row * K_ROW + col * K_COL              (mod 2^64)
//   z  = finaliser of the SplitMix64 generator (Steele, Lea, Flood 2014) applied to z
//   kind 0 ("normal"): s = sum of the four 16-bit fields of z - 131070   (Irwin-Hall, n = 4)
//                      v = (float)s * (0.1f / 37837.2f)      -> approx N(0, 0.1^2)
//   kind 1 ("int")   : v = (float)((int)(z >> 60) - 8)        -> integers in [-8, 7]
//   f16 tables store v rounded to half, bf16 tables v rounded to bfloat16, both to nearest even.
// Only integer operations, one exact int->float conversion and one correctly rounded fp32
// multiply are used, so numpy on the host and this kernel agree in every bit.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace {

constexpr uint64_t K_ROW = 0x9E3779B97F4A7C15ull;
constexpr uint64_t K_COL = 0xD1B54A32D192ED03ull;

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__device__ __forceinline__ float value_at(uint64_t seed, uint64_t row, uint64_t col, int kind) {
  const uint64_t z = mix64(seed + row * K_ROW + col * K_COL);
  if (kind == 1) return (float)((int)(z >> 60) - 8);
  const int s = (int)(z & 0xFFFF) + (int)((z >> 16) & 0xFFFF) + (int)((z >> 32) & 0xFFFF) +
                (int)((z >> 48) & 0xFFFF) - 131070;
  return __fmul_rn((float)s, 0.1f / 37837.2f);
}

// One thread produces one 16-byte vector (4 floats or 8 halves); D is a multiple of the
// vector width, so a vector never straddles two rows.
// fp32 -> bfloat16 bits, round to nearest even (finite inputs only; the generator makes no others)
__device__ __forceinline__ uint16_t bf16_bits_rn(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// ELEM: 0 = fp32, 1 = fp16, 2 = bfloat16
template <int ELEM>
__global__ __launch_bounds__(256) void fill_kernel(void* __restrict__ dst, uint64_t first_row,
                                                   uint64_t nvec, uint32_t D, uint64_t seed,
                                                   int kind) {
  constexpr uint32_t EPV = ELEM == 0 ? 4 : 8;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; v < nvec; v += stride) {
    const uint64_t e0 = v * EPV;
    const uint64_t row = e0 / D;
    const uint64_t col = e0 - row * D;
    float x[EPV];
#pragma unroll
    for (uint32_t k = 0; k < EPV; ++k) x[k] = value_at(seed, first_row + row, col + k, kind);
    if constexpr (ELEM == 1) {
      union { uint4 u; __half h[8]; } pk;
#pragma unroll
      for (uint32_t k = 0; k < EPV; ++k) pk.h[k] = __float2half_rn(x[k]);
      reinterpret_cast<uint4*>(dst)[v] = pk.u;
    } else if constexpr (ELEM == 2) {
      union { uint4 u; uint16_t h[8]; } pk;
#pragma unroll
      for (uint32_t k = 0; k < EPV; ++k) pk.h[k] = bf16_bits_rn(x[k]);
      reinterpret_cast<uint4*>(dst)[v] = pk.u;
    } else {
      reinterpret_cast<float4*>(dst)[v] = make_float4(x[0], x[1], x[2], x[3]);
    }
  }
}

// Row-wise quantised rows: D one-byte codes, then an fp32 scale and an fp32 bias (D + 8 bytes per
// row, a multiple of 16).  One thread writes one 16-byte vector of a row.  FP8: the codes are
// E4M3 numbers: the two NaN codes move to their neighbours, kind 1 clears the top exponent bit,
// and scale / bias are (256 + a) * 2e-6 / -32 * scale (kind 0) or 1 / -1 (kind 1).
template <bool FP8>
__global__ __launch_bounds__(256) void fill_quantised_kernel(uint4* __restrict__ dst,
                                                             uint64_t first_row, uint64_t nvec,
                                                             uint32_t D, uint64_t seed, int kind) {
  const uint32_t vec_per_row = (D + 8) / 16;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; v < nvec; v += stride) {
    const uint64_t row = v / vec_per_row;
    const uint32_t c0 = (uint32_t)(v - row * vec_per_row) * 16u;
    const uint64_t arow = first_row + row;
    union { uint4 u; uint8_t b[16]; uint32_t w[4]; } pk;
#pragma unroll
    for (uint32_t k = 0; k < 16; ++k) {
      const uint32_t col = c0 + k;
      uint8_t code =
          col < D ? (uint8_t)((mix64(seed + arow * K_ROW + (uint64_t)col * K_COL) >> 32) & 0xFF) : 0;
      if constexpr (FP8) {
        if ((code & 0x7F) == 0x7F) code &= 0xFE;
        if (kind == 1) code &= 0xBF;
      }
      pk.b[k] = code;
    }
    if (c0 + 16 > D) {  // this vector holds the row's last 8 codes, then scale and bias
      float scale = 1.0f;
      if (kind == 0) {
        const int a = (int)(mix64(seed + arow * K_ROW + (uint64_t)D * K_COL) & 0xFF);
        scale = __fmul_rn((float)(256 + a), FP8 ? 2.0e-6f : 3.5e-6f);
      }
      const float bias_factor = FP8 ? (kind == 1 ? -1.0f : -32.0f) : -128.0f;
      pk.w[2] = __builtin_bit_cast(uint32_t, scale);
      pk.w[3] = __builtin_bit_cast(uint32_t, __fmul_rn(bias_factor, scale));
    }
    dst[v] = pk.u;
  }
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst,
                                                   const uint4* __restrict__ src, uint64_t nvec) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; v < nvec; v += stride)
    dst[v] = src[v];
}

__global__ __launch_bounds__(256) void scrub_kernel(uint4* __restrict__ buf, uint64_t nvec) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; v < nvec; v += stride) {
    uint4 x = buf[v];
    x.x += 1u;
    buf[v] = x;
  }
}

// Read-only stream: every thread xors what it reads and writes one word only if the result is
// a value that never occurs, so the loads cannot be optimised away and nothing is written.
// Four independent non-temporal 16-byte loads per thread per trip: the fastest plain read found on
// MI355X (about 7.0 TB/s; the same loop with the default cache policy reaches 6.3 TB/s).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void read_kernel(const u32x4* __restrict__ src, uint64_t nvec,
                                                   uint32_t* __restrict__ sink) {
  constexpr int UNROLL = 4;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t x = 0;
  for (; v + (UNROLL - 1) * stride < nvec; v += UNROLL * stride) {
    u32x4 a[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) a[u] = __builtin_nontemporal_load(src + v + u * stride);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) x ^= a[u].x ^ a[u].y ^ a[u].z ^ a[u].w;
  }
  for (; v < nvec; v += stride) {
    const u32x4 a = __builtin_nontemporal_load(src + v);
    x ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (x == 0x9E3779B9u && sink) *sink = x;
}

unsigned grid_for(uint64_t nvec) {
  uint64_t blocks = (nvec + 255) / 256;
  const uint64_t cap = 256ull * 32ull;  // 32 workgroups per CU keeps every CU busy
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (unsigned)blocks;
}

}  // namespace

extern "C" {

// dst: DEVICE pointer to the first element of arena row `first_row` ([nrows, D] row-major).
// dtype: 0 = fp32, 1 = fp16, 2 = bfloat16, 3 / 4 = row-wise quantised with integer / E4M3 codes
// ([nrows, D + 8] bytes).  kind: 0 = normal, 1 = int.  Returns 0, or a negative code for a
// bad argument / a positive hipError_t for a failed launch.
int gen_fill_table(void* dst, int64_t first_row, int64_t nrows, int32_t D, int32_t dtype,
                   uint64_t seed, int32_t kind, void* stream) {
  if (nrows == 0) return 0;
  if (!dst || nrows < 0 || first_row < 0 || D <= 0) return -1;
  if (dtype < 0 || dtype > 4) return -2;
  if (kind != 0 && kind != 1) return -3;
  if (dtype >= 3) {  // quantised rows: D codes + 8 bytes, a whole number of 16-byte vectors
    if ((D + 8) % 16 != 0) return -4;
    if ((reinterpret_cast<uintptr_t>(dst) & 15) != 0) return -5;
    const uint64_t nv = (uint64_t)nrows * (uint64_t)((D + 8) / 16);
    if (dtype == 4)
      hipLaunchKernelGGL(fill_quantised_kernel<true>, dim3(grid_for(nv)), dim3(256), 0,
                         static_cast<hipStream_t>(stream), static_cast<uint4*>(dst),
                         (uint64_t)first_row, nv, (uint32_t)D, seed, kind);
    else
      hipLaunchKernelGGL(fill_quantised_kernel<false>, dim3(grid_for(nv)), dim3(256), 0,
                         static_cast<hipStream_t>(stream), static_cast<uint4*>(dst),
                         (uint64_t)first_row, nv, (uint32_t)D, seed, kind);
    return (int)hipGetLastError();
  }
  const uint32_t epv = dtype == 0 ? 4 : 8;
  if (D % epv != 0) return -4;
  if ((reinterpret_cast<uintptr_t>(dst) & 15) != 0) return -5;
  const uint64_t nvec = (uint64_t)nrows * (uint64_t)D / epv;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == 1)
    hipLaunchKernelGGL(fill_kernel<1>, dim3(grid_for(nvec)), dim3(256), 0, s, dst,
                       (uint64_t)first_row, nvec, (uint32_t)D, seed, kind);
  else if (dtype == 2)
    hipLaunchKernelGGL(fill_kernel<2>, dim3(grid_for(nvec)), dim3(256), 0, s, dst,
                       (uint64_t)first_row, nvec, (uint32_t)D, seed, kind);
  else
    hipLaunchKernelGGL(fill_kernel<0>, dim3(grid_for(nvec)), dim3(256), 0, s, dst,
                       (uint64_t)first_row, nvec, (uint32_t)D, seed, kind);
  return (int)hipGetLastError();
}

// Allocate nbytes of device memory for a table arena; *out receives the DEVICE pointer.
// contiguous != 0 asks the driver for physically contiguous VRAM (hipDeviceMallocContiguous), so
// that experiments can separate the effect of page-table fragment size from that of physical
// placement on random row gathers over 100+ GB.  Returns the hipError_t.
int gen_alloc_arena(void** out, int64_t nbytes, int32_t contiguous) {
  if (!out || nbytes <= 0) return -1;
  *out = nullptr;
  return (int)hipExtMallocWithFlags(out, (size_t)nbytes,
                                    contiguous ? hipDeviceMallocContiguous : hipDeviceMallocDefault);
}

// Free an arena from gen_alloc_arena (the caller has synchronised every stream that used it).
int gen_free_arena(void* ptr) { return ptr ? (int)hipFree(ptr) : 0; }

// Plain copy of nbytes (multiple of 16; both DEVICE pointers 16-byte aligned).
int gen_copy_bytes(void* dst, const void* src, int64_t nbytes, void* stream) {
  if (nbytes == 0) return 0;
  if (!dst || !src || nbytes < 0 || (nbytes & 15)) return -1;
  if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15) return -5;
  const uint64_t nvec = (uint64_t)nbytes / 16;
  hipLaunchKernelGGL(copy_kernel, dim3(grid_for(nvec)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<uint4*>(dst),
                     static_cast<const uint4*>(src), nvec);
  return (int)hipGetLastError();
}

// Read nbytes (multiple of 16, DEVICE pointer 16-byte aligned) and discard them: a streaming-read
// bandwidth probe.  `sink` is a DEVICE uint32 that is (practically) never written; may be NULL.
int gen_read_bytes(const void* src, int64_t nbytes, void* sink, void* stream) {
  if (nbytes == 0) return 0;
  if (!src || nbytes < 0 || (nbytes & 15)) return -1;
  if (reinterpret_cast<uintptr_t>(src) & 15) return -5;
  const uint64_t nvec = (uint64_t)nbytes / 16;
  uint64_t blocks = (nvec + 4 * 256 - 1) / (4 * 256);
  if (blocks > 32768) blocks = 32768;
  hipLaunchKernelGGL(read_kernel, dim3((unsigned)blocks), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const u32x4*>(src), nvec,
                     static_cast<uint32_t*>(sink));
  return (int)hipGetLastError();
}

// Read-modify-write over a scratch DEVICE buffer (nbytes multiple of 16) to evict caches.
int gen_scrub_cache(void* buf, int64_t nbytes, void* stream) {
  if (nbytes == 0) return 0;
  if (!buf || nbytes < 0 || (nbytes & 15)) return -1;
  if (reinterpret_cast<uintptr_t>(buf) & 15) return -5;
  const uint64_t nvec = (uint64_t)nbytes / 16;
  hipLaunchKernelGGL(scrub_kernel, dim3(grid_for(nvec)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<uint4*>(buf), nvec);
  return (int)hipGetLastError();
}

}  // extern "C"
