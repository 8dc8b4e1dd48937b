// Device fill of the seeded synthetic tensors (gfx950).  Same integer hash as
// the host fill, so both write identical bits.  No method arithmetic here.
#include <hip/hip_runtime.h>
#include "counter_rng.h"

namespace {

// One thread writes 8 consecutive elements (two 64-bit draws).
template <typename T>
__global__ __launch_bounds__(256) void fill_kernel(T* __restrict__ dst, const T* __restrict__ table,
                                                   uint64_t key, uint64_t first_elem, uint64_t n) {
  uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t base = g * 8; base < n; base += stride * 8) {
    uint64_t e0 = first_elem + base;
    if ((e0 & 3u) == 0 && base + 8 <= n) {
      uint64_t h0 = synth_bits64(key, e0 >> 2);
      uint64_t h1 = synth_bits64(key, (e0 >> 2) + 1);
      T v[8];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[j] = table[(h0 >> (16 * j)) & 0xFFFFu];
        v[4 + j] = table[(h1 >> (16 * j)) & 0xFFFFu];
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) dst[base + j] = v[j];
    } else {
      for (uint64_t j = base; j < n && j < base + 8; ++j) dst[j] = table[synth_u16(key, first_elem + j)];
    }
  }
}

}  // namespace

// dst and table are device pointers; stream is a hipStream_t (may be null).
extern "C" int synth_fill_device(void* dst, int elem_bytes, const void* table, uint64_t key,
                                 uint64_t first_elem, uint64_t n, void* stream) {
  if (!dst || !table) return 1;
  if (n == 0) return 0;
  uint64_t want = (n + 8ull * 256 - 1) / (8ull * 256);
  unsigned grid = (unsigned)(want < 65536ull ? want : 65536ull);
  hipStream_t s = (hipStream_t)stream;
  if (elem_bytes == 2) {
    hipLaunchKernelGGL(fill_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, (uint16_t*)dst,
                       (const uint16_t*)table, key, first_elem, n);
  } else if (elem_bytes == 4) {
    hipLaunchKernelGGL(fill_kernel<uint32_t>, dim3(grid), dim3(256), 0, s, (uint32_t*)dst,
                       (const uint32_t*)table, key, first_elem, n);
  } else {
    return 2;
  }
  return hipGetLastError() == hipSuccess ? 0 : 3;
}
