// Table initialisation: counter-based noise and zero fill.
//
// Section 4.1 of the paper fixes only a standard deviation for initial values.  Element idx of a
// table is Philox4x32-10 (Salmon et al., SC'11) at counter (idx_lo, idx_hi, stream, 0) under key
// (seed_lo, seed_hi); the eight 16-bit halves of the four output words are summed (an Irwin-Hall
// variate), centred by 4*65535 and scaled with one fp32 multiply.
#include "gear_internal.hpp"

#include <math.h>

namespace gear {
namespace {

struct U4 {
  uint32_t x, y, z, w;
};

__device__ __forceinline__ U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c.x;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c.z;
    U4 n;
    n.x = (uint32_t)(p1 >> 32) ^ c.y ^ k0;
    n.y = (uint32_t)p1;
    n.z = (uint32_t)(p0 >> 32) ^ c.w ^ k1;
    n.w = (uint32_t)p0;
    c = n;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c;
}

__device__ __forceinline__ float noise(uint64_t idx, uint32_t stream, uint32_t k0, uint32_t k1, float scale) {
  U4 c = {(uint32_t)idx, (uint32_t)(idx >> 32), stream, 0u};
  U4 r = philox4x32_10(c, k0, k1);
  int32_t sum = (int32_t)((r.x & 0xffffu) + (r.x >> 16) + (r.y & 0xffffu) + (r.y >> 16) + (r.z & 0xffffu) +
                          (r.z >> 16) + (r.w & 0xffffu) + (r.w >> 16));
  return (float)(sum - 4 * 65535) * scale;
}

template <typename T>
__global__ void __launch_bounds__(256) k_fill_normal(T *dst, int64_t n, uint32_t stream, uint32_t k0, uint32_t k1,
                                                     float scale) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    dst[i] = from_f32<T>(noise((uint64_t)i, stream, k0, k1, scale));
}

__global__ void __launch_bounds__(256) k_fill_zero(uint4 *dst, size_t n_vec, unsigned char *tail, size_t n_tail) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const uint4 z = {0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) dst[i] = z;
  if (blockIdx.x == 0 && threadIdx.x < n_tail) tail[threadIdx.x] = 0;
}

}  // namespace

hipError_t launch_fill_normal(void *dst, int dtype, int64_t n, uint64_t seed, uint32_t stream_id, float std,
                              hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const double var = 8.0 * (65536.0 * 65536.0 - 1.0) / 12.0;
  const float scale = (float)((double)std / sqrt(var));
  const int64_t want = (n + 255) / 256;
  const int blocks = (int)(want < 65536 ? want : 65536);
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
  if (dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_fill_normal<bf16_t>, dim3(blocks), dim3(256), 0, s, (bf16_t *)dst, n, stream_id, k0, k1, scale);
  else
    hipLaunchKernelGGL(k_fill_normal<float>, dim3(blocks), dim3(256), 0, s, (float *)dst, n, stream_id, k0, k1, scale);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void *dst, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  // dst is at least 4-byte aligned in every use; handle a non-16-byte size with a byte tail
  const size_t n_vec = bytes / 16, n_tail = bytes % 16;
  size_t want = (n_vec + 255) / 256;
  if (want == 0) want = 1;
  const int blocks = (int)(want < 65536 ? want : 65536);
  hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, s, (uint4 *)dst, n_vec,
                     (unsigned char *)dst + n_vec * 16, n_tail);
  return hipGetLastError();
}

}  // namespace gear
