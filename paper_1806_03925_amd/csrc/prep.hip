// Step prologue: reset the per-step outputs and check what only the device can see.
//
// A page view is a user id, a URL bucket and a list of image ids (Section 1, Table 1).  Every id
// later indexes a table, so a bad id must be caught before any kernel dereferences it: the first
// violation found is written to the status word and every later kernel of the step returns at
// once when that word is not zero.
#include "gear_internal.hpp"

namespace gear {
namespace {

__global__ void k_begin(int32_t *status, int32_t *n_ready, float *loss) {
  if (threadIdx.x == 0) {
    *status = 0;
    *n_ready = 0;
    *loss = 0.0f;
  }
}

__device__ __forceinline__ void flag(int32_t *status, int code) { atomicCAS(status, 0, code); }

// One thread per view (and per occurrence).  Also expands the CSR offsets into occ_view[j] = the
// view that owns occurrence j, which the accumulation uses to find dLoss/dx of an occurrence.
__global__ void __launch_bounds__(256) k_validate(int B, int nnz, const int32_t *user_id, const int32_t *url_id,
                                                  const int32_t *img_off, const int32_t *img_id, int64_t n_users,
                                                  int64_t n_urls, int64_t n_images, int32_t *occ_view,
                                                  int32_t *status) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B) {
    const int32_t u = user_id[i], v = url_id[i];
    if (u < 0 || (int64_t)u >= n_users || v < 0 || (int64_t)v >= n_urls) flag(status, GEAR_ERR_RANGE);
    const int32_t lo = img_off[i], hi = img_off[i + 1];
    const bool ok = lo >= 0 && lo <= hi && hi <= nnz;
    if (!ok) flag(status, GEAR_ERR_RANGE);
    if (i == 0 && lo != 0) flag(status, GEAR_ERR_RANGE);
    if (i == B - 1 && hi != nnz) flag(status, GEAR_ERR_RANGE);
    if (ok)
      for (int j = lo; j < hi; ++j) occ_view[j] = i;
  }
  if (i < nnz) {
    const int32_t g = img_id[i];
    if (g < 0 || (int64_t)g >= n_images) flag(status, GEAR_ERR_RANGE);
  }
}

}  // namespace

hipError_t launch_begin(int32_t *status, int32_t *n_ready, float *loss, hipStream_t s) {
  hipLaunchKernelGGL(k_begin, dim3(1), dim3(64), 0, s, status, n_ready, loss);
  return hipGetLastError();
}

hipError_t launch_validate(const gear_config &cfg, const gear_batch &b, int32_t *occ_view, int32_t *status,
                           hipStream_t s) {
  const int n = b.B > b.nnz ? b.B : b.nnz;
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_validate, dim3((n + 255) / 256), dim3(256), 0, s, b.B, b.nnz, b.user_id, b.url_id, b.img_off,
                     b.img_id, cfg.n_users, cfg.n_urls, cfg.n_images, occ_view, status);
  return hipGetLastError();
}

}  // namespace gear
