// A stand-in Dense Part: DFV[i] = Wd raw[i], a linear map from fixed per-image features to the Dense
// Feature Vector.  It closes the loop the paper describes: the Slowgear Worker runs inference to fill
// the DFV cache (Section 3, steps 1-2) and, when an image has collected M gradients, back-propagates
// their average through the Dense Part (Section 3, step 6; Eq. 1, right factor):
//   dLoss/dWd = sum over emissions e of  g_e (outer) raw[id_e],   Wd -= lr * dLoss/dWd.
// One SGD step per emission, taken in ready-list order, adds up to exactly this sum because the
// averaged gradients were formed before any of the steps.  Both directions are dense contractions
// and run on the fp32 matrix-core kernels; everything is fp32 except the rows handed to the cache.
#include "gear_internal.hpp"

#include <cmath>

namespace gear {
namespace {

// out[r] = raw[ids[r]] (ids == NULL: raw[r]); one wavefront per row, 16-byte pieces
__global__ void __launch_bounds__(256) k_gather_raw(const float4 *__restrict__ raw, int64_t n_images, int vec_per_row,
                                                    const int32_t *__restrict__ ids, int n, float4 *__restrict__ out,
                                                    int32_t *status, const int32_t *__restrict__ n_dev) {
  if (n_dev) n = min(max(*n_dev, 0), n);  // the row count is only known on the device
  const int lane = threadIdx.x & 63;
  const int waves = gridDim.x * (blockDim.x / kWave);
  for (int r = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave; r < n; r += waves) {
    int64_t id = ids ? (int64_t)ids[r] : r;
    if (id < 0 || id >= n_images) {
      if (lane == 0) atomicCAS(status, 0, GEAR_ERR_RANGE);
      id = 0;  // a valid row keeps the product defined; the status word tells the caller
    }
    for (int v = lane; v < vec_per_row; v += kWave) out[(size_t)r * vec_per_row + v] = raw[id * vec_per_row + v];
  }
}

// rows of fp32 values -> the cache's type
template <typename T>
__global__ void __launch_bounds__(256) k_rows_to(const float4 *__restrict__ src, size_t n_vec, T *__restrict__ dst) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * blockDim.x) {
    const float4 v = src[i];
    if constexpr (sizeof(T) == 4) {
      reinterpret_cast<float4 *>(dst)[i] = v;
    } else {
      reinterpret_cast<uint2 *>(dst)[i] = make_uint2(pack_bf16(v.x, v.y), pack_bf16(v.z, v.w));
    }
  }
}

struct DenseLayout {
  size_t rows, out32, partial, total;
  int splits;
};

bool dense_ok(const gear_dense_config &c) {
  return c.n_images >= 1 && c.n_images <= INT32_MAX && c.raw_dim >= 8 && c.raw_dim % 8 == 0 && c.dfv_dim >= 8 &&
         c.dfv_dim % 8 == 0 && c.max_rows >= 1 && (c.dfv_dtype == GEAR_F32 || c.dfv_dtype == GEAR_BF16);
}

constexpr int kDenseSplits = 16;

DenseLayout dense_layout(const gear_dense_config &c) {
  auto up = [](size_t b) { return (b + 255) & ~(size_t)255; };
  DenseLayout l;
  size_t cur = 0;
  l.rows = cur, cur += up((size_t)c.max_rows * c.raw_dim * 4);
  l.out32 = cur, cur += up((size_t)c.max_rows * c.dfv_dim * 4);
  l.partial = cur, cur += up((size_t)kDenseSplits * c.dfv_dim * c.raw_dim * 4);
  l.total = cur;
  l.splits = kDenseSplits;
  return l;
}

#define DENSE_HIP(expr)                       \
  do {                                        \
    if ((expr) != hipSuccess) return GEAR_ERR_HIP; \
  } while (0)

hipError_t gather_raw(const gear_dense_config &c, const float *raw, const int32_t *ids, int n, float *out,
                      int32_t *status, hipStream_t s, const int32_t *n_dev = nullptr) {
  int blocks = (n + 3) / 4;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(k_gather_raw, dim3(blocks), dim3(256), 0, s, (const float4 *)raw, c.n_images, c.raw_dim / 4, ids, n,
                     (float4 *)out, status, n_dev);
  return hipGetLastError();
}

}  // namespace
}  // namespace gear

using namespace gear;

extern "C" size_t gear_dense_workspace_bytes(const gear_dense_config *cfg) {
  return cfg && dense_ok(*cfg) ? dense_layout(*cfg).total : 0;
}

extern "C" gear_status gear_dense_infer(const gear_dense_config *cfg, const float *raw, const float *wd,
                                        const int32_t *image_ids, int32_t n, void *out_rows, void *workspace,
                                        size_t workspace_bytes, int32_t *status, void *stream) {
  if (!cfg || !dense_ok(*cfg) || !raw || !wd || !out_rows || !workspace || !status || n < 0 || n > cfg->max_rows)
    return GEAR_ERR_INVALID;
  if (!image_ids && n > cfg->n_images) return GEAR_ERR_INVALID;
  if (((uintptr_t)workspace & 255) || ((uintptr_t)raw & 15) || ((uintptr_t)wd & 15) || ((uintptr_t)out_rows & 15))
    return GEAR_ERR_INVALID;
  const DenseLayout lay = dense_layout(*cfg);
  if (workspace_bytes < lay.total) return GEAR_ERR_CAPACITY;
  hipStream_t s = (hipStream_t)stream;
  DENSE_HIP(launch_fill_zero(status, sizeof(int32_t), s));
  if (n == 0) return GEAR_OK;
  char *ws = (char *)workspace;
  float *rows = (float *)(ws + lay.rows), *out32 = (float *)(ws + lay.out32);
  DENSE_HIP(gather_raw(*cfg, raw, image_ids, n, rows, status, s));
  // out32 [n x D] = rows [n x r] * Wd [D x r]^T; the product kernel itself looks at the status word only to
  // stay idle after an earlier failure of a step, which does not apply here, so it runs on a zero word
  int32_t *zero = (int32_t *)(ws + lay.partial);
  DENSE_HIP(launch_fill_zero(zero, sizeof(int32_t), s));
  DENSE_HIP(launch_gemm_nt(GEAR_F32, rows, wd, n, cfg->dfv_dim, cfg->raw_dim, EPI_F32, nullptr, nullptr, out32, 0,
                           nullptr, nullptr, zero, s));
  const size_t n_vec = (size_t)n * cfg->dfv_dim / 4;
  const int blocks = (int)((n_vec + 255) / 256 < 16384 ? (n_vec + 255) / 256 : 16384);
  if (cfg->dfv_dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_rows_to<bf16_t>, dim3(blocks), dim3(256), 0, s, (const float4 *)out32, n_vec, (bf16_t *)out_rows);
  else
    hipLaunchKernelGGL(k_rows_to<float>, dim3(blocks), dim3(256), 0, s, (const float4 *)out32, n_vec, (float *)out_rows);
  DENSE_HIP(hipGetLastError());
  return GEAR_OK;
}

namespace {
// n_dev == NULL: n_ready emissions; otherwise up to n_ready, the real number read on the device
gear_status dense_backward(const gear_dense_config *cfg, const float *raw, float *wd, const int32_t *ready_ids,
                           const float *ready_grads, int32_t n_ready, const int32_t *n_dev, float lr, void *workspace,
                           size_t workspace_bytes, int32_t *status, void *stream) {
  if (!cfg || !dense_ok(*cfg) || !raw || !wd || !workspace || !status || n_ready < 0 || n_ready > cfg->max_rows ||
      !std::isfinite(lr))
    return GEAR_ERR_INVALID;
  if (n_ready > 0 && (!ready_ids || !ready_grads)) return GEAR_ERR_INVALID;
  if (((uintptr_t)workspace & 255) || ((uintptr_t)raw & 15) || ((uintptr_t)wd & 15) || ((uintptr_t)ready_grads & 15))
    return GEAR_ERR_INVALID;
  const DenseLayout lay = dense_layout(*cfg);
  if (workspace_bytes < lay.total) return GEAR_ERR_CAPACITY;
  hipStream_t s = (hipStream_t)stream;
  DENSE_HIP(launch_fill_zero(status, sizeof(int32_t), s));
  if (n_ready == 0) return GEAR_OK;
  char *ws = (char *)workspace;
  float *rows = (float *)(ws + lay.rows), *partial = (float *)(ws + lay.partial);
  DENSE_HIP(gather_raw(*cfg, raw, ready_ids, n_ready, rows, status, s, n_dev));
  // dWd [D x r] = ready_grads [n x D]^T * rows [n x r], split over the emissions in a fixed shape; an id out
  // of range leaves the status word set and the weights untouched (both kernels below then stay idle)
  int splits = n_dev ? lay.splits : (n_ready + 255) / 256;
  if (splits > lay.splits) splits = lay.splits;
  DENSE_HIP(launch_gemm_tn_splitk(GEAR_F32, ready_grads, rows, cfg->dfv_dim, cfg->raw_dim, n_ready, splits, partial,
                                  status, s, n_dev));
  const Optim sgd = {lr, 0.0f, 0.0f, 0.0f, 1.0f, 0};
  const Moments none = {nullptr, nullptr};
  DENSE_HIP(launch_splitk_sgd(partial, splits, (int64_t)cfg->dfv_dim * cfg->raw_dim, wd, sgd, none, status, s));
  return GEAR_OK;
}
}  // namespace

extern "C" gear_status gear_dense_backward(const gear_dense_config *cfg, const float *raw, float *wd,
                                           const int32_t *ready_ids, const float *ready_grads, int32_t n_ready,
                                           float lr, void *workspace, size_t workspace_bytes, int32_t *status,
                                           void *stream) {
  return dense_backward(cfg, raw, wd, ready_ids, ready_grads, n_ready, nullptr, lr, workspace, workspace_bytes, status,
                        stream);
}

extern "C" gear_status gear_dense_backward_n(const gear_dense_config *cfg, const float *raw, float *wd,
                                             const int32_t *ready_ids, const float *ready_grads,
                                             const int32_t *n_ready, float lr, void *workspace, size_t workspace_bytes,
                                             int32_t *status, void *stream) {
  if (!cfg || !n_ready) return GEAR_ERR_INVALID;
  return dense_backward(cfg, raw, wd, ready_ids, ready_grads, cfg->max_rows, n_ready, lr, workspace, workspace_bytes,
                        status, stream);
}
