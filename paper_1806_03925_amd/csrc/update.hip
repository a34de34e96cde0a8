// SGD on the touched embedding rows (Section 3, step 4: the Fastgear Worker applies the Sparse
// Part's gradients every step).
//
// The gradient of a row is the sum of dLoss/dx over the views that used it.  The views of one id
// are a segment of the stable grouping, ascending in batch position, and are summed in that order
// by one wavefront, which then writes the row once: no atomics, so the result does not depend on
// scheduling.
#include "gear_internal.hpp"

namespace gear {
namespace {

template <typename ET>
__global__ void __launch_bounds__(256)
k_embedding_update(GroupProblem users, GroupProblem urls, const float *__restrict__ dx, int F, int d,
                   ET *__restrict__ user_emb, ET *__restrict__ url_emb, float lr, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  const bool second = blockIdx.y == 1;
  const GroupProblem &g = second ? urls : users;
  ET *table = second ? url_emb : user_emb;
  const int col0 = second ? d : 0;
  const int lane = threadIdx.x & 63;
  const int n_seg = *g.n_unique;
  const int waves = gridDim.x * (blockDim.x / kWave);
  for (int seg = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave; seg < n_seg; seg += waves) {
    const int64_t id = g.unique[seg];
    const int q0 = g.segoff[seg], q1 = g.segoff[seg + 1];
    for (int c = lane; c < d; c += kWave) {
      float sum = 0.0f;
      int q = q0;
      for (; q + 4 <= q1; q += 4) {  // four rows in flight, added in order
        const float v0 = dx[(size_t)g.perm[q] * F + col0 + c];
        const float v1 = dx[(size_t)g.perm[q + 1] * F + col0 + c];
        const float v2 = dx[(size_t)g.perm[q + 2] * F + col0 + c];
        const float v3 = dx[(size_t)g.perm[q + 3] * F + col0 + c];
        sum = (((sum + v0) + v1) + v2) + v3;
      }
      for (; q < q1; ++q) sum += dx[(size_t)g.perm[q] * F + col0 + c];
      ET *cell = table + id * d + c;
      *cell = from_f32<ET>(to_f32<ET>(*cell) - lr * sum);
    }
  }
}

}  // namespace

hipError_t launch_embedding_update(const gear_config &cfg, const GroupProblem &users, const GroupProblem &urls,
                                   const float *dx, int F, void *user_emb, void *url_emb, float lr,
                                   const int32_t *status, hipStream_t s) {
  const int n = users.n > urls.n ? users.n : urls.n;
  if (n <= 0) return hipSuccess;
  int blocks = (n + 3) / 4;
  if (blocks > 4096) blocks = 4096;
  const dim3 grid(blocks, 2);
  if (cfg.emb_dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_embedding_update<bf16_t>, grid, dim3(256), 0, s, users, urls, dx, F, cfg.emb_dim,
                       (bf16_t *)user_emb, (bf16_t *)url_emb, lr, status);
  else
    hipLaunchKernelGGL(k_embedding_update<float>, grid, dim3(256), 0, s, users, urls, dx, F, cfg.emb_dim,
                       (float *)user_emb, (float *)url_emb, lr, status);
  return hipGetLastError();
}

}  // namespace gear
