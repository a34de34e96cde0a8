// Slowgear-side gradient bookkeeping and the DFV cache refresh.
//
// Section 3, step 5: every occurrence of an image in a page view yields (image id, dLoss/dDFV);
// with mean pooling that gradient is dLoss/dx of the view's DFV slot divided by the view's image
// count (Eq. 1, left factor).  Section 1, third point and Section 3, step 6: all gradients of an
// image are kept until M have arrived; their average is then handed on and collecting starts
// afresh.  Keeping the running sum of an unfinished group in grad_accum[image] is the same thing
// as keeping the gradients themselves, because only their sum is ever used.
//
// Work is cut into units of at most M rows (see the plan in group.hip), one workgroup per unit,
// rows added in arrival order (flat CSR order continuing the earlier steps): no float atomics.
#include "gear_internal.hpp"

namespace gear {
namespace {

// acc += sum over sorted positions [qa, qb) of dx[view(q)][col ..] / n_view, in order; eight rows in flight
__device__ __forceinline__ void add_rows(float4 &acc, const int32_t *__restrict__ row_view,
                                         const float *__restrict__ row_scale, const float *__restrict__ col, int F,
                                         int qa, int qb) {
  for (int q = qa; q < qb; q += 8) {
    int view[8];
    float scale[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool in = q + i < qb;
      view[i] = in ? row_view[q + i] : -1;
      scale[i] = in ? row_scale[q + i] : 0.0f;
    }
    float4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      v[i] = view[i] >= 0 ? *reinterpret_cast<const float4 *>(col + (size_t)view[i] * F) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      acc.x += v[i].x * scale[i];
      acc.y += v[i].y * scale[i];
      acc.z += v[i].z * scale[i];
      acc.w += v[i].w * scale[i];
    }
  }
}

__global__ void __launch_bounds__(256)
k_accumulate(AccumPlan plan, const float *__restrict__ dx, int F, int col0, int D, float *__restrict__ accum, int M,
             int32_t *__restrict__ ready_ids, float *__restrict__ ready_grads, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  const int n_units = *plan.n_units;
  const int D4 = D / 4;
  const float fM = (float)M;
  for (int u = blockIdx.x; u < n_units; u += gridDim.x) {
    const UnitDesc d = plan.units[u];
    float *arow = accum + (size_t)d.image * D;
    for (int c4 = threadIdx.x; c4 < D4; c4 += blockDim.x) {
      const float *col = dx + col0 + 4 * c4;
      float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
      if (d.q0 == d.s0) {
        // first group of this image in this step: continues what earlier steps left
        const int p = d.phase;
        const int len0 = min(M - p, d.s1 - d.s0);
        if (p != 0) acc = *reinterpret_cast<const float4 *>(arow + 4 * c4);
        add_rows(acc, plan.row_view, plan.row_scale, col, F, d.s0, d.s0 + len0);
        const bool complete = (p + len0 == M);
        if (complete) {
          *reinterpret_cast<float4 *>(ready_grads + (size_t)d.slot * D + 4 * c4) =
              make_float4(acc.x / fM, acc.y / fM, acc.z / fM, acc.w / fM);
          if (c4 == 0) ready_ids[d.slot] = d.image;
        }
        const int tail = (d.s1 - d.s0 - len0) % M;  // rows of the image's unfinished last group
        if (!complete) {
          *reinterpret_cast<float4 *>(arow + 4 * c4) = acc;
        } else if (tail == 0) {
          if (p != 0) *reinterpret_cast<float4 *>(arow + 4 * c4) = make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
          float4 rest = make_float4(0.f, 0.f, 0.f, 0.f);
          add_rows(rest, plan.row_view, plan.row_scale, col, F, d.s1 - tail, d.s1);
          *reinterpret_cast<float4 *>(arow + 4 * c4) = rest;
        }
      } else {
        // a complete middle group of M rows
        add_rows(acc, plan.row_view, plan.row_scale, col, F, d.q0, d.q0 + M);
        *reinterpret_cast<float4 *>(ready_grads + (size_t)d.slot * D + 4 * c4) =
            make_float4(acc.x / fM, acc.y / fM, acc.z / fM, acc.w / fM);
        if (c4 == 0) ready_ids[d.slot] = d.image;
      }
    }
  }
}

// counts[image] += occurrences of the image in this step (Section 1, third point: the number of
// gradients collected for an image)
__global__ void __launch_bounds__(256) k_count_update(GroupProblem img, int32_t *__restrict__ counts,
                                                      const int32_t *__restrict__ status) {
  if (*status != 0) return;
  const int n_seg = *img.n_unique;
  for (int s = blockIdx.x * blockDim.x + threadIdx.x; s < n_seg; s += gridDim.x * blockDim.x)
    counts[img.unique[s]] += img.segoff[s + 1] - img.segoff[s];
}

// dfv_cache[ids[r]] = rows[r]; one wavefront per row, 16-byte pieces
__global__ void __launch_bounds__(256) k_refresh(uint4 *__restrict__ cache, int64_t n_images, int vec_per_row,
                                                 const int32_t *__restrict__ ids, const uint4 *__restrict__ rows,
                                                 int64_t n, int32_t *status) {
  const int lane = threadIdx.x & 63;
  const int64_t waves = (int64_t)gridDim.x * (blockDim.x / kWave);
  for (int64_t r = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave; r < n; r += waves) {
    const int64_t id = ids ? (int64_t)ids[r] : r;
    if (id < 0 || id >= n_images) {
      if (status && lane == 0) atomicCAS(status, 0, GEAR_ERR_RANGE);
      continue;
    }
    for (int v = lane; v < vec_per_row; v += kWave) cache[id * vec_per_row + v] = rows[r * vec_per_row + v];
  }
}

}  // namespace

hipError_t launch_accumulate(const gear_config &cfg, const GroupProblem &img, const AccumPlan &plan, const float *dx,
                             int F, float *grad_accum, int32_t M, int32_t *ready_ids, float *ready_grads,
                             const int32_t *status, hipStream_t s) {
  if (img.n <= 0) return hipSuccess;
  const int D = cfg.dfv_dim;
  int threads = ((D / 4 + 63) / 64) * 64;
  if (threads > 256) threads = 256;
  int blocks = img.n < 16384 ? img.n : 16384;
  hipLaunchKernelGGL(k_accumulate, dim3(blocks), dim3(threads), 0, s, plan, dx, F, 2 * cfg.emb_dim, D, grad_accum, M,
                     ready_ids, ready_grads, status);
  return hipGetLastError();
}

hipError_t launch_count_update(const GroupProblem &img, int32_t *counts, const int32_t *status, hipStream_t s) {
  if (img.n <= 0) return hipSuccess;
  int blocks = (img.n + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(k_count_update, dim3(blocks), dim3(256), 0, s, img, counts, status);
  return hipGetLastError();
}

hipError_t launch_refresh(int dtype, void *dfv_cache, int64_t n_images, int dim, const int32_t *ids,
                          const void *rows, int64_t n, int32_t *status, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const int vec_per_row = (int)((size_t)dim * dtype_bytes(dtype) / 16);
  int64_t want = (n + 3) / 4;
  const int blocks = (int)(want < 16384 ? want : 16384);
  hipLaunchKernelGGL(k_refresh, dim3(blocks), dim3(256), 0, s, (uint4 *)dfv_cache, n_images, vec_per_row, ids,
                     (const uint4 *)rows, n, status);
  return hipGetLastError();
}

}  // namespace gear
