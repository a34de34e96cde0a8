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

constexpr int kRowBatch = 256;

struct RowSum {
  const int32_t *perm, *occ_view, *img_off;
  const float *dx;
  int F, col0;
  int *s_view;
  float *s_inv;
};

// acc += sum over sorted positions [qa, qb) of dx[view(q)][col0 + 4 c4 ..] / n_view, in order.
// Called by the whole workgroup (contains barriers); `active` lanes own a column group.
__device__ __forceinline__ void add_rows(float4 &acc, const RowSum &rs, int qa, int qb, int c4, bool active) {
  for (int base = qa; base < qb; base += kRowBatch) {
    const int cnt = min(kRowBatch, qb - base);
    __syncthreads();
    for (int t = threadIdx.x; t < cnt; t += blockDim.x) {
      const int view = rs.occ_view[rs.perm[base + t]];
      rs.s_view[t] = view;
      rs.s_inv[t] = 1.0f / (float)(rs.img_off[view + 1] - rs.img_off[view]);
    }
    __syncthreads();
    if (!active) continue;
    const float *col = rs.dx + rs.col0 + 4 * c4;
    int r = 0;
    for (; r + 4 <= cnt; r += 4) {
      const float4 v0 = *reinterpret_cast<const float4 *>(col + (size_t)rs.s_view[r] * rs.F);
      const float4 v1 = *reinterpret_cast<const float4 *>(col + (size_t)rs.s_view[r + 1] * rs.F);
      const float4 v2 = *reinterpret_cast<const float4 *>(col + (size_t)rs.s_view[r + 2] * rs.F);
      const float4 v3 = *reinterpret_cast<const float4 *>(col + (size_t)rs.s_view[r + 3] * rs.F);
      const float i0 = rs.s_inv[r], i1 = rs.s_inv[r + 1], i2 = rs.s_inv[r + 2], i3 = rs.s_inv[r + 3];
      acc.x = (((acc.x + v0.x * i0) + v1.x * i1) + v2.x * i2) + v3.x * i3;
      acc.y = (((acc.y + v0.y * i0) + v1.y * i1) + v2.y * i2) + v3.y * i3;
      acc.z = (((acc.z + v0.z * i0) + v1.z * i1) + v2.z * i2) + v3.z * i3;
      acc.w = (((acc.w + v0.w * i0) + v1.w * i1) + v2.w * i2) + v3.w * i3;
    }
    for (; r < cnt; ++r) {
      const float4 v0 = *reinterpret_cast<const float4 *>(col + (size_t)rs.s_view[r] * rs.F);
      const float i0 = rs.s_inv[r];
      acc.x += v0.x * i0;
      acc.y += v0.y * i0;
      acc.z += v0.z * i0;
      acc.w += v0.w * i0;
    }
  }
}

__global__ void __launch_bounds__(256)
k_accumulate(GroupProblem img, AccumPlan plan, const int32_t *__restrict__ occ_view,
             const int32_t *__restrict__ img_off, const float *__restrict__ dx, int F, int col0, int D,
             float *__restrict__ accum, const int32_t *__restrict__ counts, int M, int32_t *__restrict__ ready_ids,
             float *__restrict__ ready_grads, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  __shared__ int s_view[kRowBatch];
  __shared__ float s_inv[kRowBatch];
  const RowSum rs = {img.perm, occ_view, img_off, dx, F, col0, s_view, s_inv};
  const int n_units = *plan.n_units;
  const int D4 = D / 4;
  const float fM = (float)M;
  for (int u = blockIdx.x; u < n_units; u += gridDim.x) {
    const int q0 = plan.unit_q0[u], seg = plan.unit_seg[u], slot = plan.unit_slot[u];
    const int image = img.unique[seg];
    const int s0 = img.segoff[seg], s1 = img.segoff[seg + 1];
    float *arow = accum + (size_t)image * D;
    for (int cbase = 0; cbase < D4; cbase += blockDim.x) {
      const int c4 = cbase + threadIdx.x;
      const bool active = c4 < D4;
      float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
      if (q0 == s0) {
        // first group of this image in this step: continues what earlier steps left
        const int p = counts[image] % M;
        const int len0 = min(M - p, s1 - s0);
        if (p != 0 && active) acc = *reinterpret_cast<const float4 *>(arow + 4 * c4);
        add_rows(acc, rs, s0, s0 + len0, c4, active);
        const bool complete = (p + len0 == M);
        if (complete && active) {
          *reinterpret_cast<float4 *>(ready_grads + (size_t)slot * D + 4 * c4) =
              make_float4(acc.x / fM, acc.y / fM, acc.z / fM, acc.w / fM);
          if (c4 == 0) ready_ids[slot] = image;
        }
        const int tail = (s1 - s0 - len0) % M;  // rows of the image's unfinished last group
        if (!complete) {
          if (active) *reinterpret_cast<float4 *>(arow + 4 * c4) = acc;
        } else if (tail == 0) {
          if (p != 0 && active) *reinterpret_cast<float4 *>(arow + 4 * c4) = make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
          float4 rest = make_float4(0.f, 0.f, 0.f, 0.f);
          add_rows(rest, rs, s1 - tail, s1, c4, active);
          if (active) *reinterpret_cast<float4 *>(arow + 4 * c4) = rest;
        }
      } else {
        // a complete middle group of M rows
        add_rows(acc, rs, q0, q0 + M, c4, active);
        if (active) {
          *reinterpret_cast<float4 *>(ready_grads + (size_t)slot * D + 4 * c4) =
              make_float4(acc.x / fM, acc.y / fM, acc.z / fM, acc.w / fM);
          if (c4 == 0) ready_ids[slot] = image;
        }
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

hipError_t launch_accumulate(const gear_config &cfg, const GroupProblem &img, const AccumPlan &plan,
                             const int32_t *occ_view, const int32_t *img_off, const float *dx, int F,
                             float *grad_accum, const int32_t *counts, int32_t M, int32_t *ready_ids,
                             float *ready_grads, const int32_t *status, hipStream_t s) {
  if (img.n <= 0) return hipSuccess;
  const int D = cfg.dfv_dim;
  int threads = ((D / 4 + 63) / 64) * 64;
  if (threads > 256) threads = 256;
  int blocks = img.n < 8192 ? img.n : 8192;
  hipLaunchKernelGGL(k_accumulate, dim3(blocks), dim3(threads), 0, s, img, plan, occ_view, img_off, dx, F,
                     2 * cfg.emb_dim, D, grad_accum, counts, M, ready_ids, ready_grads, status);
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
