// Slowgear-side gradient bookkeeping and the DFV cache refresh.
//
// Section 3, step 5: every occurrence of an image in a page view yields (image id, dLoss/dDFV);
// with mean pooling that gradient is dLoss/dx of the view's DFV slot divided by the view's image
// count (Eq. 1, left factor).  For a bf16 MLP that slot is kept in bf16 like every other delta of the
// network; sums, accumulators and emitted averages are fp32.  Section 1, third point and Section 3, step 6: all gradients of an
// image are kept until M have arrived; their average is then handed on and collecting starts
// afresh.  Keeping the running sum of an unfinished group in grad_accum[image] is the same thing
// as keeping the gradients themselves, because only their sum is ever used.
//
// Work is cut into units of at most M rows (see the plan in group.hip), one workgroup per unit,
// rows added in arrival order (flat CSR order continuing the earlier steps): no float atomics.
#include "gear_internal.hpp"

namespace gear {
namespace {

// A thread owns kCols<GT> consecutive columns: 16 bytes of a dLoss/dx row (4 fp32 or 8 bf16 values),
// kept as loaded until they are added.
template <typename GT> struct Cols;
template <> struct Cols<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void widen(const uint4 &t, float (&v)[4]) {
    v[0] = __uint_as_float(t.x), v[1] = __uint_as_float(t.y), v[2] = __uint_as_float(t.z), v[3] = __uint_as_float(t.w);
  }
};
template <> struct Cols<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void widen(const uint4 &t, float (&v)[8]) {
    v[0] = __uint_as_float(t.x << 16), v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = __uint_as_float(t.y << 16), v[3] = __uint_as_float(t.y & 0xffff0000u);
    v[4] = __uint_as_float(t.z << 16), v[5] = __uint_as_float(t.z & 0xffff0000u);
    v[6] = __uint_as_float(t.w << 16), v[7] = __uint_as_float(t.w & 0xffff0000u);
  }
};

template <int N> __device__ __forceinline__ void load_f32(const float *p, float (&v)[N]) {
#pragma unroll
  for (int k = 0; k < N; k += 4) {
    const float4 t = *reinterpret_cast<const float4 *>(p + k);
    v[k] = t.x, v[k + 1] = t.y, v[k + 2] = t.z, v[k + 3] = t.w;
  }
}
template <int N> __device__ __forceinline__ void store_f32(float *p, const float (&v)[N], float scale) {
#pragma unroll
  for (int k = 0; k < N; k += 4)
    *reinterpret_cast<float4 *>(p + k) = make_float4(v[k] * scale, v[k + 1] * scale, v[k + 2] * scale, v[k + 3] * scale);
}
template <int N> __device__ __forceinline__ void store_div(float *p, const float (&v)[N], float by) {
#pragma unroll
  for (int k = 0; k < N; k += 4)
    *reinterpret_cast<float4 *>(p + k) = make_float4(v[k] / by, v[k + 1] / by, v[k + 2] / by, v[k + 3] / by);
}

// Rows a thread has in flight.  Six keep the kernel within 48 registers per lane, so that three of
// its wavefronts (not two) fit on a SIMD beside the two of a weight-gradient product; alone on the
// device it is as fast with six as with eight.
constexpr int kRowsInFlight = 6;

// acc += sum over sorted positions [qa, qb) of dx[view(q)][col ..] / n_view, in order; kRowsInFlight rows in flight
template <typename GT>
__device__ __forceinline__ void add_rows(float (&acc)[Cols<GT>::N], const int32_t *__restrict__ row_view,
                                         const float *__restrict__ row_scale, const GT *__restrict__ col, int D,
                                         int qa, int qb) {
  constexpr int N = Cols<GT>::N;
  for (int q = qa; q < qb; q += kRowsInFlight) {
    int view[kRowsInFlight];
    float scale[kRowsInFlight];
#pragma unroll
    for (int i = 0; i < kRowsInFlight; ++i) {
      const bool in = q + i < qb;
      view[i] = in ? row_view[q + i] : -1;
      scale[i] = in ? row_scale[q + i] : 0.0f;
    }
    uint4 raw[kRowsInFlight];
#pragma unroll
    for (int i = 0; i < kRowsInFlight; ++i)
      raw[i] = view[i] >= 0 ? *reinterpret_cast<const uint4 *>(col + (size_t)view[i] * D) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int i = 0; i < kRowsInFlight; ++i) {
      float v[N];
      Cols<GT>::widen(raw[i], v);
#pragma unroll
      for (int k = 0; k < N; ++k) acc[k] += v[k] * scale[i];
    }
  }
}

// dx: the DFV slot of dLoss/dx, [B x D].  One workgroup per unit, D / Cols<GT>::N threads.
template <typename GT>
__global__ void __launch_bounds__(256)
k_accumulate(AccumPlan plan, const GT *__restrict__ dx, int D, float *__restrict__ accum, int M,
             int32_t *__restrict__ ready_ids, float *__restrict__ ready_grads, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  constexpr int N = Cols<GT>::N;
  const int n_units = *plan.n_units;
  const int DC = D / N;
  const float fM = (float)M;
  int u = blockIdx.x;
  if (u >= n_units) return;
  UnitDesc d = plan.units[u];
  while (true) {
    const int u_next = u + gridDim.x;
    UnitDesc d_next = d;
    if (u_next < n_units) d_next = plan.units[u_next];  // in flight while this unit is summed
    float *arow = accum + (size_t)d.image * D;
    for (int cg = threadIdx.x; cg < DC; cg += blockDim.x) {
      const GT *col = dx + N * cg;
      float acc[N];
#pragma unroll
      for (int k = 0; k < N; ++k) acc[k] = 0.0f;
      if (d.q0 == d.s0) {
        // first group of this image in this step: continues what earlier steps left
        const int p = d.phase;
        const int len0 = min(M - p, d.s1 - d.s0);
        if (p != 0) load_f32<N>(arow + N * cg, acc);
        add_rows<GT>(acc, plan.row_view, plan.row_scale, col, D, d.s0, d.s0 + len0);
        const bool complete = (p + len0 == M);
        if (complete) {
          store_div<N>(ready_grads + (size_t)d.slot * D + N * cg, acc, fM);
          if (cg == 0) ready_ids[d.slot] = d.image;
        }
        const int tail = (d.s1 - d.s0 - len0) % M;  // rows of the image's unfinished last group
        if (!complete) {
          store_f32<N>(arow + N * cg, acc, 1.0f);
        } else if (tail == 0) {
          if (p != 0) {
            float zero[N];
#pragma unroll
            for (int k = 0; k < N; ++k) zero[k] = 0.0f;
            store_f32<N>(arow + N * cg, zero, 1.0f);
          }
        } else {
          float rest[N];
#pragma unroll
          for (int k = 0; k < N; ++k) rest[k] = 0.0f;
          add_rows<GT>(rest, plan.row_view, plan.row_scale, col, D, d.s1 - tail, d.s1);
          store_f32<N>(arow + N * cg, rest, 1.0f);
        }
      } else {
        // a complete middle group of M rows
        add_rows<GT>(acc, plan.row_view, plan.row_scale, col, D, d.q0, d.q0 + M);
        store_div<N>(ready_grads + (size_t)d.slot * D + N * cg, acc, fM);
        if (cg == 0) ready_ids[d.slot] = d.image;
      }
    }
    if (u_next >= n_units) break;
    u = u_next;
    d = d_next;
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
                                                 int64_t n, int32_t *status, const int32_t *__restrict__ n_dev) {
  if (n_dev) n = min((int64_t)max(*n_dev, 0), n);  // the row count is only known on the device
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
                             const void *dx_dfv, float *grad_accum, int32_t M, int32_t *ready_ids,
                             float *ready_grads, const int32_t *status, hipStream_t s) {
  if (img.n <= 0) return hipSuccess;
  const int D = cfg.dfv_dim;
  const int cols = cfg.mlp_dtype == GEAR_BF16 ? 8 : 4;
  int threads = ((D / cols + 63) / 64) * 64;
  if (threads > 256) threads = 256;
  int blocks = img.n < 32768 ? img.n : 32768;
  if (cfg.mlp_dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_accumulate<bf16_t>, dim3(blocks), dim3(threads), 0, s, plan, (const bf16_t *)dx_dfv, D,
                       grad_accum, M, ready_ids, ready_grads, status);
  else
    hipLaunchKernelGGL(k_accumulate<float>, dim3(blocks), dim3(threads), 0, s, plan, (const float *)dx_dfv, D,
                       grad_accum, M, ready_ids, ready_grads, status);
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
                          const void *rows, int64_t n, int32_t *status, hipStream_t s, const int32_t *n_dev) {
  if (n <= 0) return hipSuccess;
  const int vec_per_row = (int)((size_t)dim * dtype_bytes(dtype) / 16);
  int64_t want = (n + 3) / 4;
  const int blocks = (int)(want < 16384 ? want : 16384);
  hipLaunchKernelGGL(k_refresh, dim3(blocks), dim3(256), 0, s, (uint4 *)dfv_cache, n_images, vec_per_row, ids,
                     (const uint4 *)rows, n, status, n_dev);
  return hipGetLastError();
}

}  // namespace gear
