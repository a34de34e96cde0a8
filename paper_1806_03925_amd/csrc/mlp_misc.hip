// The parts of the Sparse-Part MLP that are not matrix products: operand copies of the weights,
// the logit layer with the loss and its derivative, bias gradients and the logit layer's weight
// gradient, each followed by its SGD update (Section 3, step 4: forward to the loss,
// back-propagation on the Sparse Part, gradients applied to the Sparse Part's parameters).
#include "gear_internal.hpp"

namespace gear {
namespace {

// wc = W as MLP operands [rows x cols], wct = its transpose [cols x rows]; both from the fp32 master.
template <typename T>
__global__ void __launch_bounds__(256) k_cast_weights(const float *__restrict__ w, int rows, int cols,
                                                      T *__restrict__ wc, T *__restrict__ wct,
                                                      const int32_t *__restrict__ status) {
  if (*status != 0) return;
  __shared__ float tile[32][33];
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int rr = ty; rr < 32; rr += 8) {
    const int r = r0 + rr, c = c0 + tx;
    float v = 0.0f;
    if (r < rows && c < cols) {
      v = w[(size_t)r * cols + c];
      wc[(size_t)r * cols + c] = from_f32<T>(v);
    }
    tile[rr][tx] = v;
  }
  __syncthreads();
  for (int cc = ty; cc < 32; cc += 8) {
    const int c = c0 + cc, r = r0 + tx;
    if (r < rows && c < cols) wct[(size_t)c * rows + r] = from_f32<T>(tile[tx][cc]);
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

constexpr int kMaxVecPerLane = 4;  // a lane owns up to 4 16-byte pieces of a row: H <= 2048 (bf16) / 1024 (fp32)

// Logit layer, loss and everything that hangs on dLoss/dz.  One wavefront per view, a workgroup
// owns a contiguous range of views and its waves take them round-robin, so every sum below has a
// shape fixed by B alone:
//   z = h . w + b,  loss term,  dz = (sigmoid(z) - y) / B,
//   delta[b, j] = dz * w[j] * [h[b, j] > 0]                      (delta of the last hidden layer)
//   part_w[block][j] = sum_b dz_b h[b, j],  part_b[block] = sum_b dz_b,  part_loss[block] = sum_b loss_b
//   part_d[block][j] = sum_b delta[b, j]                         (bias gradient of the last hidden layer)
template <typename T>
__global__ void __launch_bounds__(256)
k_logit_loss(const T *__restrict__ h, const T *__restrict__ w, const float *__restrict__ bias,
             const float *__restrict__ label, int B, int H, int rows_per_block, float *__restrict__ logits,
             float *__restrict__ dz_out, T *__restrict__ delta, float *__restrict__ part_w,
             float *__restrict__ part_d, float *__restrict__ part_b, float *__restrict__ part_loss,
             const int32_t *__restrict__ status) {
  if (*status != 0) return;
  constexpr int VEC = Vec16<T>::N;
  __shared__ float s_red[4][2];
  extern __shared__ float s_w[];  // [4][H] per-wave weight-gradient sums, then [4][H] delta sums
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_vec = H / VEC;
  const float b0 = bias[0], invB = 1.0f / (float)B;

  Vec16<T> wv[kMaxVecPerLane];
  float gw[kMaxVecPerLane][VEC], gd[kMaxVecPerLane][VEC];
#pragma unroll
  for (int i = 0; i < kMaxVecPerLane; ++i) {
    const int v = lane + i * kWave;
    if (v < n_vec) wv[i].v = *reinterpret_cast<const decltype(wv[i].v) *>(w + v * VEC);
#pragma unroll
    for (int e = 0; e < VEC; ++e) gw[i][e] = gd[i][e] = 0.0f;
  }
  float loss_acc = 0.0f, dz_acc = 0.0f;
  const int r0 = blockIdx.x * rows_per_block, r1 = min(B, r0 + rows_per_block);
  for (int view = r0 + wave; view < r1; view += 4) {
    const T *hr = h + (size_t)view * H;
    Vec16<T> hv[kMaxVecPerLane];
    float dot = 0.0f;
#pragma unroll
    for (int i = 0; i < kMaxVecPerLane; ++i) {
      const int v = lane + i * kWave;
      if (v < n_vec) {
        hv[i].v = *reinterpret_cast<const decltype(hv[i].v) *>(hr + v * VEC);
#pragma unroll
        for (int e = 0; e < VEC; ++e) dot += hv[i].get(e) * wv[i].get(e);
      }
    }
    const float z = wave_sum(dot) + b0;
    const float y = label[view];
    const float ex = expf(-fabsf(z));
    const float sig = z >= 0.0f ? 1.0f / (1.0f + ex) : ex / (1.0f + ex);
    const float dz = (sig - y) * invB;
    loss_acc += fmaxf(z, 0.0f) - z * y + log1pf(ex);
    dz_acc += dz;
    if (lane == 0) {
      logits[view] = z;
      dz_out[view] = dz;
    }
    T *dr = delta + (size_t)view * H;
#pragma unroll
    for (int i = 0; i < kMaxVecPerLane; ++i) {
      const int v = lane + i * kWave;
      if (v < n_vec) {
        Vec16<T> dv = hv[i];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float hval = hv[i].get(e);
          gw[i][e] += dz * hval;
          dv.set(e, hval > 0.0f ? dz * wv[i].get(e) : 0.0f);
          gd[i][e] += dv.get(e);  // the stored (rounded) value
        }
        *reinterpret_cast<decltype(dv.v) *>(dr + v * VEC) = dv.v;
      }
    }
  }
  // combine the four waves in wave order
#pragma unroll
  for (int i = 0; i < kMaxVecPerLane; ++i) {
    const int v = lane + i * kWave;
    if (v < n_vec)
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        s_w[wave * H + v * VEC + e] = gw[i][e];
        s_w[(4 + wave) * H + v * VEC + e] = gd[i][e];
      }
  }
  if (lane == 0) {
    s_red[wave][0] = loss_acc;
    s_red[wave][1] = dz_acc;
  }
  __syncthreads();
  for (int j = threadIdx.x; j < H; j += blockDim.x) {
    part_w[(size_t)blockIdx.x * H + j] = ((s_w[j] + s_w[H + j]) + s_w[2 * H + j]) + s_w[3 * H + j];
    part_d[(size_t)blockIdx.x * H + j] = ((s_w[4 * H + j] + s_w[5 * H + j]) + s_w[6 * H + j]) + s_w[7 * H + j];
  }
  if (threadIdx.x == 0) {
    part_loss[blockIdx.x] = ((s_red[0][0] + s_red[1][0]) + s_red[2][0]) + s_red[3][0];
    part_b[blockIdx.x] = ((s_red[0][1] + s_red[1][1]) + s_red[2][1]) + s_red[3][1];
  }
}

__global__ void __launch_bounds__(64) k_loss_final(const float *__restrict__ loss_partial, int n, int B,
                                                   float *__restrict__ loss, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  float part[kLossBlocks / kWave];
#pragma unroll
  for (int k = 0; k < kLossBlocks / kWave; ++k) {
    const int i = threadIdx.x + k * kWave;
    part[k] = i < n ? loss_partial[i] : 0.0f;
  }
  float v = 0.0f;
#pragma unroll
  for (int k = 0; k < kLossBlocks / kWave; ++k) v += part[k];
  v = wave_sum(v);
  if (threadIdx.x == 0) *loss = v / (float)B;
}

// partial[chunk][j] = sum over the chunk's rows of src[row][j].  A thread owns one 16-byte piece of
// the row and every RS-th row of the chunk; the RS row-lanes are then added in order.
template <typename T>
__global__ void __launch_bounds__(256)
k_colsum_partial(const T *__restrict__ src, int B, int H, int rows_per_chunk, float *__restrict__ partial,
                 const int32_t *__restrict__ status) {
  if (*status != 0) return;
  constexpr int VEC = Vec16<T>::N;
  extern __shared__ float s_part[];  // [RS][cols of this block]
  const int n_vec = H / VEC;
  const int vec_here = min(n_vec - (int)blockIdx.x * 256, 256);  // column pieces handled by this block
  const int RS = 256 / vec_here;                                  // row lanes
  const int cv = threadIdx.x % vec_here, rl = threadIdx.x / vec_here;
  const int col = (blockIdx.x * 256 + cv) * VEC;
  const int r0 = blockIdx.y * rows_per_chunk, r1 = min(B, r0 + rows_per_chunk);
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
  if (rl < RS) {
    for (int r = r0 + rl; r < r1; r += RS) {
      Vec16<T> v;
      v.v = *reinterpret_cast<const decltype(v.v) *>(src + (size_t)r * H + col);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] += v.get(e);
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) s_part[(rl * vec_here + cv) * VEC + e] = acc[e];
  }
  __syncthreads();
  for (int j = threadIdx.x; j < vec_here * VEC; j += blockDim.x) {
    float t = 0.0f;
    for (int k = 0; k < RS; ++k) t += s_part[k * vec_here * VEC + j];
    partial[(size_t)blockIdx.y * H + blockIdx.x * 256 * VEC + j] = t;
  }
}

// dst[j] -= lr * sum_p partial[p][j].  Eight columns per workgroup and 32 row lanes, each adding
// every 32nd partial in order (eight loads in flight); then the 32 lanes are added in order.
__global__ void __launch_bounds__(256) k_partial_sgd(const float *__restrict__ partial, int P, int H,
                                                     float *__restrict__ dst, float lr,
                                                     const int32_t *__restrict__ status) {
  if (*status != 0) return;
  __shared__ float s[32][8];
  const int c = threadIdx.x & 7, g = threadIdx.x >> 3;
  const int j = blockIdx.x * 8 + c;
  float acc = 0.0f;
  if (j < H) {
    int p = g;
    for (; p + 32 * 7 < P; p += 32 * 8) {
      float v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = partial[(size_t)(p + 32 * i) * H + j];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc += v[i];
    }
    for (; p < P; p += 32) acc += partial[(size_t)p * H + j];
  }
  s[g][c] = acc;
  __syncthreads();
  if (g == 0 && j < H) {
    float t = 0.0f;
#pragma unroll
    for (int k = 0; k < 32; ++k) t += s[k][c];
    dst[j] -= lr * t;
  }
}

}  // namespace

hipError_t launch_cast_weights(const float *w, int rows, int cols, int dtype, void *wc, void *wct,
                               const int32_t *status, hipStream_t s) {
  const dim3 grid((cols + 31) / 32, (rows + 31) / 32);
  if (dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_cast_weights<bf16_t>, grid, dim3(256), 0, s, w, rows, cols, (bf16_t *)wc, (bf16_t *)wct, status);
  else
    hipLaunchKernelGGL(k_cast_weights<float>, grid, dim3(256), 0, s, w, rows, cols, (float *)wc, (float *)wct, status);
  return hipGetLastError();
}

int logit_blocks(int B) {
  int blocks = (B + 31) / 32;
  return blocks < 1 ? 1 : (blocks > kLossBlocks ? kLossBlocks : blocks);
}

// Forward logit + loss + delta of the last hidden layer, then SGD on the logit layer's weight and bias.
hipError_t launch_logit_loss(int dtype, const void *h, const void *wc_last, float *w_last, float *bias_last,
                             float *bias_hidden, const float *label, int B, int H, float *logits, float *dz,
                             void *delta, float *partials, float *loss, float lr, const int32_t *status,
                             hipStream_t s) {
  if (B <= 0) return hipSuccess;
  const int blocks = logit_blocks(B);
  const int rows_per_block = (B + blocks - 1) / blocks;
  float *part_w = partials, *part_d = part_w + (size_t)kLossBlocks * H, *part_b = part_d + (size_t)kLossBlocks * H,
        *part_loss = part_b + kLossBlocks;
  const size_t smem = 8 * (size_t)H * sizeof(float);
  if (dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_logit_loss<bf16_t>, dim3(blocks), dim3(256), smem, s, (const bf16_t *)h,
                       (const bf16_t *)wc_last, bias_last, label, B, H, rows_per_block, logits, dz, (bf16_t *)delta,
                       part_w, part_d, part_b, part_loss, status);
  else
    hipLaunchKernelGGL(k_logit_loss<float>, dim3(blocks), dim3(256), smem, s, (const float *)h,
                       (const float *)wc_last, bias_last, label, B, H, rows_per_block, logits, dz, (float *)delta,
                       part_w, part_d, part_b, part_loss, status);
  hipLaunchKernelGGL(k_loss_final, dim3(1), dim3(64), 0, s, part_loss, blocks, B, loss, status);
  hipLaunchKernelGGL(k_partial_sgd, dim3((H + 7) / 8), dim3(256), 0, s, part_w, blocks, H, w_last, lr, status);
  hipLaunchKernelGGL(k_partial_sgd, dim3(1), dim3(256), 0, s, part_b, blocks, 1, bias_last, lr, status);
  hipLaunchKernelGGL(k_partial_sgd, dim3((H + 7) / 8), dim3(256), 0, s, part_d, blocks, H, bias_hidden, lr, status);
  return hipGetLastError();
}

size_t logit_partial_floats(int H) { return 2 * (size_t)kLossBlocks * H + 2 * (size_t)kLossBlocks; }

hipError_t launch_partial_sgd(const float *partial, int P, int H, float *dst, float lr, const int32_t *status,
                              hipStream_t s) {
  if (P <= 0 || H <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_partial_sgd, dim3((H + 7) / 8), dim3(256), 0, s, partial, P, H, dst, lr, status);
  return hipGetLastError();
}

// dst[j] -= lr * sum_b src[b][j]   (bias gradient of a hidden layer)
hipError_t launch_colsum_sgd(int dtype, const void *src, int B, int H, float *partial, float *dst, float lr,
                             const int32_t *status, hipStream_t s) {
  if (B <= 0 || H <= 0) return hipSuccess;
  const int chunks = (B + kColsumRows - 1) / kColsumRows;
  const int vec = dtype == GEAR_BF16 ? 8 : 4;
  const int n_vec = H / vec;
  const dim3 grid((n_vec + 255) / 256, chunks);
  const size_t smem = 256 * (size_t)vec * sizeof(float);
  if (dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_colsum_partial<bf16_t>, grid, dim3(256), smem, s, (const bf16_t *)src, B, H, kColsumRows,
                       partial, status);
  else
    hipLaunchKernelGGL(k_colsum_partial<float>, grid, dim3(256), smem, s, (const float *)src, B, H, kColsumRows,
                       partial, status);
  hipLaunchKernelGGL(k_partial_sgd, dim3((H + 7) / 8), dim3(256), 0, s, partial, chunks, H, dst, lr, status);
  return hipGetLastError();
}

}  // namespace gear
