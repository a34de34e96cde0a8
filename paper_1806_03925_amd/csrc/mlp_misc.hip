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

// One wavefront per view: logit z = h . w + b, loss term, dLoss/dz = (sigmoid(z) - y) / B, and the
// delta of the last hidden layer, delta[b, j] = dz * w[j] * [h[b, j] > 0].  Each workgroup keeps a
// running loss sum over its views in a fixed order and leaves it in loss_partial[blockIdx].
template <typename T>
__global__ void __launch_bounds__(256)
k_logit_loss(const T *__restrict__ h, const T *__restrict__ w, const float *__restrict__ bias,
             const float *__restrict__ label, int B, int H, float *__restrict__ logits, float *__restrict__ dz_out,
             T *__restrict__ delta, float *__restrict__ loss_partial, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  __shared__ float wave_loss[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float b0 = bias[0], invB = 1.0f / (float)B;
  float loss_acc = 0.0f;
  for (int view = blockIdx.x * 4 + wave; view < B; view += gridDim.x * 4) {
    const T *hr = h + (size_t)view * H;
    float dot = 0.0f;
    for (int j = lane; j < H; j += kWave) dot += to_f32<T>(hr[j]) * to_f32<T>(w[j]);
    const float z = wave_sum(dot) + b0;
    const float y = label[view];
    const float e = expf(-fabsf(z));
    const float sig = z >= 0.0f ? 1.0f / (1.0f + e) : e / (1.0f + e);
    const float dz = (sig - y) * invB;
    loss_acc += fmaxf(z, 0.0f) - z * y + log1pf(e);
    if (lane == 0) {
      logits[view] = z;
      dz_out[view] = dz;
    }
    T *dr = delta + (size_t)view * H;
    for (int j = lane; j < H; j += kWave) dr[j] = from_f32<T>(to_f32<T>(hr[j]) > 0.0f ? dz * to_f32<T>(w[j]) : 0.0f);
  }
  if (lane == 0) wave_loss[wave] = loss_acc;
  __syncthreads();
  if (threadIdx.x == 0) loss_partial[blockIdx.x] = ((wave_loss[0] + wave_loss[1]) + wave_loss[2]) + wave_loss[3];
}

__global__ void __launch_bounds__(64) k_loss_final(const float *__restrict__ loss_partial, int n, int B,
                                                   float *__restrict__ loss, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  float v = 0.0f;
  for (int i = threadIdx.x; i < n; i += kWave) v += loss_partial[i];
  v = wave_sum(v);
  if (threadIdx.x == 0) *loss = v / (float)B;
}

// partial[chunk][j] = sum over the chunk's rows (ascending) of weight[row] * src[row][j]
template <typename T>
__global__ void __launch_bounds__(256)
k_colsum_partial(const T *__restrict__ src, const float *__restrict__ row_weight, int B, int H,
                 float *__restrict__ partial, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= H) return;
  const int r0 = blockIdx.y * kColsumRows, r1 = min(B, r0 + kColsumRows);
  float acc = 0.0f;
  if (row_weight) {
    for (int r = r0; r < r1; ++r) acc += row_weight[r] * to_f32<T>(src[(size_t)r * H + j]);
  } else {
    for (int r = r0; r < r1; ++r) acc += to_f32<T>(src[(size_t)r * H + j]);
  }
  partial[(size_t)blockIdx.y * H + j] = acc;
}

// dst[j] -= lr * sum_chunk partial[chunk][j], chunks ascending
__global__ void __launch_bounds__(256) k_colsum_sgd(const float *__restrict__ partial, int chunks, int H,
                                                    float *__restrict__ dst, float lr,
                                                    const int32_t *__restrict__ status) {
  if (*status != 0) return;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= H) return;
  float g = 0.0f;
  for (int c = 0; c < chunks; ++c) g += partial[(size_t)c * H + j];
  dst[j] -= lr * g;
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

hipError_t launch_logit_loss(int dtype, const void *h, const void *wc_last, const float *bias_last,
                             const float *label, int B, int H, float *logits, float *dz, void *delta,
                             float *loss_partial, float *loss, const int32_t *status, hipStream_t s) {
  if (B <= 0) return hipSuccess;
  if (dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_logit_loss<bf16_t>, dim3(kLossBlocks), dim3(256), 0, s, (const bf16_t *)h,
                       (const bf16_t *)wc_last, bias_last, label, B, H, logits, dz, (bf16_t *)delta, loss_partial,
                       status);
  else
    hipLaunchKernelGGL(k_logit_loss<float>, dim3(kLossBlocks), dim3(256), 0, s, (const float *)h,
                       (const float *)wc_last, bias_last, label, B, H, logits, dz, (float *)delta, loss_partial,
                       status);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_loss_final, dim3(1), dim3(64), 0, s, loss_partial, kLossBlocks, B, loss, status);
  return hipGetLastError();
}

hipError_t launch_colsum_sgd(int dtype, const void *src, const float *row_weight, int B, int H, float *partial,
                             float *dst, float lr, const int32_t *status, hipStream_t s) {
  if (B <= 0 || H <= 0) return hipSuccess;
  const int chunks = (B + kColsumRows - 1) / kColsumRows;
  const int bs = H >= 256 ? 256 : 64;
  const dim3 grid((H + bs - 1) / bs, chunks);
  if (dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_colsum_partial<bf16_t>, grid, dim3(bs), 0, s, (const bf16_t *)src, row_weight, B, H, partial,
                       status);
  else
    hipLaunchKernelGGL(k_colsum_partial<float>, grid, dim3(bs), 0, s, (const float *)src, row_weight, B, H, partial,
                       status);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_colsum_sgd, dim3((H + 255) / 256), dim3(256), 0, s, partial, chunks, H, dst, lr, status);
  return hipGetLastError();
}

}  // namespace gear
