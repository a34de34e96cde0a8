// The parts of the Sparse-Part MLP that are not matrix products: operand copies of the weights,
// the logit layer with the loss and its derivative, bias gradients and the logit layer's weight
// gradient, each followed by its SGD update (Section 3, step 4: forward to the loss,
// back-propagation on the Sparse Part, gradients applied to the Sparse Part's parameters).
#include "gear_internal.hpp"

namespace gear {
namespace {

// wc = W as MLP operands [rows x cols], wct = its transpose [cols x rows]; both from the fp32 master.
// One launch serves all layers: a workgroup owns a 32 x 32 tile of one of them.
struct CastArgs {
  int count;
  const float *w[GEAR_MAX_LAYERS];
  void *wc[GEAR_MAX_LAYERS], *wct[GEAR_MAX_LAYERS];
  int rows[GEAR_MAX_LAYERS], cols[GEAR_MAX_LAYERS], first_block[GEAR_MAX_LAYERS];
};

template <typename T>
__global__ void __launch_bounds__(256) k_cast_weights(CastArgs args, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  __shared__ float tile[32][33];
  int which = 0;
  for (int i = 1; i < args.count; ++i)
    if ((int)blockIdx.x >= args.first_block[i]) which = i;
  const int rows = args.rows[which], cols = args.cols[which];
  const float *__restrict__ w = args.w[which];
  T *__restrict__ wc = static_cast<T *>(args.wc[which]);
  T *__restrict__ wct = static_cast<T *>(args.wct[which]);
  const int local = blockIdx.x - args.first_block[which], col_tiles = (cols + 31) / 32;
  const int c0 = (local % col_tiles) * 32, r0 = (local / col_tiles) * 32;
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


// Logit layer, loss and everything that hangs on dLoss/dz.  A workgroup owns a contiguous range of
// views and its lane groups take them in a fixed pattern, so every sum below has a shape fixed by
// B alone:
//   z = h . w + b,  loss term,  dz = (sigmoid(z) - y) / B,
//   delta[b, j] = dz * w[j] * [h[b, j] > 0]                      (delta of the last hidden layer)
//   part_w[block][j] = sum_b dz_b h[b, j],  part_b[block] = sum_b dz_b,  part_loss[block] = sum_b loss_b
//   part_d[block][j] = sum_b delta[b, j]                         (bias gradient of the last hidden layer)
// G lanes (32 or 64) share a view and own NV 16-byte pieces of its row each; a wavefront takes
// kLogitRows * (64 / G) views per round, all their rows in flight together.  The scalar part (loss,
// sigmoid, dLoss/dz) of view u of a group is evaluated by the group's lane u, all views of the round
// at once, and handed back to the group by a lane read.
constexpr int kLogitRows = 4;

template <int G> __device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int off = G / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// d = [h > 0] * dz * w for one 16-byte piece; returns the piece as stored and adds what was stored to gd
template <typename T> struct DeltaPiece;
template <> struct DeltaPiece<float> {
  static __device__ __forceinline__ float4 make(const Vec16<float> &h, const Vec16<float> &w, float dz, float (&gw)[4],
                                                 float (&gd)[4]) {
    float d[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float hval = h.get(e);
      gw[e] += dz * hval;
      d[e] = hval > 0.0f ? dz * w.get(e) : 0.0f;
      gd[e] += d[e];
    }
    return make_float4(d[0], d[1], d[2], d[3]);
  }
};
template <> struct DeltaPiece<bf16_t> {
  static __device__ __forceinline__ uint4 make(const Vec16<bf16_t> &h, const Vec16<bf16_t> &w, float dz, float (&gw)[8],
                                                float (&gd)[8]) {
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const float h0 = h.get(e), h1 = h.get(e + 1);
      gw[e] += dz * h0;
      gw[e + 1] += dz * h1;
      const uint32_t word = pack_bf16(h0 > 0.0f ? dz * w.get(e) : 0.0f, h1 > 0.0f ? dz * w.get(e + 1) : 0.0f);
      gd[e] += __uint_as_float(word << 16);  // the stored (rounded) values
      gd[e + 1] += __uint_as_float(word & 0xffff0000u);
      o[e >> 1] = word;
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
  }
};

template <typename T, int NV, int G>
__global__ void __launch_bounds__(256)
k_logit_loss(const T *__restrict__ h, const T *__restrict__ w, const float *__restrict__ bias,
             const float *__restrict__ label, int B, int H, int rows_per_block, float *__restrict__ logits,
             float *__restrict__ dz_out, T *__restrict__ delta, float *__restrict__ part_w,
             float *__restrict__ part_d, float *__restrict__ part_b, float *__restrict__ part_loss,
             const int32_t *__restrict__ status) {
  if (*status != 0) return;
  constexpr int VEC = Vec16<T>::N;
  constexpr int GROUPS = kWave / G;            // views a wavefront handles side by side
  constexpr int PARTS = 4 * GROUPS;            // partial sums per column in a workgroup
  __shared__ float s_red[4][2];
  extern __shared__ float s_w[];  // [PARTS][H] weight-gradient sums, then [PARTS][H] delta sums
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int gl = lane & (G - 1), gi = lane / G;
  const int n_vec = H / VEC;
  const float b0 = bias[0], invB = 1.0f / (float)B;

  Vec16<T> wv[NV];
  float gw[NV][VEC], gd[NV][VEC];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int v = gl + i * G;
    wv[i].v = decltype(wv[i].v){};
    if (v < n_vec) wv[i].v = *reinterpret_cast<const decltype(wv[i].v) *>(w + v * VEC);
#pragma unroll
    for (int e = 0; e < VEC; ++e) gw[i][e] = gd[i][e] = 0.0f;
  }
  float loss_acc = 0.0f, dz_acc = 0.0f;  // partial sums of the views this lane evaluates
  const int r0 = blockIdx.x * rows_per_block, r1 = min(B, r0 + rows_per_block);
  constexpr int ROUND = kLogitRows * GROUPS;  // views per wavefront and round
  for (int base = r0 + wave * ROUND; base < r1; base += 4 * ROUND) {
    Vec16<T> hv[kLogitRows][NV];
    float dot[kLogitRows];
    // the label of the view this lane will evaluate, asked for together with the rows
    const int my_view = base + gl * GROUPS + gi;
    const bool mine = gl < kLogitRows && my_view < r1;
    const float y = mine ? label[my_view] : 0.0f;
#pragma unroll
    for (int u = 0; u < kLogitRows; ++u) {
      const int view = base + u * GROUPS + gi;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int v = gl + i * G;
        hv[u][i].v = decltype(hv[u][i].v){};
        if (view < r1 && v < n_vec) hv[u][i].v = *reinterpret_cast<const decltype(hv[u][i].v) *>(h + (size_t)view * H + v * VEC);
      }
    }
#pragma unroll
    for (int u = 0; u < kLogitRows; ++u) {
      float d = 0.0f;
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int e = 0; e < VEC; ++e) d += hv[u][i].get(e) * wv[i].get(e);
      dot[u] = group_sum<G>(d);
    }
    // lane u of a group evaluates the group's view u
    float z = dot[0];
#pragma unroll
    for (int u = 1; u < kLogitRows; ++u) z = gl == u ? dot[u] : z;
    z += b0;
    const float ex = expf(-fabsf(z));
    const float sig = z >= 0.0f ? 1.0f / (1.0f + ex) : ex / (1.0f + ex);
    const float dzv = (sig - y) * invB;
    if (mine) {
      loss_acc += fmaxf(z, 0.0f) - z * y + log1pf(ex);
      dz_acc += dzv;
      logits[my_view] = z;
      dz_out[my_view] = dzv;
    }
#pragma unroll
    for (int u = 0; u < kLogitRows; ++u) {
      const int view = base + u * GROUPS + gi;
      const float dz = __shfl(dzv, gi * G + u, kWave);
      if (view < r1) {
        T *dr = delta + (size_t)view * H;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          const int v = gl + i * G;
          if (v < n_vec)
            *reinterpret_cast<decltype(hv[u][i].v) *>(dr + v * VEC) = DeltaPiece<T>::make(hv[u][i], wv[i], dz, gw[i], gd[i]);
        }
      }
    }
  }
  // combine the groups of the four waves in a fixed order
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int v = gl + i * G;
    if (v < n_vec)
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        s_w[(wave * GROUPS + gi) * H + v * VEC + e] = gw[i][e];
        s_w[(PARTS + wave * GROUPS + gi) * H + v * VEC + e] = gd[i][e];
      }
  }
  loss_acc = wave_sum(loss_acc);
  dz_acc = wave_sum(dz_acc);
  if (lane == 0) {
    s_red[wave][0] = loss_acc;
    s_red[wave][1] = dz_acc;
  }
  __syncthreads();
  for (int j = threadIdx.x; j < H; j += blockDim.x) {
    float tw = 0.0f, td = 0.0f;
#pragma unroll
    for (int q = 0; q < PARTS; ++q) {
      tw += s_w[q * H + j];
      td += s_w[(PARTS + q) * H + j];
    }
    part_w[(size_t)blockIdx.x * H + j] = tw;
    part_d[(size_t)blockIdx.x * H + j] = td;
  }
  if (threadIdx.x == 0) {
    part_loss[blockIdx.x] = ((s_red[0][0] + s_red[1][0]) + s_red[2][0]) + s_red[3][0];
    part_b[blockIdx.x] = ((s_red[0][1] + s_red[1][1]) + s_red[2][1]) + s_red[3][1];
  }
}

// loss = (sum of the workgroups' partial sums) / B, by one wavefront, in a fixed shape
__device__ __forceinline__ void loss_final(const float *__restrict__ loss_partial, int n, int B,
                                           float *__restrict__ loss) {
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
__device__ __forceinline__ void partial_sgd(const float *__restrict__ partial, int P, int H, float *__restrict__ dst,
                                            const Optim &opt, const Moments &mom, int block) {
  __shared__ float s[32][8];
  const int c = threadIdx.x & 7, g = threadIdx.x >> 3;
  const int j = block * 8 + c;
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
    dst[j] = optim_apply(opt, dst[j], t, mom.m + j, mom.v + j);
  }
}

__global__ void __launch_bounds__(256) k_partial_sgd(const float *__restrict__ partial, int P, int H,
                                                     float *__restrict__ dst, Optim opt, Moments mom,
                                                     const int32_t *__restrict__ status) {
  if (*status != 0) return;
  partial_sgd(partial, P, H, dst, opt, mom, blockIdx.x);
}

// Everything that follows k_logit_loss in one launch; blockIdx.y picks the job: 0 the logit layer's
// weights, 1 the last hidden layer's bias, 2 the logit bias, 3 the loss.
__global__ void __launch_bounds__(256)
k_logit_finish(const float *__restrict__ part_w, const float *__restrict__ part_d, const float *__restrict__ part_b,
               const float *__restrict__ part_loss, int P, int H, int B, float *__restrict__ w_last,
               float *__restrict__ bias_hidden, float *__restrict__ bias_last, float *__restrict__ loss, Optim opt,
               Moments mom_w, Moments mom_bh, Moments mom_bl, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  if (blockIdx.y == 0) {
    partial_sgd(part_w, P, H, w_last, opt, mom_w, blockIdx.x);
  } else if (blockIdx.y == 1) {
    partial_sgd(part_d, P, H, bias_hidden, opt, mom_bh, blockIdx.x);
  } else if (blockIdx.x == 0) {
    if (blockIdx.y == 2)
      partial_sgd(part_b, P, 1, bias_last, opt, mom_bl, 0);
    else if (threadIdx.x < kWave)
      loss_final(part_loss, P, B, loss);
  }
}

}  // namespace

hipError_t launch_cast_weights(int count, const float *const *w, const int *rows, const int *cols, int dtype,
                               void *const *wc, void *const *wct, const int32_t *status, hipStream_t s) {
  if (count < 1 || count > GEAR_MAX_LAYERS) return hipErrorInvalidValue;
  CastArgs args;
  args.count = count;
  int blocks = 0;
  for (int i = 0; i < GEAR_MAX_LAYERS; ++i) {
    const bool in = i < count;
    args.w[i] = in ? w[i] : nullptr;
    args.wc[i] = in ? wc[i] : nullptr;
    args.wct[i] = in ? wct[i] : nullptr;
    args.rows[i] = in ? rows[i] : 0;
    args.cols[i] = in ? cols[i] : 0;
    args.first_block[i] = blocks;
    if (in) blocks += ((cols[i] + 31) / 32) * ((rows[i] + 31) / 32);
  }
  if (blocks == 0) return hipSuccess;
  if (dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_cast_weights<bf16_t>, dim3(blocks), dim3(256), 0, s, args, status);
  else
    hipLaunchKernelGGL(k_cast_weights<float>, dim3(blocks), dim3(256), 0, s, args, status);
  return hipGetLastError();
}

int logit_blocks(int B) {
  int blocks = (B + 31) / 32;
  return blocks < 1 ? 1 : (blocks > kLossBlocks ? kLossBlocks : blocks);
}

// Forward logit + loss + delta of the last hidden layer, then SGD on the logit layer's weight and bias.
hipError_t launch_logit_loss(int dtype, const void *h, const void *wc_last, const float *bias_last, const float *label,
                             int B, int H, float *logits, float *dz, void *delta, float *partials,
                             const int32_t *status, hipStream_t s) {
  if (B <= 0) return hipSuccess;
  const int blocks = logit_blocks(B);
  const int rows_per_block = (B + blocks - 1) / blocks;
  float *part_w = partials, *part_d = part_w + (size_t)kLossBlocks * H, *part_b = part_d + (size_t)kLossBlocks * H,
        *part_loss = part_b + kLossBlocks;
  // lanes per view and 16-byte pieces per lane, from the width of the last hidden layer
  const int n_vec = H / (dtype == GEAR_BF16 ? 8 : 4);
#define GEAR_LOGIT(T, NV, G)                                                                                        \
  hipLaunchKernelGGL((k_logit_loss<T, NV, G>), dim3(blocks), dim3(256), 2 * 4 * (kWave / G) * (size_t)H * sizeof(float), \
                     s, (const T *)h, (const T *)wc_last, bias_last, label, B, H, rows_per_block, logits, dz,       \
                     (T *)delta, part_w, part_d, part_b, part_loss, status)
#define GEAR_LOGIT_T(T)                 \
  if (n_vec <= 32)                      \
    GEAR_LOGIT(T, 1, 32);               \
  else if (n_vec <= 64)                 \
    GEAR_LOGIT(T, 1, 64);               \
  else if (n_vec <= 128)                \
    GEAR_LOGIT(T, 2, 64);               \
  else                                  \
    GEAR_LOGIT(T, 4, 64)
  if (dtype == GEAR_BF16) {
    GEAR_LOGIT_T(bf16_t);
  } else {
    GEAR_LOGIT_T(float);
  }
#undef GEAR_LOGIT_T
#undef GEAR_LOGIT
  return hipGetLastError();
}

// The sums the launch above left in `partials`: the loss, and SGD on the logit layer's weights, its
// bias and the bias of the last hidden layer.  Nothing later in a step reads what this writes.
hipError_t launch_logit_finish(float *partials, int B, int H, float *w_last, float *bias_last, float *bias_hidden,
                               float *loss, const Optim &opt, const Moments &mom_w_last, const Moments &mom_bias_last,
                               const Moments &mom_bias_hidden, const int32_t *status, hipStream_t s) {
  if (B <= 0) return hipSuccess;
  const int blocks = logit_blocks(B);
  float *part_w = partials, *part_d = part_w + (size_t)kLossBlocks * H, *part_b = part_d + (size_t)kLossBlocks * H,
        *part_loss = part_b + kLossBlocks;
  hipLaunchKernelGGL(k_logit_finish, dim3((H + 7) / 8, 4), dim3(256), 0, s, part_w, part_d, part_b, part_loss, blocks,
                     H, B, w_last, bias_hidden, bias_last, loss, opt, mom_w_last, mom_bias_hidden, mom_bias_last, status);
  return hipGetLastError();
}

size_t logit_partial_floats(int H) { return 2 * (size_t)kLossBlocks * H + 2 * (size_t)kLossBlocks; }

hipError_t launch_partial_sgd(const float *partial, int P, int H, float *dst, const Optim &opt, const Moments &mom,
                              const int32_t *status, hipStream_t s) {
  if (P <= 0 || H <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_partial_sgd, dim3((H + 7) / 8), dim3(256), 0, s, partial, P, H, dst, opt, mom, status);
  return hipGetLastError();
}

// dst[j] -= lr * sum_b src[b][j]   (bias gradient of a hidden layer)
hipError_t launch_colsum_sgd(int dtype, const void *src, int B, int H, float *partial, float *dst, const Optim &opt,
                             const Moments &mom, const int32_t *status, hipStream_t s) {
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
  hipLaunchKernelGGL(k_partial_sgd, dim3((H + 7) / 8), dim3(256), 0, s, partial, chunks, H, dst, opt, mom, status);
  return hipGetLastError();
}

}  // namespace gear
