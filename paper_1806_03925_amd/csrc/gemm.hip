// Dense contractions of the Sparse-Part MLP on the matrix cores (Section 3, step 4: the Fastgear
// Worker runs the Sparse Part forward to the loss and back-propagates through it).
//
//   forward   a_l      = h_{l-1} W_l^T + b_l           NT, epilogue bias + ReLU
//   dgrad     d_{l-1}  = (d_l W_l) * [a_{l-1} > 0]     NT on the transposed weight copy
//   wgrad     dW_l     = d_l^T h_{l-1}                  TN, split over the batch, fixed-order sum
//
// One workgroup = 4 wavefronts (2 x 2), block tile 128 x 128, each wavefront 64 x 64 as 2 x 2
// MFMA 32x32 tiles.  bf16 operands use v_mfma_f32_32x32x16_bf16 (8 k-values per lane), fp32
// operands v_mfma_f32_32x32x2_f32; accumulation is fp32 in both.  Operand tiles sit in LDS as
// [row][k] with k contiguous, so a lane fetches its MFMA operand with one 16-byte LDS read.  For the
// TN form the global tiles are [k][row]; each thread transposes an 8 x 8 block in registers on
// the way into LDS.
#include "gear_internal.hpp"

namespace gear {
namespace {

typedef __bf16 bf16x8_v __attribute__((ext_vector_type(8)));
typedef float f32x16_v __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, THREADS = 256;

template <typename T> struct Tile;
template <> struct Tile<bf16_t> {
  static constexpr int BK = 64, LDK = 72, VEC = 8;
};
template <> struct Tile<float> {
  static constexpr int BK = 16, LDK = 17, VEC = 4;
};

union Pack16 {
  uint4 u;
  float4 f;
  bf16x8_v b;
  uint32_t w[4];
  float s[4];
};

// ---- global -> registers -----------------------------------------------------------------------
// NT: tile rows are matrix rows, k contiguous.  rows x BK elements = rows*BK/VEC 16-byte vectors.
template <typename T, int NV>
__device__ __forceinline__ void load_nt(Pack16 (&r)[NV], const T *__restrict__ src, int ld, int row0, int rows_total,
                                        int k0, int k_end, int tid) {
  constexpr int VPR = Tile<T>::BK / Tile<T>::VEC;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int v = tid + THREADS * i;
    const int row = row0 + v / VPR, k = k0 + (v % VPR) * Tile<T>::VEC;
    if (row < rows_total && k < k_end)
      r[i].u = *reinterpret_cast<const uint4 *>(src + (size_t)row * ld + k);
    else
      r[i].u = make_uint4(0u, 0u, 0u, 0u);
  }
}

template <typename T, int NV>
__device__ __forceinline__ void store_nt(const Pack16 (&r)[NV], T *lds, int tid) {
  constexpr int VPR = Tile<T>::BK / Tile<T>::VEC;
  constexpr int LDK = Tile<T>::LDK;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int v = tid + THREADS * i;
    const int row = v / VPR, kv = (v % VPR) * Tile<T>::VEC;
    if constexpr (sizeof(T) == 2) {
      *reinterpret_cast<uint4 *>(lds + row * LDK + kv) = r[i].u;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) lds[row * LDK + kv + e] = r[i].s[e];
    }
  }
}

// TN, bf16: a thread owns one 8(k) x 8(row) block: 8 vectors along `row`, one per k.
__device__ __forceinline__ void load_tn_bf16(Pack16 (&r)[8], const bf16_t *__restrict__ src, int ld, int row0,
                                             int rows_total, int k0, int k_end, int blk) {
  // 128 rows = 16 row-vectors; 64 k = 8 k-blocks; blk in [0, 128)
  const int rv = blk % 16, kb = blk / 16;
  const int row = row0 + rv * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int k = k0 + kb * 8 + e;
    if (row < rows_total && k < k_end)
      r[e].u = *reinterpret_cast<const uint4 *>(src + (size_t)k * ld + row);
    else
      r[e].u = make_uint4(0u, 0u, 0u, 0u);
  }
}

__device__ __forceinline__ void store_tn_bf16(const Pack16 (&r)[8], bf16_t *lds, int blk) {
  constexpr int LDK = Tile<bf16_t>::LDK;
  const int rv = blk % 16, kb = blk / 16;
#pragma unroll
  for (int m = 0; m < 8; ++m) {  // output row m of the block: k = 0..7 from r[k].elem[m]
    Pack16 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t a = r[2 * j].w[m >> 1], b = r[2 * j + 1].w[m >> 1];
      o.w[j] = (m & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0x0000ffffu) | (b << 16));
    }
    *reinterpret_cast<uint4 *>(lds + (rv * 8 + m) * LDK + kb * 8) = o.u;
  }
}

// TN, fp32: tile is 16(k) x 128(row) floats = 512 float4 along `row`; 2 per thread.
__device__ __forceinline__ void load_tn_f32(Pack16 (&r)[2], const float *__restrict__ src, int ld, int row0,
                                            int rows_total, int k0, int k_end, int tid) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int v = tid + THREADS * i;
    const int k = k0 + v / 32, row = row0 + (v % 32) * 4;
    if (row < rows_total && k < k_end)
      r[i].u = *reinterpret_cast<const uint4 *>(src + (size_t)k * ld + row);
    else
      r[i].u = make_uint4(0u, 0u, 0u, 0u);
  }
}

__device__ __forceinline__ void store_tn_f32(const Pack16 (&r)[2], float *lds, int tid) {
  constexpr int LDK = Tile<float>::LDK;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int v = tid + THREADS * i;
    const int k = v / 32, row = (v % 32) * 4;
#pragma unroll
    for (int e = 0; e < 4; ++e) lds[(row + e) * LDK + k] = r[i].s[e];
  }
}

// ---- LDS -> MFMA -----------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void mma_tile(f32x16_v (&acc)[2][2], const T *As, const T *Bs, int wm, int wn, int lane) {
  constexpr int LDK = Tile<T>::LDK, BK = Tile<T>::BK;
  const int r = lane & 31, g = lane >> 5;
  if constexpr (sizeof(T) == 2) {
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      Pack16 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i].u = *reinterpret_cast<const uint4 *>(As + (wm * 64 + i * 32 + r) * LDK + kk * 16 + g * 8);
        b[i].u = *reinterpret_cast<const uint4 *>(Bs + (wn * 64 + i * 32 + r) * LDK + kk * 16 + g * 8);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].b, b[j].b, acc[i][j], 0, 0, 0);
    }
  } else {
#pragma unroll
    for (int kk = 0; kk < BK / 2; ++kk) {
      float a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = As[(wm * 64 + i * 32 + r) * LDK + kk * 2 + g];
        b[i] = Bs[(wn * 64 + i * 32 + r) * LDK + kk * 2 + g];
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }
}

// Accumulator element e of a 32x32 tile sits at row 8*(e/4) + 4*(lane/32) + e%4, column lane%32.
template <typename T, int EPI>
__device__ __forceinline__ void epilogue(const f32x16_v (&acc)[2][2], int m0, int n0, int wm, int wn, int lane, int M,
                                         int N, const float *__restrict__ bias, const T *__restrict__ aux,
                                         void *__restrict__ out) {
  const int c = lane & 31, g = lane >> 5;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n0 + wn * 64 + j * 32 + c;
      if (n >= N) continue;
      float bn = 0.0f;
      if constexpr (EPI == EPI_BIAS_RELU) bn = bias[n];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm * 64 + i * 32 + 8 * (e / 4) + 4 * g + (e % 4);
        if (m >= M) continue;
        const size_t idx = (size_t)m * N + n;
        float v = acc[i][j][e];
        if constexpr (EPI == EPI_BIAS_RELU) {
          v += bn;
          static_cast<T *>(out)[idx] = from_f32<T>(v > 0.0f ? v : 0.0f);
        } else if constexpr (EPI == EPI_MASK) {
          static_cast<T *>(out)[idx] = from_f32<T>(to_f32<T>(aux[idx]) > 0.0f ? v : 0.0f);
        } else {
          static_cast<float *>(out)[idx] = v;
        }
      }
    }
}

// ---- kernels ---------------------------------------------------------------------------------------
template <typename T, int EPI>
__global__ void __launch_bounds__(THREADS)
k_gemm_nt(const T *__restrict__ A, const T *__restrict__ B, int M, int N, int K, const float *__restrict__ bias,
          const T *__restrict__ aux, void *__restrict__ out, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  constexpr int BK = Tile<T>::BK, LDK = Tile<T>::LDK;
  constexpr int NV = BM * (BK / Tile<T>::VEC) / THREADS;
  __shared__ __attribute__((aligned(16))) T As[BM * LDK];
  __shared__ __attribute__((aligned(16))) T Bs[BN * LDK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int n_tiles = (N + BN - 1) / BN;
  const int m0 = (blockIdx.x / n_tiles) * BM, n0 = (blockIdx.x % n_tiles) * BN;

  f32x16_v acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  Pack16 ra[NV], rb[NV];
  load_nt<T, NV>(ra, A, K, m0, M, 0, K, tid);
  load_nt<T, NV>(rb, B, K, n0, N, 0, K, tid);
  for (int k0 = 0; k0 < K; k0 += BK) {
    store_nt<T, NV>(ra, As, tid);
    store_nt<T, NV>(rb, Bs, tid);
    __syncthreads();
    if (k0 + BK < K) {
      load_nt<T, NV>(ra, A, K, m0, M, k0 + BK, K, tid);
      load_nt<T, NV>(rb, B, K, n0, N, k0 + BK, K, tid);
    }
    mma_tile<T>(acc, As, Bs, wm, wn, lane);
    __syncthreads();
  }
  epilogue<T, EPI>(acc, m0, n0, wm, wn, lane, M, N, bias, aux, out);
}

template <typename T>
__global__ void __launch_bounds__(THREADS)
k_gemm_tn(const T *__restrict__ A, const T *__restrict__ B, int M, int N, int K, int k_chunk,
          float *__restrict__ partial, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  constexpr int BK = Tile<T>::BK, LDK = Tile<T>::LDK;
  __shared__ __attribute__((aligned(16))) T As[BM * LDK];
  __shared__ __attribute__((aligned(16))) T Bs[BN * LDK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int n_tiles = (N + BN - 1) / BN;
  const int m0 = (blockIdx.x / n_tiles) * BM, n0 = (blockIdx.x % n_tiles) * BN;
  const int k_begin = blockIdx.z * k_chunk;
  const int k_end = min(K, k_begin + k_chunk);

  f32x16_v acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  if constexpr (sizeof(T) == 2) {
    // threads 0..127 stage A blocks, 128..255 stage B blocks
    const bool isB = tid >= 128;
    const int blk = tid & 127;
    const T *src = isB ? B : A;
    const int ld = isB ? N : M, row0 = isB ? n0 : m0, rows = isB ? N : M;
    T *dst = isB ? Bs : As;
    Pack16 r[8];
    load_tn_bf16(r, src, ld, row0, rows, k_begin, k_end, blk);
    for (int k0 = k_begin; k0 < k_end; k0 += BK) {
      store_tn_bf16(r, dst, blk);
      __syncthreads();
      if (k0 + BK < k_end) load_tn_bf16(r, src, ld, row0, rows, k0 + BK, k_end, blk);
      mma_tile<T>(acc, As, Bs, wm, wn, lane);
      __syncthreads();
    }
  } else {
    Pack16 ra[2], rb[2];
    load_tn_f32(ra, A, M, m0, M, k_begin, k_end, tid);
    load_tn_f32(rb, B, N, n0, N, k_begin, k_end, tid);
    for (int k0 = k_begin; k0 < k_end; k0 += BK) {
      store_tn_f32(ra, As, tid);
      store_tn_f32(rb, Bs, tid);
      __syncthreads();
      if (k0 + BK < k_end) {
        load_tn_f32(ra, A, M, m0, M, k0 + BK, k_end, tid);
        load_tn_f32(rb, B, N, n0, N, k0 + BK, k_end, tid);
      }
      mma_tile<T>(acc, As, Bs, wm, wn, lane);
      __syncthreads();
    }
  }
  epilogue<T, EPI_F32>(acc, m0, n0, wm, wn, lane, M, N, nullptr, nullptr, partial + (size_t)blockIdx.z * M * N);
}

// W -= lr * sum_z partial[z], z ascending
__global__ void __launch_bounds__(256) k_splitk_sgd(const float *__restrict__ partial, int splits, int64_t count,
                                                    float *__restrict__ w, float lr,
                                                    const int32_t *__restrict__ status) {
  if (*status != 0) return;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  float g = 0.0f;
  for (int z = 0; z < splits; ++z) g += partial[(size_t)z * count + i];
  w[i] -= lr * g;
}

template <typename T>
hipError_t run_nt(const void *A, const void *B, int M, int N, int K, int epi, const float *bias, const void *aux,
                  void *out, const int32_t *status, hipStream_t s) {
  const dim3 grid(((M + BM - 1) / BM) * ((N + BN - 1) / BN));
#define GEAR_NT(E)                                                                                                  \
  hipLaunchKernelGGL((k_gemm_nt<T, E>), grid, dim3(THREADS), 0, s, (const T *)A, (const T *)B, M, N, K, bias,       \
                     (const T *)aux, out, status)
  if (epi == EPI_BIAS_RELU)
    GEAR_NT(EPI_BIAS_RELU);
  else if (epi == EPI_MASK)
    GEAR_NT(EPI_MASK);
  else
    GEAR_NT(EPI_F32);
#undef GEAR_NT
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_nt(int dtype, const void *A, const void *B, int M, int N, int K, int epilogue_kind,
                          const float *bias, const void *aux, void *out, const int32_t *status, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  return dtype == GEAR_BF16 ? run_nt<bf16_t>(A, B, M, N, K, epilogue_kind, bias, aux, out, status, s)
                            : run_nt<float>(A, B, M, N, K, epilogue_kind, bias, aux, out, status, s);
}

hipError_t launch_gemm_tn_splitk(int dtype, const void *A, const void *B, int M, int N, int K, int splits,
                                 float *partial, const int32_t *status, hipStream_t s) {
  if (M <= 0 || N <= 0 || splits <= 0) return hipSuccess;
  const int bk = dtype == GEAR_BF16 ? Tile<bf16_t>::BK : Tile<float>::BK;
  int k_chunk = (K + splits - 1) / splits;
  k_chunk = ((k_chunk + bk - 1) / bk) * bk;
  if (k_chunk == 0) k_chunk = bk;
  const dim3 grid(((M + BM - 1) / BM) * ((N + BN - 1) / BN), 1, splits);
  if (dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_gemm_tn<bf16_t>, grid, dim3(THREADS), 0, s, (const bf16_t *)A, (const bf16_t *)B, M, N, K,
                       k_chunk, partial, status);
  else
    hipLaunchKernelGGL(k_gemm_tn<float>, grid, dim3(THREADS), 0, s, (const float *)A, (const float *)B, M, N, K,
                       k_chunk, partial, status);
  return hipGetLastError();
}

hipError_t launch_splitk_sgd(const float *partial, int splits, int64_t count, float *w, float lr,
                             const int32_t *status, hipStream_t s) {
  if (count <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_splitk_sgd, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, partial, splits, count, w,
                     lr, status);
  return hipGetLastError();
}

}  // namespace gear
