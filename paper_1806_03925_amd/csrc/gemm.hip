// Dense contractions of the Sparse-Part MLP on the matrix cores (Section 3, step 4: the Fastgear
// Worker runs the Sparse Part forward to the loss and back-propagates through it).
//
//   forward   a_l      = h_{l-1} W_l^T + b_l           NT, epilogue bias + ReLU
//   dgrad     d_{l-1}  = (d_l W_l) * [a_{l-1} > 0]     NT on the transposed weight copy
//   wgrad     dW_l     = d_l^T h_{l-1}                  TN, split over the batch, fixed-order sum
//
// bf16, K a multiple of 32 (every workload): one workgroup = 8 wavefronts (2 x 4) on a 256 x 256
// block tile, a wavefront owns 128 x 64 as 4 x 2 MFMA 32x32x16 tiles.  Operand tiles of k-depth 32
// are copied global -> LDS by DMA (global_load_lds_dwordx4) into four stages.  NT form: two k-tiles
// are copied together while the two before them are multiplied (the halves of a 128-byte line then
// meet in the vector cache), one wait and one s_barrier per pair; LDS rows are [row][32 k] with the
// four 16-byte k-pieces XOR-swizzled by the row so that ds_read_b128 operand fetches do not conflict.
// TN form (wgrad): one k-tile per barrier, two in flight; LDS keeps the global [k][row] order and
// ds_read_b64_tr_b16 assembles the operand.
// bf16 results leave through a per-wave LDS patch so that every lane stores 16 contiguous bytes.
// Consecutive workgroup ids are spread over the eight XCDs by the hardware; the tile index is
// remapped so that workgroups on one XCD walk neighbouring tiles and share operands in its L2.
//
// Everything else (fp32 operands with v_mfma_f32_32x32x2_f32, K not a multiple of 32) goes through a
// register-staged kernel: 4 wavefronts on a 256 x 128 tile, operands in LDS as [row][k], the next
// k-tile prefetched into registers, TN tiles transposed in registers on the way into LDS.
#include "gear_internal.hpp"

#include <type_traits>

namespace gear {
namespace {

typedef __bf16 bf16x8_v __attribute__((ext_vector_type(8)));
typedef float f32x16_v __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 128, THREADS = 256;
constexpr int WM = 128, WN = 64;           // wave tile
constexpr int TM = WM / 32, TN = WN / 32;  // MFMA tiles per wave
constexpr int kXcds = 8;

// Block geometry of the register-staged kernels: 2 x 2 wavefronts, each TM_ x TN_ MFMA tiles of 32 x 32.
// The DMA kernels are written for the big one only (the constants above).  The smaller ones exist
// because a product of few rows has too few 256 x 128 tiles to reach every CU.
template <int TM_, int TN_> struct Geo {
  static constexpr int TM = TM_, TN = TN_, WM = 32 * TM_, WN = 32 * TN_, BM = 2 * WM, BN = 2 * WN;
};
using GeoBig = Geo<4, 2>;    // 256 x 128
using GeoMid = Geo<2, 2>;    // 128 x 128
using GeoSmall = Geo<1, 1>;  //  64 x  64
#define GEAR_GEO(G) \
  constexpr int TM = G::TM, TN = G::TN, WM = G::WM, WN = G::WN, BM = G::BM, BN = G::BN; \
  (void)TM, (void)TN, (void)WM, (void)WN, (void)BM, (void)BN

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

// workgroup id -> tile id such that the workgroups of one XCD (ids congruent modulo 8) cover a
// contiguous range of tiles
__device__ __forceinline__ int xcd_remap(int bid, int n_blocks) {
  const int per = n_blocks / kXcds, rem = n_blocks % kXcds;
  const int xcd = bid % kXcds, local = bid / kXcds;
  // the first `rem` XCDs own per + 1 tiles
  const int start = xcd * per + (xcd < rem ? xcd : rem);
  return start + local;
}

// ---- global -> registers -> LDS, NT form: tile rows are matrix rows, k contiguous ------------------
template <typename T, int ROWS>
struct StageNT {
  static constexpr int VPR = Tile<T>::BK / Tile<T>::VEC;  // 16-byte vectors per tile row
  static constexpr int NV = ROWS * VPR / THREADS;
  Pack16 r[NV];

  __device__ __forceinline__ void load(const T *__restrict__ src, int ld, int row0, int rows_total, int k0, int k_end,
                                       int tid) {
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
  __device__ __forceinline__ void store(T *lds, int tid) const {
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
};

// ---- TN form, bf16: the global tile is [64 k][ROWS], a thread owns 8(k) x 8(row) blocks ------------
template <int ROWS>
struct StageTNbf16 {
  static constexpr int BLOCKS = (ROWS / 8) * 8;                       // 8 k-blocks
  static constexpr int NB = (BLOCKS + THREADS - 1) / THREADS;         // blocks per thread (1)
  Pack16 r[NB][8];

  __device__ __forceinline__ void load(const bf16_t *__restrict__ src, int ld, int row0, int rows_total, int k0,
                                       int k_end, int tid) {
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int blk = tid + THREADS * b;
      const int rv = blk % (ROWS / 8), kb = blk / (ROWS / 8);
      const int row = row0 + rv * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int k = k0 + kb * 8 + e;
        if (blk < BLOCKS && row < rows_total && k < k_end)
          r[b][e].u = *reinterpret_cast<const uint4 *>(src + (size_t)k * ld + row);
        else
          r[b][e].u = make_uint4(0u, 0u, 0u, 0u);
      }
    }
  }
  __device__ __forceinline__ void store(bf16_t *lds, int tid) const {
    constexpr int LDK = Tile<bf16_t>::LDK;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int blk = tid + THREADS * b;
      if (blk >= BLOCKS) continue;
      const int rv = blk % (ROWS / 8), kb = blk / (ROWS / 8);
#pragma unroll
      for (int m = 0; m < 8; ++m) {  // row m of the block collects element m of the eight k-vectors
        Pack16 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t a = r[b][2 * j].w[m >> 1], c = r[b][2 * j + 1].w[m >> 1];
          o.w[j] = (m & 1) ? ((a >> 16) | (c & 0xffff0000u)) : ((a & 0x0000ffffu) | (c << 16));
        }
        *reinterpret_cast<uint4 *>(lds + (rv * 8 + m) * LDK + kb * 8) = o.u;
      }
    }
  }
};

// ---- TN form, fp32: the global tile is [16 k][ROWS] floats = ROWS*4 float4 along `row` -------------
template <int ROWS>
struct StageTNf32 {
  static constexpr int NV = ROWS * 4 / THREADS;
  Pack16 r[NV];
  __device__ __forceinline__ void load(const float *__restrict__ src, int ld, int row0, int rows_total, int k0,
                                       int k_end, int tid) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int v = tid + THREADS * i;
      const int k = k0 + v / (ROWS / 4), row = row0 + (v % (ROWS / 4)) * 4;
      if (row < rows_total && k < k_end)
        r[i].u = *reinterpret_cast<const uint4 *>(src + (size_t)k * ld + row);
      else
        r[i].u = make_uint4(0u, 0u, 0u, 0u);
    }
  }
  __device__ __forceinline__ void store(float *lds, int tid) const {
    constexpr int LDK = Tile<float>::LDK;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int v = tid + THREADS * i;
      const int k = v / (ROWS / 4), row = (v % (ROWS / 4)) * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) lds[(row + e) * LDK + k] = r[i].s[e];
    }
  }
};

// ---- LDS -> MFMA -----------------------------------------------------------------------------------
template <typename T, typename G = GeoBig>
__device__ __forceinline__ void mma_tile(f32x16_v (&acc)[G::TM][G::TN], const T *As, const T *Bs, int wm, int wn,
                                         int lane) {
  GEAR_GEO(G);
  constexpr int LDK = Tile<T>::LDK, BK = Tile<T>::BK;
  const int r = lane & 31, g = lane >> 5;
  if constexpr (sizeof(T) == 2) {
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      Pack16 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i].u = *reinterpret_cast<const uint4 *>(As + (wm * WM + i * 32 + r) * LDK + kk * 16 + g * 8);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j].u = *reinterpret_cast<const uint4 *>(Bs + (wn * WN + j * 32 + r) * LDK + kk * 16 + g * 8);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].b, b[j].b, acc[i][j], 0, 0, 0);
    }
  } else {
#pragma unroll
    for (int kk = 0; kk < BK / 2; ++kk) {
      float a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) a[i] = As[(wm * WM + i * 32 + r) * LDK + kk * 2 + g];
#pragma unroll
      for (int j = 0; j < TN; ++j) b[j] = Bs[(wn * WN + j * 32 + r) * LDK + kk * 2 + g];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }
}

// Accumulator element e of a 32x32 tile sits at row 8*(e/4) + 4*(lane/32) + e%4, column lane%32.
// fp32 results are stored straight from that layout (a half-wave covers 128 contiguous bytes).
template <typename T, int EPI, typename G = GeoBig>
__device__ __forceinline__ void epilogue_direct(const f32x16_v (&acc)[G::TM][G::TN], int m0, int n0, int wm, int wn,
                                                int lane, int M, int N, const float *__restrict__ bias,
                                                const T *__restrict__ aux, void *__restrict__ out, int split = 0) {
  GEAR_GEO(G);
  const int c = lane & 31, g = lane >> 5;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn * WN + j * 32 + c;
      if (n >= N) continue;
      float bn = 0.0f;
      if constexpr (EPI == EPI_BIAS_RELU) bn = bias[n];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm * WM + i * 32 + 8 * (e / 4) + 4 * g + (e % 4);
        if (m >= M) continue;
        const size_t idx = (size_t)m * N + n;
        float v = acc[i][j][e];
        if constexpr (EPI == EPI_BIAS_RELU) {
          v += bn;
          static_cast<T *>(out)[idx] = from_f32<T>(v > 0.0f ? v : 0.0f);
        } else if constexpr (EPI == EPI_MASK) {
          static_cast<T *>(out)[idx] = from_f32<T>(to_f32<T>(aux[idx]) > 0.0f ? v : 0.0f);
        } else if constexpr (EPI == EPI_DX) {
          // columns below `split` stay fp32 in `out`, the others go to `aux` in the operand type
          if (n < split)
            static_cast<float *>(out)[(size_t)m * split + n] = v;
          else
            const_cast<T *>(aux)[(size_t)m * (N - split) + (n - split)] = from_f32<T>(v);
        } else {
          static_cast<float *>(out)[idx] = v;
        }
      }
    }
}

// bf16 results: each wave parks 64 rows x 64 columns at a time in its own LDS patch, then every lane
// moves 16 contiguous bytes (eight lanes per 128-byte row piece); the ReLU mask of the dgrad is read
// with the same 16-byte pattern.
template <int EPI, typename G = GeoBig>
__device__ __forceinline__ void epilogue_bf16(const f32x16_v (&acc)[G::TM][G::TN], bf16_t *patch, int m0, int n0, int wm,
                                              int wn, int lane, int M, int N, const float *__restrict__ bias,
                                              const bf16_t *__restrict__ aux, bf16_t *__restrict__ out) {
  GEAR_GEO(G);
  static_assert(G::TM % 2 == 0 && G::TN == 2, "the patch holds 64 rows x 64 columns of a wave's tile");
  constexpr int LDC = WN + 8;  // bf16 elements per patch row
  const int c = lane & 31, g = lane >> 5;
#pragma unroll
  for (int half = 0; half < TM / 2; ++half) {
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int i = half * 2 + ii;
        const int n = n0 + wn * WN + j * 32 + c;
        float bn = 0.0f;
        if constexpr (EPI == EPI_BIAS_RELU) bn = n < N ? bias[n] : 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          float v = acc[i][j][e];
          if constexpr (EPI == EPI_BIAS_RELU) {
            v += bn;
            v = v > 0.0f ? v : 0.0f;
          }
          patch[(ii * 32 + 8 * (e / 4) + 4 * g + (e % 4)) * LDC + j * 32 + c] = f32_to_bf16(v);
        }
      }
    // the patch is private to this wave: no workgroup barrier needed, only the wave's own LDS order
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = it * 8 + (lane >> 3), cv = (lane & 7) * 8;
      const int m = m0 + wm * WM + half * 64 + row, n = n0 + wn * WN + cv;
      if (m < M && n < N) {
        Pack16 v;
        v.u = *reinterpret_cast<const uint4 *>(patch + row * LDC + cv);
        const size_t idx = (size_t)m * N + n;
        if constexpr (EPI == EPI_MASK) {
          Pack16 h;
          h.u = *reinterpret_cast<const uint4 *>(aux + idx);
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            // keep a half-word where the forward activation was positive (bf16 > 0: sign clear, not zero)
            const uint32_t lo = h.w[w] & 0xffffu, hi = h.w[w] >> 16;
            uint32_t keep = 0u;
            if (lo != 0u && lo < 0x8000u) keep |= 0x0000ffffu;
            if (hi != 0u && hi < 0x8000u) keep |= 0xffff0000u;
            v.w[w] &= keep;
          }
        }
        *reinterpret_cast<uint4 *>(out + idx) = v.u;
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}


// ---- NT form, bf16, K % 32 == 0: global -> LDS by DMA, four stages, 256 x 256 tile, 8 waves ---------
typedef __attribute__((address_space(3))) void *lds_ptr_t;
constexpr int DK = 32;                      // k-depth of a stage
constexpr int DM = 256, DN = 256, DTHREADS = 512;
constexpr int A_ELEMS = DM * DK;
// Two shapes of the workgroup's tile.  Wide: 256 result columns, four stages, one pair of k-tiles in flight
// beside the pair that is being multiplied.  Narrow, for results of at most 128 columns (dLoss/dx of the
// embedding slots): a product of so few columns has little arithmetic per k-tile and waits for its copies,
// so the B tile is 128 rows, a stage is 24 KB, and six stages keep two pairs in flight.
// The eight wavefronts cover the tile as 2 x 4 wave tiles of 128 x 64 (wide) or as 4 x 2 of 64 x 64 (narrow),
// so that all of them have columns in either shape; TMW = 32-row MFMA tiles per wave tile.
struct NtWide {
  static constexpr int BN = 256, STAGES = 4, AHEAD = 1, TMW = 4, WAVES_N = 4;
};
struct NtNarrow {
  static constexpr int BN = 128, STAGES = 6, AHEAD = 2, TMW = 2, WAVES_N = 2;
};
template <typename C> constexpr int stage_elems() { return A_ELEMS + C::BN * DK; }
// global_load_lds instructions a wave issues per pair of k-tiles: 16 rows of A twice, 16 rows of B per 128, two k-tiles
template <typename C> constexpr int dma_per_pair() { return 2 * (2 + C::BN / 128); }

__device__ __forceinline__ int swz(int row) { return (row >> 2) & 3; }

template <int N> __device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}
__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

struct DmaPlan {
  size_t a_off[2], b_off[2];  // element offsets of this lane's 16-byte pieces at k0 = 0
};

// Two consecutive k-tiles at once: a 128-byte line of an operand row holds the row's share of both,
// and its two 64-byte halves are requested by back-to-back instructions of one wave, which meet in
// the vector cache -- one L2 access per line instead of two.
template <typename C>
__device__ __forceinline__ void dma_pair(const bf16_t *__restrict__ A, const bf16_t *__restrict__ B, const DmaPlan &p,
                                         int k0, int k1, bf16_t *s0, bf16_t *s1, int wave) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    __builtin_amdgcn_global_load_lds((const void *)(A + p.a_off[i] + k0), (lds_ptr_t)(s0 + (i * 8 + wave) * 512), 16, 0, 0);
    __builtin_amdgcn_global_load_lds((const void *)(A + p.a_off[i] + k1), (lds_ptr_t)(s1 + (i * 8 + wave) * 512), 16, 0, 0);
  }
#pragma unroll
  for (int i = 0; i < C::BN / 128; ++i) {
    __builtin_amdgcn_global_load_lds((const void *)(B + p.b_off[i] + k0), (lds_ptr_t)(s0 + A_ELEMS + (i * 8 + wave) * 512), 16, 0, 0);
    __builtin_amdgcn_global_load_lds((const void *)(B + p.b_off[i] + k1), (lds_ptr_t)(s1 + A_ELEMS + (i * 8 + wave) * 512), 16, 0, 0);
  }
}

// MFMA operands are fetched with explicit ds_read_b128 so that the only waits on the LDS path are
// the ones written here (the compiler would otherwise make every LDS read wait for all DMA in flight).
typedef uint32_t u32x4_v __attribute__((ext_vector_type(4)));
#define LDS_READ16(dst, addr, OFF) asm volatile("ds_read_b128 %0, %1 offset:" #OFF : "=v"(dst) : "v"(addr) : "memory")
#define MFMA_BF16(acc_, a_, b_) \
  acc_ = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_v, a_), __builtin_bit_cast(bf16x8_v, b_), acc_, 0, 0, 0)
// The NT kernel takes the product as (B rows) x (A rows)^T: a lane then holds, for ONE row
// m = lane % 32 of the result, the columns n = 8 (e / 4) + 4 (lane / 32) + e % 4 -- four consecutive
// columns per group of four accumulator elements, which is what its epilogue packs and stores.
#define MFMA_BF16_T(acc_, a_, b_) MFMA_BF16(acc_, b_, a_)

__device__ __forceinline__ void mma_stage(f32x16_v (&acc)[2][TN], uint32_t a_addr0, uint32_t a_addr1, uint32_t b_addr0,
                                          uint32_t b_addr1) {
  u32x4_v p0, p1, q0, q1;   // k-step 0: A rows of the two m-tiles, B rows of the two n-tiles
  u32x4_v r0, r1, s0, s1;   // k-step 1
  LDS_READ16(p0, a_addr0, 0);
  LDS_READ16(p1, a_addr0, 2048);
  LDS_READ16(q0, b_addr0, 0);
  LDS_READ16(q1, b_addr0, 2048);
  LDS_READ16(r0, a_addr1, 0);
  LDS_READ16(r1, a_addr1, 2048);
  LDS_READ16(s0, b_addr1, 0);
  LDS_READ16(s1, b_addr1, 2048);
  asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(p0), "+v"(p1), "+v"(q0), "+v"(q1)::"memory");
  MFMA_BF16_T(acc[0][0], p0, q0);
  MFMA_BF16_T(acc[0][1], p0, q1);
  MFMA_BF16_T(acc[1][0], p1, q0);
  MFMA_BF16_T(acc[1][1], p1, q1);
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(r0), "+v"(r1), "+v"(s0), "+v"(s1)::"memory");
  MFMA_BF16_T(acc[0][0], r0, s0);
  MFMA_BF16_T(acc[0][1], r0, s1);
  MFMA_BF16_T(acc[1][0], r1, s0);
  MFMA_BF16_T(acc[1][1], r1, s1);
}

__device__ __forceinline__ void mma_stage(f32x16_v (&acc)[TM][TN], uint32_t a_addr0, uint32_t a_addr1, uint32_t b_addr0,
                                          uint32_t b_addr1) {
  u32x4_v p0, p1, p2, p3, q0, q1;   // k-step 0: A rows of the four m-tiles, B rows of the two n-tiles
  u32x4_v r0, r1, r2, r3, s0, s1;   // k-step 1
  LDS_READ16(p0, a_addr0, 0);
  LDS_READ16(p1, a_addr0, 2048);
  LDS_READ16(p2, a_addr0, 4096);
  LDS_READ16(p3, a_addr0, 6144);
  LDS_READ16(q0, b_addr0, 0);
  LDS_READ16(q1, b_addr0, 2048);
  LDS_READ16(r0, a_addr1, 0);
  LDS_READ16(r1, a_addr1, 2048);
  LDS_READ16(r2, a_addr1, 4096);
  LDS_READ16(r3, a_addr1, 6144);
  LDS_READ16(s0, b_addr1, 0);
  LDS_READ16(s1, b_addr1, 2048);
  asm volatile("s_waitcnt lgkmcnt(6)" : "+v"(p0), "+v"(p1), "+v"(p2), "+v"(p3), "+v"(q0), "+v"(q1)::"memory");
  MFMA_BF16_T(acc[0][0], p0, q0);
  MFMA_BF16_T(acc[0][1], p0, q1);
  MFMA_BF16_T(acc[1][0], p1, q0);
  MFMA_BF16_T(acc[1][1], p1, q1);
  MFMA_BF16_T(acc[2][0], p2, q0);
  MFMA_BF16_T(acc[2][1], p2, q1);
  MFMA_BF16_T(acc[3][0], p3, q0);
  MFMA_BF16_T(acc[3][1], p3, q1);
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(r0), "+v"(r1), "+v"(r2), "+v"(r3), "+v"(s0), "+v"(s1)::"memory");
  MFMA_BF16_T(acc[0][0], r0, s0);
  MFMA_BF16_T(acc[0][1], r0, s1);
  MFMA_BF16_T(acc[1][0], r1, s0);
  MFMA_BF16_T(acc[1][1], r1, s1);
  MFMA_BF16_T(acc[2][0], r2, s0);
  MFMA_BF16_T(acc[2][1], r2, s1);
  MFMA_BF16_T(acc[3][0], r3, s0);
  MFMA_BF16_T(acc[3][1], r3, s1);
}

// Results of the DMA kernel.  A lane holds row m = lane % 32 of each 32 x 32 tile and, per group of
// four accumulator elements, four consecutive columns.  fp32 results are stored from there as
// 16-byte pieces.  bf16 results are converted in pairs (v_cvt_pk_bf16_f32), written as 8-byte pieces
// into a per-wave LDS patch of 32 rows x 64 columns and read back row-wise so that every lane stores
// 16 contiguous bytes and a row of the patch leaves as one 128-byte line; the ReLU mask of a dgrad
// (EPI_MASK) is read with the same 16-byte pattern before the patch is written.  EPI_DX splits the
// columns: below `split` fp32 into `out` [M x split], the rest bf16 into `aux` [M x (N - split)].
constexpr int PATCH_LD = WN + 8;  // bf16 elements per patch row (144 bytes: the 8-byte writes of a wave spread over all banks)

template <int EPI, int TMW>
__device__ __forceinline__ void epilogue_patch(const f32x16_v (&acc)[TMW][TN], bf16_t *patch, int m0, int n0, int wm,
                                               int wn, int lane, int M, int N, const float *__restrict__ bias,
                                               const bf16_t *__restrict__ aux, void *__restrict__ out, int split,
                                               uint8_t *__restrict__ relu_bits, float (&colacc)[8],
                                               const float *tile_bias, const uint32_t (&hbits)[TMW][4]) {
  const int c = lane & 31, g = lane >> 5;
  const int wave_m0 = m0 + wm * (32 * TMW), wave_n0 = n0 + wn * WN;
  // where this wave's columns go
  bool direct_f32 = EPI == EPI_F32, mixed = false;
  int ld_f32 = N, ld_bf = N, col_shift = 0;
  bf16_t *out_bf = static_cast<bf16_t *>(out);
  if constexpr (EPI == EPI_DX) {
    ld_f32 = split;
    ld_bf = N - split;
    col_shift = split;
    out_bf = const_cast<bf16_t *>(aux);
    direct_f32 = wave_n0 + WN <= split;
    mixed = !direct_f32 && wave_n0 < split;
  }
  if (mixed) {  // the split falls inside this wave's columns: element by element
#pragma unroll
    for (int i = 0; i < TMW; ++i) {
      const int m = wave_m0 + i * 32 + c;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int n = wave_n0 + j * 32 + 8 * (e / 4) + 4 * g + (e % 4);
          if (m < M && n < N) {
            if (n < split)
              static_cast<float *>(out)[(size_t)m * ld_f32 + n] = acc[i][j][e];
            else
              out_bf[(size_t)m * ld_bf + (n - col_shift)] = f32_to_bf16(acc[i][j][e]);
          }
        }
    }
    return;
  }
  if (direct_f32) {
    // column counts are multiples of 8, so a group of four columns is inside the matrix or outside
#pragma unroll
    for (int i = 0; i < TMW; ++i) {
      const int m = wave_m0 + i * 32 + c;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = wave_n0 + j * 32 + 8 * q + 4 * g;
          if (m < M && n < N)
            *reinterpret_cast<float4 *>(static_cast<float *>(out) + (size_t)m * ld_f32 + n) =
                make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        }
    }
    return;
  }
  if constexpr (EPI != EPI_F32) {
    float bn[TN][16];
    if constexpr (EPI == EPI_BIAS_RELU) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          // the tile's biases were staged in LDS before the main loop (zero beyond N)
          bn[j][e] = tile_bias[wn * WN + j * 32 + 8 * (e / 4) + 4 * g + (e % 4)];
        }
    }
    // lane's 16-byte pieces: rows it*8 + lane/8 of each 32-row band, columns (lane%8)*8 .. +7
    const int prow = lane >> 3, cv = (lane & 7) * 8;
    const int n_vec = wave_n0 + cv;
    Pack16 h[EPI == EPI_MASK ? TMW : 1][4];
    if constexpr (EPI == EPI_MASK) {
#pragma unroll
      for (int i = 0; i < TMW; ++i)
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int m = wave_m0 + i * 32 + it * 8 + prow;
          if (m < M && n_vec < N)
            h[i][it].u = *reinterpret_cast<const uint4 *>(aux + (size_t)m * N + n_vec);
          else
            h[i][it].u = make_uint4(0u, 0u, 0u, 0u);
        }
    }
#pragma unroll
    for (int i = 0; i < TMW; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float v[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            v[r] = acc[i][j][4 * q + r];
            if constexpr (EPI == EPI_BIAS_RELU) {
              v[r] += bn[j][4 * q + r];
              v[r] = v[r] > 0.0f ? v[r] : 0.0f;
            }
          }
          *reinterpret_cast<uint2 *>(patch + c * PATCH_LD + j * 32 + 8 * q + 4 * g) =
              make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
        }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int row = it * 8 + prow;
        const int m = wave_m0 + i * 32 + row;
        Pack16 v;
        v.u = *reinterpret_cast<const uint4 *>(patch + row * PATCH_LD + cv);
        if (m < M && n_vec < N) {
          if constexpr (EPI == EPI_BIAS_RELU) {
            if (relu_bits) {
              // results are >= 0: a value is positive exactly when its bf16 pattern is not zero
              uint32_t byte = 0u;
#pragma unroll
              for (int w = 0; w < 4; ++w) {
                if (v.w[w] & 0x0000ffffu) byte |= 1u << (2 * w);
                if (v.w[w] & 0xffff0000u) byte |= 2u << (2 * w);
              }
              relu_bits[(size_t)m * (N >> 3) + (n_vec >> 3)] = (uint8_t)byte;
            }
          }
          if constexpr (EPI == EPI_MASK || EPI == EPI_MASK_BITS) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
              uint32_t keep = 0u;
              if constexpr (EPI == EPI_MASK) {
                // keep a half-word where the forward activation was positive (bf16 > 0: sign clear, not zero)
                const uint32_t lo = h[i][it].w[w] & 0xffffu, hi = h[i][it].w[w] >> 16;
                if (lo != 0u && lo < 0x8000u) keep |= 0x0000ffffu;
                if (hi != 0u && hi < 0x8000u) keep |= 0xffff0000u;
              } else {
                if (hbits[i][it] & (1u << (2 * w))) keep |= 0x0000ffffu;
                if (hbits[i][it] & (2u << (2 * w))) keep |= 0xffff0000u;
              }
              v.w[w] &= keep;
              // column sums of what is stored (the bias gradient of the layer below)
              colacc[2 * w] += __uint_as_float(v.w[w] << 16);
              colacc[2 * w + 1] += __uint_as_float(v.w[w] & 0xffff0000u);
            }
          }
          // streamed out: nobody on this XCD reads these lines again before they would be evicted,
          // and operand lines that other tiles are about to share stay in its L2 instead
          __builtin_nontemporal_store(u32x4_v{v.u.x, v.u.y, v.u.z, v.u.w},
                                      reinterpret_cast<u32x4_v *>(out_bf + (size_t)m * ld_bf + (n_vec - col_shift)));
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
}

constexpr int STAGES = 4;                       // of the TN kernel below

// Tiles t and t + 1 (t even) are copied together into stages t % S and (t + 1) % S while the pairs
// before them are multiplied: one wait and one barrier per pair.  C::AHEAD pairs are in flight beyond the
// one being multiplied; vector memory operations finish in issue order, so waiting until only the later
// pairs' instructions are outstanding means the current pair has landed.  When nk is odd the last pair's
// second half copies the last tile again, into a stage nobody reads.
template <bool MMA, typename C>
__device__ __forceinline__ void nt_main_loop(f32x16_v (&acc)[C::TMW][TN], const bf16_t *__restrict__ A,
                                             const bf16_t *__restrict__ B, const DmaPlan &plan, bf16_t *lds, int nk,
                                             int wave, const uint32_t (&a_rel)[2], const uint32_t (&b_rel)[2]) {
  constexpr int SE = stage_elems<C>();
  static_assert(C::AHEAD == 1 || C::AHEAD == 2, "pairs in flight");
  static_assert(C::STAGES == 2 * (C::AHEAD + 1), "a pair being multiplied and AHEAD pairs being copied");
  auto issue = [&](int t) {
    const int t1 = min(t + 1, nk - 1);
    dma_pair<C>(A, B, plan, t * DK, t1 * DK, lds + (t % C::STAGES) * SE, lds + ((t + 1) % C::STAGES) * SE, wave);
  };
  issue(0);
  if (C::AHEAD == 2 && 2 < nk) issue(2);
  for (int t = 0; t < nk; ++t) {
    if ((t & 1) == 0) {
      // this wave's share of tiles t and t + 1 has landed
      if (C::AHEAD == 2 && t + 2 < nk)
        wait_vm<dma_per_pair<C>()>();
      else
        wait_vm<0>();
      block_barrier();  // ... everybody's has, and everybody is done reading tiles t - 2 and t - 1
      if (t + 2 * C::AHEAD < nk) issue(t + 2 * C::AHEAD);
    }
    const uint32_t so = (uint32_t)(t % C::STAGES) * (2u * SE);
    if constexpr (MMA) mma_stage(acc, a_rel[0] + so, a_rel[1] + so, b_rel[0] + so, b_rel[1] + so);
  }
}

template <int EPI, typename C = NtWide>
__global__ void __launch_bounds__(DTHREADS)
k_gemm_nt_dma(const bf16_t *__restrict__ A, const bf16_t *__restrict__ B, int M, int N, int K,
              const float *__restrict__ bias, const bf16_t *__restrict__ aux, void *__restrict__ out, int split,
              float *__restrict__ colpart, uint8_t *__restrict__ relu_bits, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  __shared__ __attribute__((aligned(1024))) bf16_t lds[C::STAGES * stage_elems<C>()];   // [stage][A tile | B tile]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int TMW = C::TMW, WMW = 32 * C::TMW;   // this shape's wave tile: WMW rows x WN columns
  const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
  const int n_tiles = (N + C::BN - 1) / C::BN;
  const int tile = xcd_remap(blockIdx.x, gridDim.x);
  const int m0 = (tile / n_tiles) * DM, n0 = (tile % n_tiles) * C::BN;

  DmaPlan plan;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = (i * 8 + wave) * 16 + (lane >> 2);
    const int kv = (lane & 3) ^ swz(row);
    plan.a_off[i] = (size_t)min(m0 + row, M - 1) * K + kv * 8;
    plan.b_off[i] = (size_t)min(n0 + row, N - 1) * K + kv * 8;
  }
  // byte offsets, inside a stage, of this lane's MFMA operands for the two k-steps
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
  uint32_t a_rel[2], b_rel[2];
  {
    const int r = lane & 31, g = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const int off = r * DK + (((2 * kk + g) ^ swz(r)) * 8);
      a_rel[kk] = lds_base + 2u * (uint32_t)(wm * WMW * DK + off);
      b_rel[kk] = lds_base + 2u * (uint32_t)(A_ELEMS + wn * WN * DK + off);
    }
  }

  // What the epilogue needs from global memory is requested here, so that it arrives while the
  // products run: the tile's biases go to LDS (the barriers of the main loop make them visible), the
  // sign bits of the lane's sixteen 16-byte pieces (eight bits each) stay in registers.
  __shared__ float s_bias[EPI == EPI_BIAS_RELU ? C::BN : 1];
  if constexpr (EPI == EPI_BIAS_RELU) {
    if (tid < C::BN) s_bias[tid] = n0 + tid < N ? bias[n0 + tid] : 0.0f;
  }
  uint32_t hbits[TMW][4];
#pragma unroll
  for (int i = 0; i < TMW; ++i)
#pragma unroll
    for (int it = 0; it < 4; ++it) hbits[i][it] = 0u;
  if constexpr (EPI == EPI_MASK_BITS) {
    const uint8_t *bits = reinterpret_cast<const uint8_t *>(aux);
    const int n_vec = n0 + wn * WN + (lane & 7) * 8;
#pragma unroll
    for (int i = 0; i < TMW; ++i)
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int m = m0 + wm * WMW + i * 32 + it * 8 + (lane >> 3);
        if (m < M && n_vec < N) hbits[i][it] = bits[(size_t)m * (N >> 3) + (n_vec >> 3)];
      }
  }

  f32x16_v acc[TMW][TN];
#pragma unroll
  for (int i = 0; i < TMW; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // in a tile whose right part lies beyond N, the waves without columns copy tiles and meet the
  // barriers but skip the operand reads and the products
  const bool has_columns = n0 + wn * WN < N;
  if (has_columns)
    nt_main_loop<true, C>(acc, A, B, plan, lds, K / DK, wave, a_rel, b_rel);
  else
    nt_main_loop<false, C>(acc, A, B, plan, lds, K / DK, wave, a_rel, b_rel);
  wait_vm<0>();
  block_barrier();  // every wave is done with the operand tiles: the first stages become the output patches
  static_assert((8 * 32 * PATCH_LD) * 2 + 8 * 64 * 4 <= C::STAGES * stage_elems<C>() * 2, "patches and column sums fit");
  bf16_t *patch = lds + wave * 32 * PATCH_LD;
  float colacc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (has_columns)
    epilogue_patch<EPI, TMW>(acc, patch, m0, n0, wm, wn, lane, M, N, bias, aux, out, split, relu_bits, colacc, s_bias, hbits);
  if constexpr (EPI == EPI_MASK || EPI == EPI_MASK_BITS) {
    static_assert(C::WAVES_N == 4, "the column sums below add the two wave rows of the wide shape");
    if (colpart) {
      // colpart[m-tile][n] = sum over the tile's rows of the stored values: lanes that share lane % 8
      // hold the same eight columns, then the two waves that share the columns are added
      float *s_col = reinterpret_cast<float *>(lds + 8 * 32 * PATCH_LD);  // behind the eight output patches
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float v = colacc[e];
        v += __shfl_xor(v, 8, kWave);
        v += __shfl_xor(v, 16, kWave);
        v += __shfl_xor(v, 32, kWave);
        if (lane < 8) s_col[wave * 64 + lane * 8 + e] = v;
      }
      __syncthreads();
      if (wm == 0 && lane < 8) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int n = n0 + wn * WN + lane * 8 + e;
          if (n < N) colpart[(size_t)(m0 / DM) * N + n] = s_col[wave * 64 + lane * 8 + e] + s_col[(wave + 4) * 64 + lane * 8 + e];
        }
      }
    }
  }
}

// ---- TN form (wgrad), bf16, by DMA and LDS transpose reads ---------------------------------------
// Global tiles are [k][row] with `row` contiguous, which is also how they are kept in LDS: a DMA
// instruction copies two k-rows of 256 values (1 KB).  The MFMA operand (8 k-values of one row per
// lane) is assembled by ds_read_b64_tr_b16: sixteen lanes hand in the addresses of a 4(k) x 16(row)
// block as four-value pieces and each lane gets back one row's four k-values.  Both operands use
// the same pattern, so they agree on which k sits in which slot.
typedef uint32_t u32x2_v __attribute__((ext_vector_type(2)));
constexpr int TCHUNK = 1024 + 32;                 // bytes: two k-rows of 512 B, then a pad
constexpr int TSTAGE = 2 * 16 * TCHUNK;           // A chunks then B chunks
#define LDS_READ_TR(dst, addr, OFF) \
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "i"(OFF) : "memory")

struct TnPlan {
  size_t a_off[2], b_off[2];
};

__device__ __forceinline__ void dma_tile_tn(const bf16_t *__restrict__ A, const bf16_t *__restrict__ B,
                                            const TnPlan &p, int k0, int M, int N, unsigned char *stage, int wave) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
    __builtin_amdgcn_global_load_lds((const void *)(A + p.a_off[i] + (size_t)k0 * M),
                                     (lds_ptr_t)(stage + (i * 8 + wave) * TCHUNK), 16, 0, 0);
#pragma unroll
  for (int i = 0; i < 2; ++i)
    __builtin_amdgcn_global_load_lds((const void *)(B + p.b_off[i] + (size_t)k0 * N),
                                     (lds_ptr_t)(stage + (16 + i * 8 + wave) * TCHUNK), 16, 0, 0);
}

// operand of MFMA tile at immediate OFF (bytes) for k-step KK: two transpose reads, k-rows +0..3 and +4..7
#define TN_OPERAND(dst, base, OFF, KK)                                   \
  {                                                                      \
    u32x2_v lo_, hi_;                                                    \
    LDS_READ_TR(lo_, base, (KK) * 8 * TCHUNK + (OFF));                   \
    LDS_READ_TR(hi_, base, (KK) * 8 * TCHUNK + 2 * TCHUNK + (OFF));      \
    dst = u32x4_v{lo_.x, lo_.y, hi_.x, hi_.y};                           \
  }

__device__ __forceinline__ void mma_stage_tn(f32x16_v (&acc)[TM][TN], uint32_t a_even, uint32_t a_odd, uint32_t b_even,
                                             uint32_t b_odd) {
#define TN_KSTEP(KK)                                       \
  {                                                        \
    u32x4_v p0, p1, p2, p3, q0, q1;                        \
    TN_OPERAND(p0, a_even, 0, KK)                          \
    TN_OPERAND(p1, a_odd, 64, KK)                          \
    TN_OPERAND(p2, a_even, 128, KK)                        \
    TN_OPERAND(p3, a_odd, 192, KK)                         \
    TN_OPERAND(q0, b_even, 0, KK)                          \
    TN_OPERAND(q1, b_odd, 64, KK)                          \
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(p0), "+v"(p1), "+v"(p2), "+v"(p3), "+v"(q0), "+v"(q1)::"memory"); \
    MFMA_BF16(acc[0][0], p0, q0);                          \
    MFMA_BF16(acc[0][1], p0, q1);                          \
    MFMA_BF16(acc[1][0], p1, q0);                          \
    MFMA_BF16(acc[1][1], p1, q1);                          \
    MFMA_BF16(acc[2][0], p2, q0);                          \
    MFMA_BF16(acc[2][1], p2, q1);                          \
    MFMA_BF16(acc[3][0], p3, q0);                          \
    MFMA_BF16(acc[3][1], p3, q1);                          \
  }
  TN_KSTEP(0)
  TN_KSTEP(1)
#undef TN_KSTEP
}

template <bool MMA>
__device__ __forceinline__ void tn_main_loop(f32x16_v (&acc)[TM][TN], const bf16_t *__restrict__ A,
                                             const bf16_t *__restrict__ B, const TnPlan &plan, int k_begin, int nk, int M,
                                             int N, unsigned char *lds, int wave, uint32_t a_even, uint32_t a_odd,
                                             uint32_t b_even, uint32_t b_odd) {
#pragma unroll
  for (int p = 0; p < STAGES - 1; ++p)
    if (p < nk) dma_tile_tn(A, B, plan, k_begin + p * DK, M, N, lds + p * TSTAGE, wave);

  int stage = 0;
  for (int t = 0; t < nk; ++t) {
    if (t + 2 < nk)
      wait_vm<8>();
    else if (t + 1 < nk)
      wait_vm<4>();
    else
      wait_vm<0>();
    block_barrier();
    if (t + 3 < nk) dma_tile_tn(A, B, plan, k_begin + (t + 3) * DK, M, N, lds + ((stage + 3) & 3) * TSTAGE, wave);
    const uint32_t so = (uint32_t)stage * TSTAGE;
    if constexpr (MMA) mma_stage_tn(acc, a_even + so, a_odd + so, b_even + so, b_odd + so);
    stage = (stage + 1) & 3;
  }
}

// One workgroup's share: tile `tile` of the [M x N] result over the k-range `split`, left in
// partial[split][M x N].
__device__ __forceinline__ void tn_dma_work(const bf16_t *__restrict__ A, const bf16_t *__restrict__ B, int M, int N,
                                            int K, int k_chunk, float *__restrict__ partial, int split, int tile,
                                            unsigned char *lds) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int n_tiles = (N + DN - 1) / DN;
  const int m0 = (tile / n_tiles) * DM, n0 = (tile % n_tiles) * DN;
  const int k_begin = split * k_chunk;
  const int k_end = min(K, k_begin + k_chunk);

  // DMA: chunk c = k-rows 2c, 2c+1; lane p holds LDS slot p%32 of k-row p/32, which receives the
  // 8-value piece (p%32) ^ (4 * (p/32)) so that odd k-rows sit 64 bytes away from even ones
  TnPlan plan;
  {
    const int krow = lane >> 5, piece = (lane & 31) ^ (4 * krow);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int k = 2 * (i * 8 + wave) + krow;
      const int ma = min(m0 + piece * 8, M - 8), nb = min(n0 + piece * 8, N - 8);  // stay inside the row
      plan.a_off[i] = (size_t)k * M + ma;
      plan.b_off[i] = (size_t)k * N + nb;
    }
  }
  // transpose reads: lane l -> j = l%16, half = (l/16)%2 (rows +16), g = l/32 (k-rows +8);
  // it addresses k-row 8 g + j/4 (+4 for the second read), rows 16 half + 4 (j%4) .. +3
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
  uint32_t a_even, a_odd, b_even, b_odd;
  {
    const int j = lane & 15, half = (lane >> 4) & 1, g = lane >> 5;
    const int k = 8 * g + (j >> 2);
    const int odd = k & 1;
    const uint32_t row_off = (uint32_t)(k >> 1) * TCHUNK + (uint32_t)odd * 512u;
    const uint32_t ca = 2u * (uint32_t)(wm * WM + 16 * half + 4 * (j & 3));
    const uint32_t cb = 2u * (uint32_t)(wn * WN + 16 * half + 4 * (j & 3));
    // odd k-rows are stored with the 64-byte halves of every 128 bytes swapped
    a_even = lds_base + row_off + ca + (odd ? 64u : 0u);
    a_odd = lds_base + row_off + ca - (odd ? 64u : 0u);
    b_even = lds_base + 16u * TCHUNK + row_off + cb + (odd ? 64u : 0u);
    b_odd = lds_base + 16u * TCHUNK + row_off + cb - (odd ? 64u : 0u);
  }

  f32x16_v acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  const int nk = (k_end - k_begin + DK - 1) / DK;   // k_end - k_begin is a multiple of DK (checked by the host)
  // in a tile whose right part lies beyond N, the waves without columns copy tiles and meet the
  // barriers but skip the operand reads and the products
  if (n0 + wn * WN < N)
    tn_main_loop<true>(acc, A, B, plan, k_begin, nk, M, N, lds, wave, a_even, a_odd, b_even, b_odd);
  else
    tn_main_loop<false>(acc, A, B, plan, k_begin, nk, M, N, lds, wave, a_even, a_odd, b_even, b_odd);
  // fp32 partial of this k range
  float *dst = partial + (size_t)split * M * N;
  const int c = lane & 31, g = lane >> 5;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn * WN + j * 32 + c;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm * WM + i * 32 + 8 * (e / 4) + 4 * g + (e % 4);
        if (m < M && n < N) dst[(size_t)m * N + n] = acc[i][j][e];
      }
    }
}

__global__ void __launch_bounds__(DTHREADS)
k_gemm_tn_dma(const bf16_t *__restrict__ A, const bf16_t *__restrict__ B, int M, int N, int K, int k_chunk,
              float *__restrict__ partial, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  __shared__ __attribute__((aligned(1024))) unsigned char lds[STAGES * TSTAGE];
  // one-dimensional grid of tiles x k-ranges; the workgroups of one XCD take neighbouring (range, tile)
  // pairs, so the tiles that read the same rows of the batch share them in that XCD's L2
  const int tiles = ((M + DM - 1) / DM) * ((N + DN - 1) / DN);
  const int work = xcd_remap(blockIdx.x, gridDim.x);
  tn_dma_work(A, B, M, N, K, k_chunk, partial, work / tiles, work % tiles, lds);
}

// Several contractions over the same K rows in one launch: the grid is k-ranges x (all tiles of all
// problems), so every workgroup does the same amount of work whichever result it belongs to.
struct TnBatchArgs {
  int count, tiles;
  TnProblem p[GEAR_MAX_LAYERS];
  int first_tile[GEAR_MAX_LAYERS];
};

__global__ void __launch_bounds__(DTHREADS)
k_gemm_tn_dma_batch(TnBatchArgs args, int K, int k_chunk, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  __shared__ __attribute__((aligned(1024))) unsigned char lds[STAGES * TSTAGE];
  const int work = xcd_remap(blockIdx.x, gridDim.x);
  const int split = work / args.tiles, tile = work % args.tiles;
  int which = 0;
  for (int i = 1; i < args.count; ++i)
    if (tile >= args.first_tile[i]) which = i;
  const TnProblem &q = args.p[which];
  tn_dma_work((const bf16_t *)q.A, (const bf16_t *)q.B, q.M, q.N, K, k_chunk, q.partial, split,
              tile - args.first_tile[which], lds);
}

// ---- kernels ---------------------------------------------------------------------------------------
template <typename G = GeoBig> constexpr size_t lds_bytes(size_t elem, int ldk) {
  return (size_t)(G::BM + G::BN) * ldk * elem;
}

template <typename T, int EPI, typename G>
__global__ void __launch_bounds__(THREADS)
k_gemm_nt(const T *__restrict__ A, const T *__restrict__ B, int M, int N, int K, const float *__restrict__ bias,
          const T *__restrict__ aux, void *__restrict__ out, int split, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  GEAR_GEO(G);
  constexpr int BK = Tile<T>::BK, LDK = Tile<T>::LDK;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T *As = reinterpret_cast<T *>(smem);
  T *Bs = As + BM * LDK;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int n_tiles = (N + BN - 1) / BN;
  const int tile = xcd_remap(blockIdx.x, gridDim.x);
  const int m0 = (tile / n_tiles) * BM, n0 = (tile % n_tiles) * BN;

  f32x16_v acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  StageNT<T, BM> sa;
  StageNT<T, BN> sb;
  sa.load(A, K, m0, M, 0, K, tid);
  sb.load(B, K, n0, N, 0, K, tid);
  for (int k0 = 0; k0 < K; k0 += BK) {
    sa.store(As, tid);
    sb.store(Bs, tid);
    __syncthreads();
    if (k0 + BK < K) {
      sa.load(A, K, m0, M, k0 + BK, K, tid);
      sb.load(B, K, n0, N, k0 + BK, K, tid);
    }
    mma_tile<T, G>(acc, As, Bs, wm, wn, lane);
    __syncthreads();
  }
  if constexpr (sizeof(T) == 2 && EPI != EPI_F32 && EPI != EPI_DX && G::TM % 2 == 0 && G::TN == 2) {
    bf16_t *patch = reinterpret_cast<bf16_t *>(smem) + wave * 64 * (WN + 8);
    epilogue_bf16<EPI, G>(acc, patch, m0, n0, wm, wn, lane, M, N, bias, reinterpret_cast<const bf16_t *>(aux),
                          static_cast<bf16_t *>(out));
  } else {
    epilogue_direct<T, EPI, G>(acc, m0, n0, wm, wn, lane, M, N, bias, aux, out, split);
  }
}

template <typename T>
__global__ void __launch_bounds__(THREADS)
k_gemm_tn(const T *__restrict__ A, const T *__restrict__ B, int M, int N, int K, int k_chunk,
          float *__restrict__ partial, const int32_t *__restrict__ status, const int32_t *__restrict__ k_dev) {
  if (*status != 0) return;
  constexpr int BK = Tile<T>::BK, LDK = Tile<T>::LDK;
  if (k_dev) {
    // the contraction length is only known on the device (at most K): the same split into gridDim.z
    // ranges as the host would make; ranges beyond it are empty and leave a partial of zeros
    K = min(max(*k_dev, 0), K);
    k_chunk = (K + (int)gridDim.z - 1) / (int)gridDim.z;
    k_chunk = max((k_chunk + BK - 1) / BK * BK, BK);
  }
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T *As = reinterpret_cast<T *>(smem);
  T *Bs = As + BM * LDK;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int n_tiles = (N + BN - 1) / BN;
  const int tile = xcd_remap(blockIdx.x, gridDim.x);
  const int m0 = (tile / n_tiles) * BM, n0 = (tile % n_tiles) * BN;
  const int k_begin = blockIdx.z * k_chunk;
  const int k_end = min(K, k_begin + k_chunk);

  f32x16_v acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  using SA = typename std::conditional<sizeof(T) == 2, StageTNbf16<BM>, StageTNf32<BM>>::type;
  using SB = typename std::conditional<sizeof(T) == 2, StageTNbf16<BN>, StageTNf32<BN>>::type;
  SA sa;
  SB sb;
  sa.load(A, M, m0, M, k_begin, k_end, tid);
  sb.load(B, N, n0, N, k_begin, k_end, tid);
  for (int k0 = k_begin; k0 < k_end; k0 += BK) {
    sa.store(As, tid);
    sb.store(Bs, tid);
    __syncthreads();
    if (k0 + BK < k_end) {
      sa.load(A, M, m0, M, k0 + BK, k_end, tid);
      sb.load(B, N, n0, N, k0 + BK, k_end, tid);
    }
    mma_tile<T>(acc, As, Bs, wm, wn, lane);
    __syncthreads();
  }
  epilogue_direct<T, EPI_F32>(acc, m0, n0, wm, wn, lane, M, N, nullptr, nullptr,
                              partial + (size_t)blockIdx.z * M * N);
}

// W <- update(W, sum_z partial[z]), z ascending; a thread owns four consecutive elements (count is a
// multiple of 4 because layer widths are multiples of 8) and keeps eight partials in flight
__device__ __forceinline__ void splitk_sgd_at(const float *__restrict__ partial, int splits, int64_t count,
                                              float *__restrict__ w, const Optim &opt, const Moments &mom, int64_t i) {
  if (i >= count) return;
  float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
  int z = 0;
  for (; z + 8 <= splits; z += 8) {
    float4 v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = *reinterpret_cast<const float4 *>(partial + (size_t)(z + k) * count + i);
#pragma unroll
    for (int k = 0; k < 8; ++k) g.x += v[k].x, g.y += v[k].y, g.z += v[k].z, g.w += v[k].w;
  }
  for (; z < splits; ++z) {
    const float4 v = *reinterpret_cast<const float4 *>(partial + (size_t)z * count + i);
    g.x += v.x, g.y += v.y, g.z += v.z, g.w += v.w;
  }
  float4 cur = *reinterpret_cast<float4 *>(w + i);
  if (!opt.adam) {
    cur.x -= opt.lr * g.x, cur.y -= opt.lr * g.y, cur.z -= opt.lr * g.z, cur.w -= opt.lr * g.w;
  } else {
    float4 m = *reinterpret_cast<float4 *>(mom.m + i), v = *reinterpret_cast<float4 *>(mom.v + i);
    cur.x = optim_apply(opt, cur.x, g.x, &m.x, &v.x);
    cur.y = optim_apply(opt, cur.y, g.y, &m.y, &v.y);
    cur.z = optim_apply(opt, cur.z, g.z, &m.z, &v.z);
    cur.w = optim_apply(opt, cur.w, g.w, &m.w, &v.w);
    *reinterpret_cast<float4 *>(mom.m + i) = m;
    *reinterpret_cast<float4 *>(mom.v + i) = v;
  }
  *reinterpret_cast<float4 *>(w + i) = cur;
}

__global__ void __launch_bounds__(256) k_splitk_sgd(const float *__restrict__ partial, int splits, int64_t count,
                                                    float *__restrict__ w, Optim opt, Moments mom,
                                                    const int32_t *__restrict__ status) {
  if (*status != 0) return;
  splitk_sgd_at(partial, splits, count, w, opt, mom, ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4);
}

// the same for the results of a batched launch: a workgroup belongs to one of them
struct SplitkBatchArgs {
  int count;
  SplitkProblem p[GEAR_MAX_LAYERS];
  int first_block[GEAR_MAX_LAYERS];
};

__global__ void __launch_bounds__(256) k_splitk_sgd_batch(SplitkBatchArgs args, int splits, Optim opt,
                                                          const int32_t *__restrict__ status) {
  if (*status != 0) return;
  int which = 0;
  for (int i = 1; i < args.count; ++i)
    if ((int)blockIdx.x >= args.first_block[i]) which = i;
  const SplitkProblem &q = args.p[which];
  splitk_sgd_at(q.partial, splits, q.count, q.w, opt, q.mom,
                ((int64_t)(blockIdx.x - args.first_block[which]) * blockDim.x + threadIdx.x) * 4);
}

template <typename T>
hipError_t run_nt(const void *A, const void *B, int M, int N, int K, int epi, const float *bias, const void *aux,
                  void *out, int split, float *colpart, uint8_t *relu_bits, const int32_t *status, hipStream_t s) {
  if constexpr (sizeof(T) == 2) {
    if (K % DK == 0) {
      const bool narrow = N <= NtNarrow::BN && (epi == EPI_DX || epi == EPI_F32);
      const dim3 grid(((M + DM - 1) / DM) * (narrow ? 1 : (N + DN - 1) / DN));
#define GEAR_DMA_C(E, C)                                                                                              \
  hipLaunchKernelGGL((k_gemm_nt_dma<E, C>), grid, dim3(DTHREADS), 0, s, (const bf16_t *)A, (const bf16_t *)B, M, N, K, \
                     bias, (const bf16_t *)aux, out, split, colpart, relu_bits, status)
#define GEAR_DMA(E) GEAR_DMA_C(E, NtWide)
      if (epi == EPI_BIAS_RELU)
        GEAR_DMA(EPI_BIAS_RELU);
      else if (epi == EPI_MASK)
        GEAR_DMA(EPI_MASK);
      else if (epi == EPI_MASK_BITS)
        GEAR_DMA(EPI_MASK_BITS);
      else if (epi == EPI_DX) {
        if (narrow)
          GEAR_DMA_C(EPI_DX, NtNarrow);
        else
          GEAR_DMA(EPI_DX);
      } else {
        if (narrow)
          GEAR_DMA_C(EPI_F32, NtNarrow);
        else
          GEAR_DMA(EPI_F32);
      }
#undef GEAR_DMA
#undef GEAR_DMA_C
      return hipGetLastError();
    }
  }
  // the largest geometry that still gives every CU a tile (else the smallest)
#define GEAR_NT_G(E, G)                                                                                             \
  hipLaunchKernelGGL((k_gemm_nt<T, E, G>), dim3(((M + G::BM - 1) / G::BM) * ((N + G::BN - 1) / G::BN)), dim3(THREADS), \
                     lds_bytes<G>(sizeof(T), Tile<T>::LDK), s, (const T *)A, (const T *)B, M, N, K, bias,          \
                     (const T *)aux, out, split, status)
#define GEAR_NT(E)                                                                        \
  {                                                                                       \
    if (tiles_of(GeoBig::BM, GeoBig::BN) >= 256)                                          \
      GEAR_NT_G(E, GeoBig);                                                               \
    else if (tiles_of(GeoMid::BM, GeoMid::BN) >= 256)                                     \
      GEAR_NT_G(E, GeoMid);                                                               \
    else                                                                                  \
      GEAR_NT_G(E, GeoSmall);                                                             \
  }
  auto tiles_of = [&](int bm, int bn) { return (long long)((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
  if (epi == EPI_BIAS_RELU)
    GEAR_NT(EPI_BIAS_RELU)
  else if (epi == EPI_MASK)
    GEAR_NT(EPI_MASK)
  else if (epi == EPI_DX)
    GEAR_NT(EPI_DX)
  else
    GEAR_NT(EPI_F32)
#undef GEAR_NT_G
#undef GEAR_NT
  return hipGetLastError();
}

}  // namespace

// Split count of the wgrad contraction, never decreasing in K (a workspace sized for the largest batch
// holds the partials of any smaller one).  bf16 with K a multiple of 32 (the DMA kernel): one
// workgroup per CU holds a 256 x 256 tile, so aim at one full round of the 256 CUs; every range keeps
// at least 512 rows of the batch.  Everything else goes through the register-staged kernel, whose
// workgroup walks its range sixteen (fp32) rows at a time, each step waiting for its loads: there
// short ranges pay, down to 128 rows, as long as the ranges of all 256 x 128 tiles fit one round.
static int splitk_rule(bool dma, int M, int N, int K) {
  const int tiles = dma ? ((M + DM - 1) / DM) * ((N + DN - 1) / DN) : ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  int s = 256 / tiles;
  int cap = K / (dma ? 512 : 128);
  if (cap < 1) cap = 1;
  if (s > cap) s = cap;
  if (s > 64) s = 64;
  return s < 1 ? 1 : s;
}
int gemm_splitk_for(int dtype, int M, int N, int K) {
  return splitk_rule(dtype == GEAR_BF16 && K % DK == 0, M, N, K);
}
// the largest count gemm_splitk_for gives for any K' <= K (which kernel a batch takes depends on K' % 32)
int gemm_splitk_max(int dtype, int M, int N, int K) {
  const int a = splitk_rule(false, M, N, K);
  if (dtype != GEAR_BF16) return a;
  const int b = splitk_rule(true, M, N, K);
  return a > b ? a : b;
}

// Number of row-tile partials the EPI_MASK product leaves in `colpart` ([parts x N] column sums of
// its result), or 0 if this shape goes through the kernel that does not produce them.
int gemm_nt_colsum_parts(int dtype, int M, int N, int K) {
  return (dtype == GEAR_BF16 && K % DK == 0 && M > 0) ? (M + DM - 1) / DM : 0;
}

// The sign bitmap of a bias + ReLU product is written, and taken as a mask, by the DMA kernel only.
bool gemm_nt_has_bits(int dtype, int K) { return dtype == GEAR_BF16 && K % DK == 0; }

hipError_t launch_gemm_nt(int dtype, const void *A, const void *B, int M, int N, int K, int epilogue_kind,
                          const float *bias, const void *aux, void *out, int split, float *colpart,
                          uint8_t *relu_bits, const int32_t *status, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (epilogue_kind == EPI_MASK_BITS && !gemm_nt_has_bits(dtype, K)) return hipErrorInvalidValue;
  return dtype == GEAR_BF16
             ? run_nt<bf16_t>(A, B, M, N, K, epilogue_kind, bias, aux, out, split, colpart, relu_bits, status, s)
             : run_nt<float>(A, B, M, N, K, epilogue_kind, bias, aux, out, split, colpart, relu_bits, status, s);
}

// Split count shared by the problems of a batched launch: one round of the 256 CUs, every range at
// least 512 rows.  0 when the set does not go through the batched kernel.
int gemm_tn_batch_splits(int dtype, const TnProblem *p, int count, int K) {
  if (dtype != GEAR_BF16 || count < 2 || count > GEAR_MAX_LAYERS || K <= 0 || K % DK != 0) return 0;
  int tiles = 0;
  for (int i = 0; i < count; ++i) {
    if (p[i].M < 8 || p[i].N < 8) return 0;
    tiles += ((p[i].M + DM - 1) / DM) * ((p[i].N + DN - 1) / DN);
  }
  if (tiles > 128) return 0;
  int s = 256 / tiles;
  const int cap = K / 512 < 1 ? 1 : K / 512;
  if (s > cap) s = cap;
  return s > 64 ? 64 : s;
}

hipError_t launch_gemm_tn_batch(const TnProblem *p, int count, int K, int splits, const int32_t *status,
                                hipStream_t s) {
  if (count < 1 || count > GEAR_MAX_LAYERS || splits < 1 || K % DK != 0) return hipErrorInvalidValue;
  TnBatchArgs args;
  args.count = count;
  args.tiles = 0;
  for (int i = 0; i < count; ++i) {
    if (p[i].M < 8 || p[i].N < 8 || !p[i].A || !p[i].B || !p[i].partial) return hipErrorInvalidValue;
    args.p[i] = p[i];
    args.first_tile[i] = args.tiles;
    args.tiles += ((p[i].M + DM - 1) / DM) * ((p[i].N + DN - 1) / DN);
  }
  for (int i = count; i < GEAR_MAX_LAYERS; ++i) {
    args.p[i] = TnProblem{nullptr, nullptr, nullptr, 0, 0};
    args.first_tile[i] = args.tiles;
  }
  const int kc = ((((K + splits - 1) / splits) + DK - 1) / DK) * DK;
  hipLaunchKernelGGL(k_gemm_tn_dma_batch, dim3(args.tiles * splits), dim3(DTHREADS), 0, s, args, K, kc, status);
  return hipGetLastError();
}

hipError_t launch_gemm_tn_splitk(int dtype, const void *A, const void *B, int M, int N, int K, int splits,
                                 float *partial, const int32_t *status, hipStream_t s, const int32_t *k_dev) {
  if (M <= 0 || N <= 0 || splits <= 0) return hipSuccess;
  const int bk = dtype == GEAR_BF16 ? Tile<bf16_t>::BK : Tile<float>::BK;
  int k_chunk = (K + splits - 1) / splits;
  k_chunk = ((k_chunk + bk - 1) / bk) * bk;
  if (k_chunk == 0) k_chunk = bk;
  if (!k_dev && dtype == GEAR_BF16 && K % DK == 0 && M >= 8 && N >= 8) {
    const int kc = ((((K + splits - 1) / splits) + DK - 1) / DK) * DK;
    const dim3 grid_dma(((M + DM - 1) / DM) * ((N + DN - 1) / DN) * splits);
    hipLaunchKernelGGL(k_gemm_tn_dma, grid_dma, dim3(DTHREADS), 0, s, (const bf16_t *)A, (const bf16_t *)B, M, N, K, kc,
                       partial, status);
    return hipGetLastError();
  }
  const dim3 grid(((M + BM - 1) / BM) * ((N + BN - 1) / BN), 1, splits);
  if (dtype == GEAR_BF16)
    hipLaunchKernelGGL(k_gemm_tn<bf16_t>, grid, dim3(THREADS), lds_bytes<>(2, Tile<bf16_t>::LDK), s, (const bf16_t *)A,
                       (const bf16_t *)B, M, N, K, k_chunk, partial, status, k_dev);
  else
    hipLaunchKernelGGL(k_gemm_tn<float>, grid, dim3(THREADS), lds_bytes<>(4, Tile<float>::LDK), s, (const float *)A,
                       (const float *)B, M, N, K, k_chunk, partial, status, k_dev);
  return hipGetLastError();
}

hipError_t launch_splitk_sgd(const float *partial, int splits, int64_t count, float *w, const Optim &opt,
                             const Moments &mom, const int32_t *status, hipStream_t s) {
  if (count <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_splitk_sgd, dim3((unsigned)((count / 4 + 255) / 256)), dim3(256), 0, s, partial, splits, count,
                     w, opt, mom, status);
  return hipGetLastError();
}

hipError_t launch_splitk_sgd_batch(const SplitkProblem *p, int count, int splits, const Optim &opt,
                                   const int32_t *status, hipStream_t s) {
  if (count < 1 || count > GEAR_MAX_LAYERS || splits < 1) return hipErrorInvalidValue;
  SplitkBatchArgs args;
  args.count = count;
  int blocks = 0;
  for (int i = 0; i < GEAR_MAX_LAYERS; ++i) {
    args.p[i] = i < count ? p[i] : SplitkProblem{nullptr, nullptr, Moments{nullptr, nullptr}, 0};
    args.first_block[i] = blocks;
    if (i < count) blocks += (int)((p[i].count / 4 + 255) / 256);
  }
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(k_splitk_sgd_batch, dim3(blocks), dim3(256), 0, s, args, splits, opt, status);
  return hipGetLastError();
}

}  // namespace gear
