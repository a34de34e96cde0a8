// Internal declarations shared by the libgear translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "gear.h"

namespace gear {

// ------------------------------------------------------------------------------------------------
// storage types
// ------------------------------------------------------------------------------------------------
using bf16_t = uint16_t;  // raw bfloat16 bits: sign, 8 exponent bits, 7 fraction bits

__host__ __device__ inline size_t dtype_bytes(int dt) { return dt == GEAR_BF16 ? 2 : 4; }

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round to nearest, ties to even
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// two floats -> two bf16 in one word (round to nearest even, one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// How a gradient changes a parameter (Section 3, step 4 applies the Sparse Part's gradients every
// step; Section 4.1 trains with Adam).  SGD: w -= lr g.  Adam (Kingma & Ba, Algorithm 1):
// m = b1 m + (1 - b1) g, v = b2 v + (1 - b2) g^2, w -= lr / (1 - b1^t) * m / (sqrt(v) / sqrt(1 - b2^t) + eps);
// the two factors that depend on t are computed by the host.
struct Optim {
  float lr;        // SGD: the rate.  Adam: lr / (1 - beta1^t)
  float beta1, beta2, eps;
  float inv_bc2;   // Adam: 1 / sqrt(1 - beta2^t)
  int32_t adam;    // 0 = SGD
};
struct Moments {   // first and second moment arrays of the same shape as the parameters; null for SGD
  float *m, *v;
};
__host__ __device__ __forceinline__ Moments moments_at(const Moments &base, ptrdiff_t offset) {
  Moments r = {base.m ? base.m + offset : nullptr, base.v ? base.v + offset : nullptr};
  return r;
}
__device__ __forceinline__ float optim_apply(const Optim &o, float w, float g, float *m, float *v) {
  if (!o.adam) return w - o.lr * g;
  const float mn = o.beta1 * *m + (1.0f - o.beta1) * g;
  const float vn = o.beta2 * *v + (1.0f - o.beta2) * g * g;
  *m = mn;
  *v = vn;
  return w - o.lr * mn / (sqrtf(vn) * o.inv_bc2 + o.eps);
}

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

// 16-byte vector of T
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  float4 v;
  __device__ __forceinline__ float get(int i) const { return (&v.x)[i]; }
  __device__ __forceinline__ void set(int i, float f) { (&v.x)[i] = f; }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  uint4 v;
  __device__ __forceinline__ float get(int i) const {
    uint32_t w = (&v.x)[i >> 1];
    return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
  }
  __device__ __forceinline__ void set(int i, float f) {
    uint32_t b = f32_to_bf16(f);
    uint32_t &w = (&v.x)[i >> 1];
    w = (i & 1) ? ((w & 0x0000ffffu) | (b << 16)) : ((w & 0xffff0000u) | b);
  }
};

constexpr int kWave = 64;

// ------------------------------------------------------------------------------------------------
// grouping (sort by key + segments) problem descriptors
// ------------------------------------------------------------------------------------------------
constexpr int kSortBlock = 256;                       // threads
constexpr int kSortItems = 8;                         // keys per thread
constexpr int kSortTile = kSortBlock * kSortItems;    // keys per workgroup
constexpr int kMaxRadixBits = 9;
constexpr int kMaxRadix = 1 << kMaxRadixBits;
constexpr int kMaxProblems = 3;

struct GroupProblem {
  const int32_t *keys_in;  // [n] original keys (read by the first pass)
  int32_t n;
  int32_t key_bits;        // significant bits of a key
  int32_t passes;          // radix passes
  int32_t digit_bits;      // bits per pass
  int32_t *keys[2];        // ping-pong key buffers [n]
  int32_t *vals[2];        // ping-pong position buffers [n]
  int32_t *block_hist;     // [n_tiles x radix] digit counts per tile, then exclusive offsets
  int32_t *sorted_keys;    // = keys[passes & 1]
  int32_t *perm;           // = vals[passes & 1]
  int32_t *tile_heads;     // [n_tiles] number of segment heads per tile
  int32_t *unique;         // [n]   distinct keys ascending
  int32_t *segoff;         // [n+1] segment offsets
  int32_t *pos_seg;        // [n]   segment index of each sorted position (may be NULL)
  int32_t *n_unique;       // [1]
};

struct GroupBatch {
  GroupProblem p[kMaxProblems];
  int32_t count;
};

// plan of the windowed accumulation over the sorted image occurrences
struct UnitDesc {         // one workgroup's share of the accumulation (32 bytes)
  int32_t q0;             // first sorted position of the unit
  int32_t image;          // image id
  int32_t slot;           // ready-list slot of the unit's (first) emission
  int32_t s0, s1;         // the image's range of sorted positions
  int32_t phase;          // gradients already collected for the image before this step, modulo M
  int32_t pad[2];
};

struct AccumPlan {
  int32_t *tile_units;   // [n_tiles] unit heads per tile
  int32_t *tile_emits;   // [n_tiles] completed groups per tile
  UnitDesc *units;       // [nnz]
  int32_t *row_view;     // [nnz] view that owns the occurrence at each sorted position
  float *row_scale;      // [nnz] 1 / (images of that view): backward of the mean
  int32_t *n_units;      // [1]
};

// ------------------------------------------------------------------------------------------------
// workspace layout (byte offsets from a 256-byte aligned base)
// ------------------------------------------------------------------------------------------------
struct Layout {
  int32_t F;                         // MLP input width
  int32_t L;                         // layers
  int32_t in_dim[GEAR_MAX_LAYERS];   // input width of each layer
  int32_t out_dim[GEAR_MAX_LAYERS];
  int64_t w_off[GEAR_MAX_LAYERS];    // float offsets into mlp_params
  int64_t b_off[GEAR_MAX_LAYERS];
  int64_t n_params;
  int32_t splitk[GEAR_MAX_LAYERS];   // wgrad split count per layer
  int32_t colsum_chunks;             // row chunks of the column-sum kernels
  size_t act_bytes;                  // sizeof(mlp_dtype)

  size_t x, h[GEAR_MAX_LAYERS], delta[GEAR_MAX_LAYERS], logits, dz, loss_partial, dx_emb, dx_dfv;
  size_t relu_bits[GEAR_MAX_LAYERS];  // [B x out/8] sign bitmaps of the hidden activations
  size_t wc[GEAR_MAX_LAYERS], wct[GEAR_MAX_LAYERS], wgrad_partial, colsum_partial, emb_partial;
  size_t colsum_stride;              // floats between the column-sum partials of consecutive layers
  size_t wgrad_partial_bytes;        // size of the split-K partial region
  size_t occ_view;
  struct G {
    size_t keys[2], vals[2], block_hist, tile_heads, unique, segoff, pos_seg, n_unique;
  } g[kMaxProblems];
  size_t tile_units, tile_emits, units, row_view, row_scale, n_units;
  size_t expiry_marks, expiry_tiles;  // gear_expired_ids: byte map over the images, marked bytes per tile
  size_t total;
};

bool make_layout(const gear_config &cfg, Layout *lay);
bool config_ok(const gear_config &cfg);

constexpr int kColsumRows = 128;     // rows per partial of a column sum
constexpr int kLossBlocks = 2048;    // most workgroups (and partial sums) of the logit/loss kernel

// ------------------------------------------------------------------------------------------------
// kernel launchers (each defined next to its kernel)
// ------------------------------------------------------------------------------------------------
hipError_t launch_fill_normal(void *dst, int dtype, int64_t n_elems, uint64_t seed, uint32_t stream_id,
                              float std, hipStream_t s);
hipError_t launch_fill_zero(void *dst, size_t bytes, hipStream_t s);

hipError_t launch_begin(int32_t *status, int32_t *n_ready, float *loss, hipStream_t s);
hipError_t launch_validate(const gear_config &cfg, const gear_batch &b, int32_t *occ_view, int32_t *status,
                           hipStream_t s);

hipError_t launch_group(const GroupBatch &gb, const int32_t *status, hipStream_t s);
// distinct ids of a grouped list whose cache entry is older than `expiry`, ascending
// words (four images each) of the byte map over all images that the expiry filter marks, and tiles
// of kSortTile words
inline int64_t expiry_words(int64_t n_images) { return (n_images + 3) / 4; }
inline int64_t expiry_tiles(int64_t n_images) { return (expiry_words(n_images) + kSortTile - 1) / kSortTile; }
hipError_t launch_expired(const int32_t *image_ids, int n, const int32_t *stamp, int64_t n_images, int32_t now,
                          int32_t expiry, uint8_t *marks, int32_t *tile_counts, int32_t *out_ids, int32_t *n_out,
                          int32_t *status, hipStream_t s);
hipError_t launch_stamp(int32_t *stamp, int64_t n_images, const int32_t *ids, int64_t n, int32_t now, int32_t *status,
                        hipStream_t s, const int32_t *n_dev = nullptr);
hipError_t launch_accum_plan(const GroupProblem &img, const AccumPlan &plan, const int32_t *occ_view,
                             const int32_t *img_off, const int32_t *counts, int32_t M, int32_t ready_cap,
                             int32_t *n_ready, int32_t *status, hipStream_t s);

hipError_t launch_gather_pool(const gear_config &cfg, const gear_batch &b, const gear_tables &t,
                              const void *dfv_cache, void *x, hipStream_t s);

hipError_t launch_cast_weights(int count, const float *const *w, const int *rows, const int *cols, int dtype,
                               void *const *wc, void *const *wct, const int32_t *status, hipStream_t s);

enum GemmEpilogue {
  EPI_BIAS_RELU = 0,  // out(T)   = max(acc + bias[n], 0)
  EPI_MASK = 1,       // out(T)   = aux[m,n] > 0 ? acc : 0
  EPI_F32 = 2,        // out(f32) = acc
  EPI_DX = 3,         // columns < split: out(f32)[M x split] = acc; others: aux(T)[M x (N - split)] = acc
  EPI_MASK_BITS = 4,  // EPI_MASK with aux = the bitmap [M x N/8] an EPI_BIAS_RELU product left in `relu_bits`
};
// C[M x N] = A[M x K] * B[N x K]^T, both operands K-contiguous, type `dtype`.
// relu_bits (EPI_BIAS_RELU only, may be NULL): bit (n % 8) of byte [m][n / 8] = (out[m][n] > 0); only
// written by the kernel gemm_nt_has_bits() names, which is also the only one that takes EPI_MASK_BITS.
hipError_t launch_gemm_nt(int dtype, const void *A, const void *B, int M, int N, int K, int epilogue,
                          const float *bias, const void *aux, void *out, int split, float *colpart,
                          uint8_t *relu_bits, const int32_t *status, hipStream_t s);
int gemm_nt_colsum_parts(int dtype, int M, int N, int K);
bool gemm_nt_has_bits(int dtype, int K);
// dst[j] -= lr * sum_p partial[p][j], p ascending in a fixed two-level shape
hipError_t launch_partial_sgd(const float *partial, int P, int H, float *dst, const Optim &opt, const Moments &mom,
                              const int32_t *status, hipStream_t s);
// partial[z][M x N] = sum over the z-th K range of A[K x M]^T * B[K x N] (operands M-/N-contiguous).
// k_dev (may be NULL): device word holding the real contraction length, at most K; the split into
// `splits` ranges is then made on the device.
hipError_t launch_gemm_tn_splitk(int dtype, const void *A, const void *B, int M, int N, int K, int splits,
                                 float *partial, const int32_t *status, hipStream_t s, const int32_t *k_dev = nullptr);
int gemm_splitk_for(int dtype, int M, int N, int K);  // wgrad split count for a [M x N] result contracted over K
int gemm_splitk_max(int dtype, int M, int N, int K);  // the largest such count over all contraction lengths up to K
// Several such contractions over the same K rows of bf16 operands in one launch, all with the same
// number of k-ranges: partial_i[z][M_i x N_i].  gemm_tn_batch_splits gives that number (it looks at
// M and N only), or 0 if the set has to go through one launch per problem.
struct TnProblem {
  const void *A, *B;
  float *partial;
  int M, N;
};
int gemm_tn_batch_splits(int dtype, const TnProblem *p, int count, int K);
hipError_t launch_gemm_tn_batch(const TnProblem *p, int count, int K, int splits, const int32_t *status,
                                hipStream_t s);
// w_i <- update(w_i, sum_z partial_i[z]) for the results of such a launch, in one launch
struct SplitkProblem {
  const float *partial;
  float *w;
  Moments mom;
  int64_t count;
};
hipError_t launch_splitk_sgd_batch(const SplitkProblem *p, int count, int splits, const Optim &opt,
                                   const int32_t *status, hipStream_t s);
hipError_t launch_splitk_sgd(const float *partial, int splits, int64_t count, float *w, const Optim &opt,
                             const Moments &mom, const int32_t *status, hipStream_t s);

hipError_t launch_logit_loss(int dtype, const void *h, const void *wc_last, const float *bias_last, const float *label,
                             int B, int H, float *logits, float *dz, void *delta, float *partials,
                             const int32_t *status, hipStream_t s);
hipError_t launch_logit_finish(float *partials, int B, int H, float *w_last, float *bias_last, float *bias_hidden,
                               float *loss, const Optim &opt, const Moments &mom_w_last, const Moments &mom_bias_last,
                               const Moments &mom_bias_hidden, const int32_t *status, hipStream_t s);
size_t logit_partial_floats(int H);

hipError_t launch_colsum_sgd(int dtype, const void *src, int B, int H, float *partial, float *dst, const Optim &opt,
                             const Moments &mom, const int32_t *status, hipStream_t s);

hipError_t launch_embedding_update(const gear_config &cfg, const GroupProblem &users, const GroupProblem &urls,
                                   const float *dx_emb, void *user_emb, void *url_emb, float *partials,
                                   const Optim &opt, const Moments &mom_user, const Moments &mom_url,
                                   const int32_t *status, hipStream_t s);
size_t embedding_partial_floats(const gear_config &cfg);

hipError_t launch_accumulate(const gear_config &cfg, const GroupProblem &img, const AccumPlan &plan,
                             const void *dx_dfv, float *grad_accum, int32_t M, int32_t *ready_ids,
                             float *ready_grads, const int32_t *status, hipStream_t s);
hipError_t launch_count_update(const GroupProblem &img, int32_t *counts, const int32_t *status, hipStream_t s);

// n_dev (may be NULL): device word holding the real row count, at most n
hipError_t launch_refresh(int dtype, void *dfv_cache, int64_t n_images, int dim, const int32_t *ids,
                          const void *rows, int64_t n, int32_t *status, hipStream_t s, const int32_t *n_dev = nullptr);

}  // namespace gear
