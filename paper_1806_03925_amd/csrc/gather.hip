// Sparse-Part input: x_b = [user_emb[user_b] | url_emb[url_b] | mean of the view's cached DFVs].
//
// The Dense Part is not evaluated during a step; its outputs are fetched from the cache by image
// id (Section 1, second point; Section 3, steps 1-3).  A page view carries several image ids
// (Section 1); how their DFVs meet the sparse features is in the paper's lost model figure, and is
// taken here as a mean over the view's images.
//
// One wavefront per page view.  A lane owns 16-byte pieces of the row, so a DFV row is read with
// fully coalesced 1 KB wave loads, several images in flight; the sum runs in fp32 in CSR order.
#include "gear_internal.hpp"

namespace gear {
namespace {

constexpr int kMaxPieces = 2;

__device__ __forceinline__ int64_t clamp_id(int32_t id, int64_t n) {
  return id < 0 ? 0 : ((int64_t)id >= n ? n - 1 : (int64_t)id);
}

template <typename ET, typename DT, typename XT>
__global__ void __launch_bounds__(256)
k_gather_pool(int B, int nnz, int d, int D, int64_t n_users, int64_t n_urls, int64_t n_images,
              const int32_t *__restrict__ user_id, const int32_t *__restrict__ url_id,
              const int32_t *__restrict__ img_off, const int32_t *__restrict__ img_id, const ET *__restrict__ user_emb,
              const ET *__restrict__ url_emb, const DT *__restrict__ dfv, XT *__restrict__ x) {
  // The ids are being checked on the helper stream while this kernel runs, so it does not trust
  // them: every id and offset is clamped into its range before it is used as an index.  If one had
  // to be clamped, the check finds it too and the step stops before anything reads this x.
  const int lane = threadIdx.x & (kWave - 1);
  const int view = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave));
  if (view >= B) return;
  const int F = 2 * d + D;
  XT *xrow = x + (size_t)view * F;

  // embeddings: 16-byte pieces of the two rows
  {
    constexpr int EN = Vec16<ET>::N;
    const int pieces = d / EN;  // per table
    for (int p = lane; p < 2 * pieces; p += kWave) {
      const bool second = p >= pieces;
      const int col = (second ? p - pieces : p) * EN;
      const int64_t id = second ? clamp_id(url_id[view], n_urls) : clamp_id(user_id[view], n_users);
      const ET *src = (second ? url_emb : user_emb) + id * d + col;
      Vec16<ET> v;
      v.v = *reinterpret_cast<const decltype(v.v) *>(src);
      XT *dst = xrow + (second ? d : 0) + col;
#pragma unroll
      for (int e = 0; e < EN; ++e) dst[e] = from_f32<XT>(v.get(e));
    }
  }

  // mean of the view's DFV rows: a lane owns up to kMaxPieces 16-byte pieces of the row (columns
  // lane*DN + p*64*DN); the pieces of four rows are requested together, the sum runs in CSR order
  constexpr int DN = Vec16<DT>::N;
  const int lo = min(max(img_off[view], 0), nnz), hi = min(max(img_off[view + 1], lo), nnz);
  const float inv = hi > lo ? 1.0f / (float)(hi - lo) : 0.0f;
  for (int col0 = 0; col0 < D; col0 += kMaxPieces * kWave * DN) {
    float acc[kMaxPieces][DN];
#pragma unroll
    for (int p = 0; p < kMaxPieces; ++p)
#pragma unroll
      for (int e = 0; e < DN; ++e) acc[p][e] = 0.0f;
    for (int j = lo; j < hi; j += 4) {
      Vec16<DT> v[4][kMaxPieces];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t id = j + r < hi ? clamp_id(img_id[j + r], n_images) : -1;
#pragma unroll
        for (int p = 0; p < kMaxPieces; ++p) {
          const int col = col0 + (p * kWave + lane) * DN;
          if (id >= 0 && col < D)
            v[r][p].v = *reinterpret_cast<const decltype(v[r][p].v) *>(dfv + id * D + col);
          else
            v[r][p].v = decltype(v[r][p].v){};
        }
      }
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int p = 0; p < kMaxPieces; ++p)
#pragma unroll
          for (int e = 0; e < DN; ++e) acc[p][e] += v[r][p].get(e);
    }
#pragma unroll
    for (int p = 0; p < kMaxPieces; ++p) {
      const int col = col0 + (p * kWave + lane) * DN;
      if (col < D) {
        XT *dst = xrow + 2 * d + col;
        if constexpr (sizeof(XT) == 2) {
          Vec16<XT> o;
          o.v = decltype(o.v){};
#pragma unroll
          for (int e = 0; e < DN; ++e) o.set(e % 8, acc[p][e] * inv), (void)0;
          if constexpr (DN == 8) {
            *reinterpret_cast<uint4 *>(dst) = o.v;
          } else {  // four values: half a vector
            *reinterpret_cast<uint2 *>(dst) = make_uint2(o.v.x, o.v.y);
          }
        } else {
#pragma unroll
          for (int e = 0; e < DN; e += 4)
            *reinterpret_cast<float4 *>(dst + e) =
                make_float4(acc[p][e] * inv, acc[p][e + 1] * inv, acc[p][e + 2] * inv, acc[p][e + 3] * inv);
        }
      }
    }
  }
}

template <typename ET, typename DT, typename XT>
hipError_t run(const gear_config &cfg, const gear_batch &b, const gear_tables &t, const void *dfv, void *x,
               hipStream_t s) {
  const int waves = 4;
  hipLaunchKernelGGL((k_gather_pool<ET, DT, XT>), dim3((b.B + waves - 1) / waves), dim3(waves * kWave), 0, s, b.B, b.nnz,
                     cfg.emb_dim, cfg.dfv_dim, cfg.n_users, cfg.n_urls, cfg.n_images, b.user_id, b.url_id, b.img_off,
                     b.img_id, (const ET *)t.user_emb, (const ET *)t.url_emb, (const DT *)dfv, (XT *)x);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gather_pool(const gear_config &cfg, const gear_batch &b, const gear_tables &t, const void *dfv,
                              void *x, hipStream_t s) {
  if (b.B <= 0) return hipSuccess;
  const int key = (cfg.emb_dtype << 2) | (cfg.dfv_dtype << 1) | cfg.mlp_dtype;
  switch (key) {
    case 0: return run<float, float, float>(cfg, b, t, dfv, x, s);
    case 1: return run<float, float, bf16_t>(cfg, b, t, dfv, x, s);
    case 2: return run<float, bf16_t, float>(cfg, b, t, dfv, x, s);
    case 3: return run<float, bf16_t, bf16_t>(cfg, b, t, dfv, x, s);
    case 4: return run<bf16_t, float, float>(cfg, b, t, dfv, x, s);
    case 5: return run<bf16_t, float, bf16_t>(cfg, b, t, dfv, x, s);
    case 6: return run<bf16_t, bf16_t, float>(cfg, b, t, dfv, x, s);
    default: return run<bf16_t, bf16_t, bf16_t>(cfg, b, t, dfv, x, s);
  }
}

}  // namespace gear
