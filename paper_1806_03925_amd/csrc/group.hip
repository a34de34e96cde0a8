// Sort-by-key grouping of a step's ids, and the plan of the per-image accumulation.
//
// The Sparse Part's gradients are applied per embedding row (Section 3, step 4) and the DFV
// gradients are collected per image id (Section 3, steps 5-6).  Both need "all positions that
// carry the same id, in their original order": a stable LSD radix sort of (id, position) pairs
// followed by a head-flag scan gives the distinct ids, the segment offsets and the stable
// permutation.  Up to three id lists (users, URLs, images) go through the same launches.
//
// Everything here is integer work whose result does not depend on scheduling: digit counts are
// integer sums, ranks come from wave ballots in lane order, scans run in a fixed shape.
#include "gear_internal.hpp"

namespace gear {
namespace {

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int t = __shfl_up(v, off, kWave);
    if (lane >= off) v += t;
  }
  return v;
}

// exclusive scan of one int per thread over a 256-thread workgroup; *total = sum of all
__device__ __forceinline__ int block_exclusive_scan(int v, int *total, int *smem /* >= 5 ints */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int inc = wave_inclusive_scan(v, lane);
  __syncthreads();  // smem may still be read from a previous call
  if (lane == 63) smem[wave] = inc;
  __syncthreads();
  int base = 0, sum = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const int t = smem[w];
    if (w < wave) base += t;
    sum += t;
  }
  *total = sum;
  return base + inc - v;
}

// sum of tile_vals[0 .. tile) for tile <= 256 * 4, computed by the whole workgroup
__device__ __forceinline__ int sum_before(const int32_t *tile_vals, int tile, int *smem) {
  int v = 0;
  for (int t = threadIdx.x; t < tile; t += blockDim.x) v += tile_vals[t];
  int total;
  block_exclusive_scan(v, &total, smem);
  return total;
}

__device__ __forceinline__ const int32_t *pass_keys(const GroupProblem &p, int pass) {
  return pass == 0 ? p.keys_in : p.keys[pass & 1];
}

// ---- radix pass: per-tile digit histogram ----------------------------------------------------------
__global__ void __launch_bounds__(kSortBlock) k_radix_hist(GroupBatch gb, int pass, const int32_t *status) {
  if (*status != 0) return;
  const GroupProblem &p = gb.p[blockIdx.y];
  if (pass >= p.passes) return;
  const int tile0 = blockIdx.x * kSortTile;
  if (tile0 >= p.n) return;
  __shared__ int hist[kMaxRadix];
  const int radix = 1 << p.digit_bits, shift = pass * p.digit_bits;
  for (int d = threadIdx.x; d < radix; d += kSortBlock) hist[d] = 0;
  __syncthreads();
  const int32_t *keys = pass_keys(p, pass);
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int q = tile0 + i * kSortBlock + threadIdx.x;
    if (q < p.n) atomicAdd(&hist[(keys[q] >> shift) & (radix - 1)], 1);
  }
  __syncthreads();
  for (int d = threadIdx.x; d < radix; d += kSortBlock) p.block_hist[(size_t)blockIdx.x * radix + d] = hist[d];
}

// ---- radix pass: offsets over tiles.  block_hist[t][d] becomes the number of keys with digit d in
// tiles before t; row n_tiles receives the total of digit d.  One workgroup per 64 digits (a lane
// owns a digit); its four waves split a chunk of up to 128 tiles into four contiguous ranges and
// hold their part in registers, so all loads of a chunk are in flight together and nothing is read
// twice (integer sums: any shape gives the same result).
constexpr int kScanPerWave = 32;  // tiles a wave holds at a time
__global__ void __launch_bounds__(256) k_radix_scan(GroupBatch gb, int pass, const int32_t *status) {
  if (*status != 0) return;
  const GroupProblem &p = gb.p[blockIdx.y];
  const int radix = 1 << p.digit_bits;
  if (pass >= p.passes || p.n <= 0 || (int)blockIdx.x * 64 >= radix) return;
  __shared__ int range_sum[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int d = blockIdx.x * 64 + lane;
  const bool live = d < radix;
  const int n_tiles = (p.n + kSortTile - 1) / kSortTile;
  int32_t *col = p.block_hist + (live ? d : 0);
  int carry = 0;  // keys with this digit in the chunks before
  for (int c0 = 0; c0 < n_tiles; c0 += 4 * kScanPerWave) {
    const int chunk = min(n_tiles - c0, 4 * kScanPerWave);
    const int per = (chunk + 3) / 4;
    const int t0 = c0 + min(chunk, wave * per), t1 = c0 + min(chunk, (wave + 1) * per);
    int v[kScanPerWave];
    int sum = 0;
#pragma unroll
    for (int i = 0; i < kScanPerWave; ++i) {
      v[i] = (live && t0 + i < t1) ? col[(size_t)(t0 + i) * radix] : 0;
      sum += v[i];
    }
    __syncthreads();  // range_sum may still be read from the chunk before
    range_sum[wave][lane] = sum;
    __syncthreads();
    int run = carry, total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int r = range_sum[w][lane];
      if (w < wave) run += r;
      total += r;
    }
    carry += total;
#pragma unroll
    for (int i = 0; i < kScanPerWave; ++i) {
      if (live && t0 + i < t1) col[(size_t)(t0 + i) * radix] = run;
      run += v[i];
    }
  }
  if (live && wave == 0) col[(size_t)n_tiles * radix] = carry;  // the digit's total
}

// sum of the four bytes of a word
__device__ __forceinline__ int byte_sum(uint32_t c) {
  return (int)((((c & 0x00ff00ffu) + ((c >> 8) & 0x00ff00ffu)) * 0x00010001u) >> 16);
}

// ---- radix pass: stable scatter ---------------------------------------------------------------------
// A key's place = start of its digit (over all tiles) + keys of that digit in earlier tiles + in
// earlier rounds of this tile + in earlier waves of its round + its rank among the wave's keys of
// that digit (ballots, in lane order).  LDS is kept under 32 KB so that a workgroup fits on a CU
// beside one of the matrix-product kernel.
__global__ void __launch_bounds__(kSortBlock) k_radix_scatter(GroupBatch gb, int pass, const int32_t *status) {
  if (*status != 0) return;
  const GroupProblem &p = gb.p[blockIdx.y];
  if (pass >= p.passes) return;
  const int tile0 = blockIdx.x * kSortTile;
  if (tile0 >= p.n) return;
  __shared__ uint32_t wave_cnt[kSortItems * kMaxRadix];    // [round][digit]: one byte per wave, keys of that digit (<= 64)
  __shared__ uint16_t round_off[kSortItems * kMaxRadix];   // [round][digit]: keys of that digit in earlier rounds (< 2048)
  __shared__ int digit_off[kMaxRadix];
  __shared__ int scan_smem[8];
  static_assert(kSortBlock == 256, "one byte of wave_cnt per wave");
  const int radix = 1 << p.digit_bits, shift = pass * p.digit_bits;
  const int n_tiles = (p.n + kSortTile - 1) / kSortTile;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  for (int i = threadIdx.x; i < kSortItems * radix; i += kSortBlock) wave_cnt[i] = 0u;
  {
    // exclusive scan of the digit totals (radix <= 2 * kSortBlock: two adjacent digits per thread)
    const int d0 = 2 * threadIdx.x, d1 = d0 + 1;
    const int c0 = d0 < radix ? p.block_hist[(size_t)n_tiles * radix + d0] : 0;
    const int c1 = d1 < radix ? p.block_hist[(size_t)n_tiles * radix + d1] : 0;
    int total;
    const int before = block_exclusive_scan(c0 + c1, &total, scan_smem);
    if (d0 < radix) digit_off[d0] = before + p.block_hist[(size_t)blockIdx.x * radix + d0];
    if (d1 < radix) digit_off[d1] = before + c0 + p.block_hist[(size_t)blockIdx.x * radix + d1];
  }
  __syncthreads();

  const int32_t *keys_in = pass_keys(p, pass);
  const int32_t *vals_in = p.vals[pass & 1];
  uint8_t *wave_cnt8 = reinterpret_cast<uint8_t *>(wave_cnt);
  int32_t key[kSortItems], val[kSortItems], rank[kSortItems];
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int q = tile0 + i * kSortBlock + threadIdx.x;
    const bool valid = q < p.n;
    key[i] = valid ? keys_in[q] : 0;
    val[i] = valid ? (pass == 0 ? q : vals_in[q]) : 0;
    const int digit = (key[i] >> shift) & (radix - 1);
    unsigned long long peers = __ballot(valid);
    for (int b = 0; b < p.digit_bits; ++b) {
      const bool bit = (digit >> b) & 1;
      const unsigned long long m = __ballot(bit);
      peers &= bit ? m : ~m;
    }
    rank[i] = __popcll(peers & ((1ull << lane) - 1ull));
    if (valid && rank[i] == 0) wave_cnt8[(i * radix + digit) * 4 + wave] = (uint8_t)__popcll(peers);
  }
  __syncthreads();
  // keys of a digit in the rounds before, for every round
  for (int d = threadIdx.x; d < radix; d += kSortBlock) {
    int run = 0;
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
      round_off[r * radix + d] = (uint16_t)run;
      const uint32_t c = wave_cnt[r * radix + d];
      run += byte_sum(c);
    }
  }
  __syncthreads();
  int32_t *keys_out = p.keys[(pass + 1) & 1];
  int32_t *vals_out = p.vals[(pass + 1) & 1];
  const uint32_t waves_before = wave == 0 ? 0u : (0xffffffffu >> (32 - 8 * wave));
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int q = tile0 + i * kSortBlock + threadIdx.x;
    if (q < p.n) {
      const int digit = (key[i] >> shift) & (radix - 1);
      const int pos = digit_off[digit] + round_off[i * radix + digit] +
                      byte_sum(wave_cnt[i * radix + digit] & waves_before) + rank[i];
      keys_out[pos] = key[i];
      vals_out[pos] = val[i];
    }
  }
}

// ---- segments: head flags over the sorted keys ------------------------------------------------------
// Blocked arrangement: thread t owns positions tile0 + 8 t .. + 7, so a scan keeps position order.
__global__ void __launch_bounds__(kSortBlock) k_seg_count(GroupBatch gb, const int32_t *status) {
  if (*status != 0) return;
  const GroupProblem &p = gb.p[blockIdx.y];
  const int tile0 = blockIdx.x * kSortTile;
  if (tile0 >= p.n) return;
  __shared__ int smem[8];
  const int32_t *sk = p.sorted_keys;
  int heads = 0;
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int q = tile0 + threadIdx.x * kSortItems + i;
    if (q < p.n) heads += (q == 0 || sk[q] != sk[q - 1]) ? 1 : 0;
  }
  int total;
  block_exclusive_scan(heads, &total, smem);
  if (threadIdx.x == 0) p.tile_heads[blockIdx.x] = total;
}

__global__ void __launch_bounds__(kSortBlock) k_seg_scatter(GroupBatch gb, const int32_t *status) {
  if (*status != 0) return;
  const GroupProblem &p = gb.p[blockIdx.y];
  const int tile0 = blockIdx.x * kSortTile;
  if (p.n <= 0) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      *p.n_unique = 0;
      p.segoff[0] = 0;
    }
    return;
  }
  if (tile0 >= p.n) return;
  __shared__ int smem[8];
  const int32_t *sk = p.sorted_keys;
  const int base = sum_before(p.tile_heads, blockIdx.x, smem);
  bool head[kSortItems];
  int mine = 0;
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int q = tile0 + threadIdx.x * kSortItems + i;
    head[i] = q < p.n && (q == 0 || sk[q] != sk[q - 1]);
    mine += head[i] ? 1 : 0;
  }
  int total;
  int idx = base + block_exclusive_scan(mine, &total, smem);
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int q = tile0 + threadIdx.x * kSortItems + i;
    if (q < p.n) {
      if (head[i]) {
        p.unique[idx] = sk[q];
        p.segoff[idx] = q;
        ++idx;
      }
      if (p.pos_seg) p.pos_seg[q] = idx - 1;
    }
  }
  if (tile0 + kSortTile >= p.n && threadIdx.x == 0) {  // last tile
    *p.n_unique = base + total;
    p.segoff[base + total] = p.n;
  }
}

// ---- plan of the windowed accumulation -----------------------------------------------------------------
// Section 1, third point: the gradients of one image are collected until M have arrived, then
// averaged.  With c gradients already collected in earlier steps, the occurrence at in-step rank r
// has ordinal k = c + r; ordinals kM .. kM+M-1 form one group.  A "unit" is the work of one
// workgroup: the first (possibly partial, possibly continuing) group of an image together with its
// unfinished last group, or one complete middle group.  An "emission" is a completed group.
struct UnitFlags {
  bool unit, emit;
};

__device__ __forceinline__ UnitFlags unit_flags(const GroupProblem &p, const int32_t *counts, int M, int q) {
  const int32_t *sk = p.sorted_keys;
  const int i = sk[q];
  const int s0 = p.segoff[p.pos_seg[q]];
  const int k = counts[i] + (q - s0);
  const int ph = k % M;
  UnitFlags f;
  f.unit = (q == s0) || (ph == 0 && M <= p.n - q && sk[q + M - 1] == i);
  f.emit = (ph == M - 1);
  return f;
}

__global__ void __launch_bounds__(kSortBlock) k_plan_count(GroupProblem p, AccumPlan plan, const int32_t *counts,
                                                           int M, const int32_t *status) {
  if (*status != 0) return;
  const int tile0 = blockIdx.x * kSortTile;
  if (tile0 >= p.n) return;
  __shared__ int smem[8];
  int units = 0, emits = 0;
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int q = tile0 + threadIdx.x * kSortItems + i;
    if (q < p.n) {
      const UnitFlags f = unit_flags(p, counts, M, q);
      units += f.unit ? 1 : 0;
      emits += f.emit ? 1 : 0;
    }
  }
  int tu, te;
  block_exclusive_scan(units, &tu, smem);
  block_exclusive_scan(emits, &te, smem);
  if (threadIdx.x == 0) {
    plan.tile_units[blockIdx.x] = tu;
    plan.tile_emits[blockIdx.x] = te;
  }
}

__global__ void __launch_bounds__(kSortBlock) k_plan_scatter(GroupProblem p, AccumPlan plan,
                                                             const int32_t *__restrict__ occ_view,
                                                             const int32_t *__restrict__ img_off,
                                                             const int32_t *counts, int M, int ready_cap,
                                                             int32_t *n_ready, int32_t *status) {
  if (*status != 0) return;
  const int tile0 = blockIdx.x * kSortTile;
  if (p.n <= 0) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      *plan.n_units = 0;
      *n_ready = 0;
    }
    return;
  }
  if (tile0 >= p.n) return;
  __shared__ int smem[8];
  const int base_u = sum_before(plan.tile_units, blockIdx.x, smem);
  const int base_e = sum_before(plan.tile_emits, blockIdx.x, smem);
  UnitFlags f[kSortItems];
  int units = 0, emits = 0;
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int q = tile0 + threadIdx.x * kSortItems + i;
    f[i].unit = f[i].emit = false;
    if (q < p.n) f[i] = unit_flags(p, counts, M, q);
    units += f[i].unit ? 1 : 0;
    emits += f[i].emit ? 1 : 0;
  }
  int tu, te;
  int u = base_u + block_exclusive_scan(units, &tu, smem);
  int e = base_e + block_exclusive_scan(emits, &te, smem);
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int q = tile0 + threadIdx.x * kSortItems + i;
    if (q < p.n) {
      // where the occurrence's gradient lives: dLoss/dx of its view, divided by the view's image count
      const int view = occ_view[p.perm[q]];
      plan.row_view[q] = view;
      plan.row_scale[q] = 1.0f / (float)(img_off[view + 1] - img_off[view]);
      if (f[i].unit) {
        const int seg = p.pos_seg[q];
        const int image = p.sorted_keys[q];
        UnitDesc d;
        d.q0 = q;
        d.image = image;
        d.slot = e;
        d.s0 = p.segoff[seg];
        d.s1 = p.segoff[seg + 1];
        d.phase = counts[image] % M;
        d.pad[0] = d.pad[1] = 0;
        plan.units[u] = d;
        ++u;
      }
      if (f[i].emit) ++e;
    }
  }
  if (tile0 + kSortTile >= p.n && threadIdx.x == 0) {
    *plan.n_units = base_u + tu;
    // a list that does not fit is reported as empty: nobody may read ready_ids past ready_cap
    const bool over = base_e + te > ready_cap;
    *n_ready = over ? 0 : base_e + te;
    if (over) atomicCAS(status, 0, GEAR_ERR_CAPACITY);
  }
}

// ---- expiry of cached inference results ------------------------------------------------------------
// Every occurrence whose cached row is old writes a 1 into its image's byte of a map over all images
// (a plain store of the same value, whoever comes first; an atomic OR into a bitmap was tried and
// spent 260 us on the thousands of occurrences of the most popular image, all aimed at one word);
// the marked bytes are then counted per tile and written out in ascending order at the tile's
// offset.  No sort is needed: the map is already in id order.
__device__ __forceinline__ bool is_expired(const int32_t *__restrict__ stamp, int64_t n_images, int id, int32_t now,
                                           int32_t expiry, int32_t *status) {
  if (id < 0 || id >= n_images) {
    atomicCAS(status, 0, GEAR_ERR_RANGE);
    return false;
  }
  return (int64_t)now - (int64_t)stamp[id] >= (int64_t)expiry;
}

__global__ void __launch_bounds__(256) k_expired_mark(const int32_t *__restrict__ ids, int n,
                                                      const int32_t *__restrict__ stamp, int64_t n_images, int32_t now,
                                                      int32_t expiry, uint8_t *__restrict__ marks, int32_t *status) {
  for (int r = blockIdx.x * blockDim.x + threadIdx.x; r < n; r += gridDim.x * blockDim.x) {
    const int id = ids[r];
    if (is_expired(stamp, n_images, id, now, expiry, status)) marks[id] = 1;
  }
}

// The map is read as words of four images; thread t of a tile owns the words tile0 + 8 t .. + 7, so a
// scan keeps id order.  The map is padded with zeros to a whole number of words.
__global__ void __launch_bounds__(kSortBlock) k_expired_count(const uint32_t *__restrict__ marks, int64_t n_words,
                                                              int32_t *__restrict__ tile_counts) {
  const int64_t tile0 = (int64_t)blockIdx.x * kSortTile;
  __shared__ int smem[8];
  int c = 0;
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int64_t w = tile0 + threadIdx.x * kSortItems + i;
    if (w < n_words) c += __popc(marks[w]);
  }
  int total;
  block_exclusive_scan(c, &total, smem);
  if (threadIdx.x == 0) tile_counts[blockIdx.x] = total;
}

__global__ void __launch_bounds__(kSortBlock) k_expired_scatter(const uint32_t *__restrict__ marks, int64_t n_words,
                                                                const int32_t *__restrict__ tile_counts,
                                                                int32_t *__restrict__ out_ids, int32_t *n_out,
                                                                const int32_t *status) {
  const int64_t tile0 = (int64_t)blockIdx.x * kSortTile;
  __shared__ int smem[8];
  const int base = sum_before(tile_counts, blockIdx.x, smem);
  uint32_t word[kSortItems];
  int c = 0;
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int64_t w = tile0 + threadIdx.x * kSortItems + i;
    word[i] = w < n_words ? marks[w] : 0u;
    c += __popc(word[i]);
  }
  int total;
  int at = base + block_exclusive_scan(c, &total, smem);
  const bool bad = *status != 0;   // set by the marking pass, which saw every id: the list is then empty
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int64_t w = tile0 + threadIdx.x * kSortItems + i;
#pragma unroll
    for (int byte = 0; byte < 4; ++byte)
      if (word[i] & (1u << (8 * byte))) {
        if (!bad) out_ids[at] = (int32_t)(w * 4 + byte);
        ++at;
      }
  }
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) *n_out = bad ? 0 : base + total;
}

__global__ void __launch_bounds__(256) k_stamp(int32_t *__restrict__ stamp, int64_t n_images,
                                               const int32_t *__restrict__ ids, int64_t n, int32_t now, int32_t *status,
                                               const int32_t *__restrict__ n_dev) {
  if (n_dev) n = min((int64_t)max(*n_dev, 0), n);  // the row count is only known on the device
  for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n; r += (int64_t)gridDim.x * blockDim.x) {
    const int64_t id = ids ? (int64_t)ids[r] : r;
    if (id < 0 || id >= n_images) {
      if (status) atomicCAS(status, 0, GEAR_ERR_RANGE);
      continue;
    }
    stamp[id] = now;
  }
}

}  // namespace

hipError_t launch_expired(const int32_t *image_ids, int n, const int32_t *stamp, int64_t n_images, int32_t now,
                          int32_t expiry, uint8_t *marks, int32_t *tile_counts, int32_t *out_ids, int32_t *n_out,
                          int32_t *status, hipStream_t s) {
  const int64_t n_words = expiry_words(n_images);
  hipError_t e = launch_fill_zero(marks, (size_t)n_words * sizeof(uint32_t), s);
  if (e != hipSuccess) return e;
  if (n > 0) {
    int blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_expired_mark, dim3(blocks), dim3(256), 0, s, image_ids, n, stamp, n_images, now, expiry, marks,
                       status);
  }
  const int tiles = (int)expiry_tiles(n_images);
  hipLaunchKernelGGL(k_expired_count, dim3(tiles), dim3(kSortBlock), 0, s, (const uint32_t *)marks, n_words,
                     tile_counts);
  hipLaunchKernelGGL(k_expired_scatter, dim3(tiles), dim3(kSortBlock), 0, s, (const uint32_t *)marks, n_words,
                     tile_counts, out_ids, n_out, status);
  return hipGetLastError();
}

hipError_t launch_stamp(int32_t *stamp, int64_t n_images, const int32_t *ids, int64_t n, int32_t now, int32_t *status,
                        hipStream_t s, const int32_t *n_dev) {
  if (n <= 0) return hipSuccess;
  int64_t want = (n + 255) / 256;
  const int blocks = (int)(want < 4096 ? want : 4096);
  hipLaunchKernelGGL(k_stamp, dim3(blocks), dim3(256), 0, s, stamp, n_images, ids, n, now, status, n_dev);
  return hipGetLastError();
}

hipError_t launch_group(const GroupBatch &gb, const int32_t *status, hipStream_t s) {
  int max_tiles = 1, max_passes = 0;
  for (int i = 0; i < gb.count; ++i) {
    const int t = (gb.p[i].n + kSortTile - 1) / kSortTile;
    if (t > max_tiles) max_tiles = t;
    if (gb.p[i].n > 0 && gb.p[i].passes > max_passes) max_passes = gb.p[i].passes;
  }
  const dim3 grid(max_tiles, gb.count);
  for (int pass = 0; pass < max_passes; ++pass) {
    hipLaunchKernelGGL(k_radix_hist, grid, dim3(kSortBlock), 0, s, gb, pass, status);
    hipLaunchKernelGGL(k_radix_scan, dim3(kMaxRadix / 64, gb.count), dim3(256), 0, s, gb, pass, status);
    hipLaunchKernelGGL(k_radix_scatter, grid, dim3(kSortBlock), 0, s, gb, pass, status);
  }
  hipLaunchKernelGGL(k_seg_count, grid, dim3(kSortBlock), 0, s, gb, status);
  hipLaunchKernelGGL(k_seg_scatter, grid, dim3(kSortBlock), 0, s, gb, status);
  return hipGetLastError();
}

hipError_t launch_accum_plan(const GroupProblem &img, const AccumPlan &plan, const int32_t *occ_view,
                             const int32_t *img_off, const int32_t *counts, int32_t M, int32_t ready_cap,
                             int32_t *n_ready, int32_t *status, hipStream_t s) {
  int tiles = (img.n + kSortTile - 1) / kSortTile;
  if (tiles < 1) tiles = 1;
  hipLaunchKernelGGL(k_plan_count, dim3(tiles), dim3(kSortBlock), 0, s, img, plan, counts, M, status);
  hipLaunchKernelGGL(k_plan_scatter, dim3(tiles), dim3(kSortBlock), 0, s, img, plan, occ_view, img_off, counts, M,
                     ready_cap, n_ready, status);
  return hipGetLastError();
}

}  // namespace gear
