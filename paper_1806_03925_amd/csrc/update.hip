// SGD on the touched embedding rows (Section 3, step 4: the Fastgear Worker applies the Sparse
// Part's gradients every step).
//
// The gradient of a row is the sum of dLoss/dx over the views that used it.  After the stable
// sort by id those views are a run of the sorted positions, ascending in batch position.  Zipf
// traffic makes a few runs thousands of views long, so the sum has a fixed two-level shape that
// depends on the data only, never on scheduling: the sorted positions are cut into chunks of kChunk
// and a worker adds the rows of its chunk run by run, in order.  A run that lies inside one
// chunk is finished on the spot (one read-modify-write of the row).  A run that crosses chunk
// borders leaves one partial per chunk; the worker of the chunk where the run starts then adds
// those partials in chunk order and writes the row.  No atomics anywhere.
//
// A worker is d/4 lanes, each owning one float4 column group of the row.
#include "gear_internal.hpp"

#include <type_traits>

namespace gear {
namespace {

constexpr int kChunk = 16;

struct Table {
  const int32_t *keys;   // sorted ids
  const int32_t *perm;   // batch position of each sorted position
  int n;
  void *rows;            // embedding table
  int col0;              // first column of this table's slice inside a dx row
  float *part_first;     // [chunks x d] partial of a run that began in an earlier chunk
  float *part_last;      // [chunks x d] partial of a run that begins here and goes on
  Moments mom;           // Adam: fp32 moment tables of the same shape as `rows` (only touched rows move)
};

// one float4 column group of a row: row <- update(row, g); mrow / vrow are the row's moments (Adam)
template <typename ET>
__device__ __forceinline__ void apply_row(ET *row, float *mrow, float *vrow, int c4, float4 g, const Optim &o) {
  float4 m = make_float4(0.f, 0.f, 0.f, 0.f), v = m;
  if (o.adam) {
    m = reinterpret_cast<float4 *>(mrow)[c4];
    v = reinterpret_cast<float4 *>(vrow)[c4];
  }
  if constexpr (sizeof(ET) == 4) {
    float4 *cell = reinterpret_cast<float4 *>(row) + c4;
    float4 w = *cell;
    w.x = optim_apply(o, w.x, g.x, &m.x, &v.x);
    w.y = optim_apply(o, w.y, g.y, &m.y, &v.y);
    w.z = optim_apply(o, w.z, g.z, &m.z, &v.z);
    w.w = optim_apply(o, w.w, g.w, &m.w, &v.w);
    *cell = w;
  } else {
    uint2 *cell = reinterpret_cast<uint2 *>(row) + c4;
    uint2 w = *cell;
    const float a = optim_apply(o, __uint_as_float(w.x << 16), g.x, &m.x, &v.x);
    const float b = optim_apply(o, __uint_as_float(w.x & 0xffff0000u), g.y, &m.y, &v.y);
    const float c = optim_apply(o, __uint_as_float(w.y << 16), g.z, &m.z, &v.z);
    const float d = optim_apply(o, __uint_as_float(w.y & 0xffff0000u), g.w, &m.w, &v.w);
    w.x = (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
    w.y = (uint32_t)f32_to_bf16(c) | ((uint32_t)f32_to_bf16(d) << 16);
    *cell = w;
  }
  if (o.adam) {
    reinterpret_cast<float4 *>(mrow)[c4] = m;
    reinterpret_cast<float4 *>(vrow)[c4] = v;
  }
}

__device__ __forceinline__ void add4(float4 &a, const float4 &b) {
  a.x += b.x;
  a.y += b.y;
  a.z += b.z;
  a.w += b.w;
}

// level 1: one worker per chunk of sorted positions
template <typename ET>
__global__ void __launch_bounds__(256)
k_embedding_chunks(Table users, Table urls, const float *__restrict__ dx, int F, int d, int lanes_per_worker, Optim opt,
                   const int32_t *__restrict__ status) {
  if (*status != 0) return;
  const Table &t = blockIdx.y == 1 ? urls : users;
  const int tid = blockIdx.x * blockDim.x + threadIdx.x;
  const int chunk = tid / lanes_per_worker, c4 = tid % lanes_per_worker;
  const int q_begin = chunk * kChunk;
  if (q_begin >= t.n || c4 >= d / 4) return;
  const int q_end = min(t.n, q_begin + kChunk);
  const float *col = dx + t.col0 + 4 * c4;

  // ids, batch positions and rows of the whole chunk first, so that all loads are in flight at once
  int keys[kChunk + 1], pos[kChunk];
#pragma unroll
  for (int i = 0; i < kChunk; ++i) {
    const int q = q_begin + i;
    keys[i] = q < t.n ? t.keys[q] : -1;
    pos[i] = q < t.n ? t.perm[q] : 0;
  }
  keys[kChunk] = q_begin + kChunk < t.n ? t.keys[q_begin + kChunk] : -1;
  float4 row[kChunk];
#pragma unroll
  for (int i = 0; i < kChunk; ++i)
    row[i] = q_begin + i < q_end ? *reinterpret_cast<const float4 *>(col + (size_t)pos[i] * F)
                                 : make_float4(0.f, 0.f, 0.f, 0.f);

  // running sums inside each run, in place and in order: row[i] becomes the sum of its run so far
#pragma unroll
  for (int i = 1; i < kChunk; ++i)
    if (q_begin + i < q_end && keys[i] == keys[i - 1]) {
      float4 sum = row[i - 1];
      add4(sum, row[i]);
      row[i] = sum;
    }
  // A run is complete here when it starts and ends inside the chunk; the first run may have begun in
  // an earlier chunk, the last one may go on into the next.
  const bool first_starts_here = q_begin == 0 || t.keys[q_begin - 1] != keys[0];
  bool whole[kChunk];
#pragma unroll
  for (int i = 0; i < kChunk; ++i) {
    const bool in = q_begin + i < q_end;
    const bool ends_here = keys[i + 1] != keys[i];
    const bool starts_here = keys[i] != keys[0] || first_starts_here;
    whole[i] = in && ends_here && starts_here;
    if (in && !whole[i] && (ends_here || q_begin + i + 1 == q_end)) {
      float *dst = (starts_here ? t.part_last : t.part_first) + (size_t)chunk * d;
      *reinterpret_cast<float4 *>(dst + 4 * c4) = row[i];
    }
  }
  if (opt.adam) {
#pragma unroll
    for (int i = 0; i < kChunk; ++i)
      if (whole[i]) {
        const size_t at = (size_t)keys[i] * d;
        apply_row<ET>(static_cast<ET *>(t.rows) + at, t.mom.m + at, t.mom.v + at, c4, row[i], opt);
      }
    return;
  }
  // Plain SGD: the rows of all complete runs are requested together, then updated and written back
  // (ids in a sorted chunk are distinct per run, so no two of these cells are the same).  One after
  // the other, each waiting for its own load, sixteen rows cost sixteen memory latencies.
  using Cell = typename std::conditional<sizeof(ET) == 4, float4, uint2>::type;
  Cell w[kChunk];
#pragma unroll
  for (int i = 0; i < kChunk; ++i)
    if (whole[i]) w[i] = reinterpret_cast<const Cell *>(static_cast<const ET *>(t.rows) + (size_t)keys[i] * d)[c4];
#pragma unroll
  for (int i = 0; i < kChunk; ++i)
    if (whole[i]) {
      Cell *cell = reinterpret_cast<Cell *>(static_cast<ET *>(t.rows) + (size_t)keys[i] * d) + c4;
      const float4 g = row[i];
      if constexpr (sizeof(ET) == 4) {
        *cell = make_float4(w[i].x - opt.lr * g.x, w[i].y - opt.lr * g.y, w[i].z - opt.lr * g.z, w[i].w - opt.lr * g.w);
      } else {
        const float a = __uint_as_float(w[i].x << 16) - opt.lr * g.x, b = __uint_as_float(w[i].x & 0xffff0000u) - opt.lr * g.y;
        const float c = __uint_as_float(w[i].y << 16) - opt.lr * g.z, e = __uint_as_float(w[i].y & 0xffff0000u) - opt.lr * g.w;
        *cell = make_uint2((uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16),
                           (uint32_t)f32_to_bf16(c) | ((uint32_t)f32_to_bf16(e) << 16));
      }
    }
}

constexpr int kSpanInFlight = 32;   // partials of a long run that one lane has in flight

// level 2: one wavefront per chunk; if a border-crossing run starts in this chunk the wave adds
// the run's partials in chunk order (lane = column) and writes the row
template <typename ET>
__global__ void __launch_bounds__(256)
k_embedding_spans(Table users, Table urls, const int32_t *__restrict__ user_pos_seg,
                  const int32_t *__restrict__ user_segoff, const int32_t *__restrict__ url_pos_seg,
                  const int32_t *__restrict__ url_segoff, int d, Optim opt, const int32_t *__restrict__ status) {
  if (*status != 0) return;
  const bool second = blockIdx.y == 1;
  const Table &t = second ? urls : users;
  const int32_t *pos_seg = second ? url_pos_seg : user_pos_seg;
  const int32_t *segoff = second ? url_segoff : user_segoff;
  const int lane = threadIdx.x & 63;
  const int chunk = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int q_begin = chunk * kChunk;
  if (q_begin >= t.n) return;
  const int q_last = min(t.n, q_begin + kChunk) - 1;
  if (q_last + 1 >= t.n) return;              // nothing after this chunk
  const int key = t.keys[q_last];
  if (t.keys[q_last + 1] != key) return;      // the last run ends inside this chunk
  const int seg = pos_seg[q_last];
  const int s0 = segoff[seg], s1 = segoff[seg + 1];
  if (s0 < q_begin) return;                   // the run began in an earlier chunk: not ours
  const int k_last = (s1 - 1) / kChunk;
  for (int c = lane; c < d; c += kWave) {
    float sum = t.part_last[(size_t)chunk * d + c];
    int k = chunk + 1;
    for (; k + kSpanInFlight <= k_last + 1; k += kSpanInFlight) {   // added in order, requested together
      float v[kSpanInFlight];
#pragma unroll
      for (int i = 0; i < kSpanInFlight; ++i) v[i] = t.part_first[(size_t)(k + i) * d + c];
#pragma unroll
      for (int i = 0; i < kSpanInFlight; ++i) sum += v[i];
    }
    for (; k <= k_last; ++k) sum += t.part_first[(size_t)k * d + c];
    const size_t at = (size_t)key * d + c;
    ET *cell = static_cast<ET *>(t.rows) + at;
    *cell = from_f32<ET>(optim_apply(opt, to_f32<ET>(*cell), sum, t.mom.m + at, t.mom.v + at));
  }
}

}  // namespace

hipError_t launch_embedding_update(const gear_config &cfg, const GroupProblem &users, const GroupProblem &urls,
                                   const float *dx, void *user_emb, void *url_emb, float *partials,
                                   const Optim &opt, const Moments &mom_user, const Moments &mom_url,
                                   const int32_t *status, hipStream_t s) {
  const int F = 2 * cfg.emb_dim;  // dx holds the two embedding slots of dLoss/dx only
  const int n = users.n > urls.n ? users.n : urls.n;
  if (n <= 0) return hipSuccess;
  const int d = cfg.emb_dim;
  int lanes = 1;
  while (lanes < d / 4) lanes <<= 1;  // power of two so that workers do not straddle wavefronts
  const int chunks = (n + kChunk - 1) / kChunk;
  const size_t per = (size_t)((cfg.max_batch + kChunk - 1) / kChunk) * d;
  Table tu = {users.sorted_keys, users.perm, users.n, user_emb, 0, partials, partials + per, mom_user};
  Table tl = {urls.sorted_keys, urls.perm, urls.n, url_emb, d, partials + 2 * per, partials + 3 * per, mom_url};
  const long long threads = (long long)chunks * lanes;
  const dim3 grid((unsigned)((threads + 255) / 256), 2);
  const dim3 grid2((chunks + 3) / 4, 2);
  if (cfg.emb_dtype == GEAR_BF16) {
    hipLaunchKernelGGL(k_embedding_chunks<bf16_t>, grid, dim3(256), 0, s, tu, tl, dx, F, d, lanes, opt, status);
    hipLaunchKernelGGL(k_embedding_spans<bf16_t>, grid2, dim3(256), 0, s, tu, tl, users.pos_seg, users.segoff,
                       urls.pos_seg, urls.segoff, d, opt, status);
  } else {
    hipLaunchKernelGGL(k_embedding_chunks<float>, grid, dim3(256), 0, s, tu, tl, dx, F, d, lanes, opt, status);
    hipLaunchKernelGGL(k_embedding_spans<float>, grid2, dim3(256), 0, s, tu, tl, users.pos_seg, users.segoff,
                       urls.pos_seg, urls.segoff, d, opt, status);
  }
  return hipGetLastError();
}

size_t embedding_partial_floats(const gear_config &cfg) {
  return 4 * (size_t)((cfg.max_batch + kChunk - 1) / kChunk) * cfg.emb_dim;
}

}  // namespace gear
