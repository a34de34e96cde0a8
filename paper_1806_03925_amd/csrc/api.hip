// C ABI of libgear: argument checks, workspace layout and the launch sequence of one step.
#include "gear_internal.hpp"

#include <math.h>
#include <string.h>

#include <mutex>
#include <new>

namespace gear {

namespace {

constexpr size_t kAlign = 256;

size_t take(size_t *cursor, size_t bytes) {
  const size_t at = *cursor;
  *cursor = (at + bytes + kAlign - 1) / kAlign * kAlign;
  return at;
}

int bits_for(int64_t range) {
  int b = 1;
  while (b < 31 && ((int64_t)1 << b) < range) ++b;
  return b;
}

GroupProblem make_problem(const Layout &lay, char *ws, int slot, const int32_t *keys, int n, int64_t range) {
  GroupProblem p;
  memset(&p, 0, sizeof(p));
  p.keys_in = keys;
  p.n = n;
  p.key_bits = bits_for(range);
  p.passes = (p.key_bits + kMaxRadixBits - 1) / kMaxRadixBits;
  p.digit_bits = (p.key_bits + p.passes - 1) / p.passes;
  const Layout::G &g = lay.g[slot];
  for (int i = 0; i < 2; ++i) {
    p.keys[i] = (int32_t *)(ws + g.keys[i]);
    p.vals[i] = (int32_t *)(ws + g.vals[i]);
  }
  p.block_hist = (int32_t *)(ws + g.block_hist);
  p.sorted_keys = p.keys[p.passes & 1];
  p.perm = p.vals[p.passes & 1];
  p.tile_heads = (int32_t *)(ws + g.tile_heads);
  p.unique = (int32_t *)(ws + g.unique);
  p.segoff = (int32_t *)(ws + g.segoff);
  p.pos_seg = (int32_t *)(ws + g.pos_seg);
  p.n_unique = (int32_t *)(ws + g.n_unique);
  return p;
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

}  // namespace gear

// HIP-event pool for per-launch timing of a step
struct gear_profile {
  static constexpr int kMaxSpans = 96;
  hipEvent_t start[kMaxSpans], stop[kMaxSpans];
  const char *name[kMaxSpans];
  int used;
};

namespace gear {
namespace {

struct Span {
  gear_profile *p;
  hipStream_t s;
  int slot;
  Span(gear_profile *prof, const char *name, hipStream_t stream) : p(prof), s(stream), slot(-1) {
    if (p && p->used < gear_profile::kMaxSpans) {
      slot = p->used++;
      p->name[slot] = name;
      (void)hipEventRecord(p->start[slot], s);
    }
  }
  ~Span() {
    if (slot >= 0) (void)hipEventRecord(p->stop[slot], s);
  }
};

}  // namespace

bool config_ok(const gear_config &c) {
  if (c.n_users < 1 || c.n_urls < 1 || c.n_images < 1) return false;
  if (c.n_users > INT32_MAX || c.n_urls > INT32_MAX || c.n_images > INT32_MAX) return false;
  if (c.emb_dim < 8 || c.emb_dim % 8 || c.dfv_dim < 8 || c.dfv_dim % 8) return false;
  if (c.n_layers < 2 || c.n_layers > GEAR_MAX_LAYERS) return false;
  for (int l = 0; l < c.n_layers - 1; ++l)
    if (c.layer_out[l] < 8 || c.layer_out[l] % 8) return false;
  if (c.layer_out[c.n_layers - 1] != 1) return false;
  if (c.layer_out[c.n_layers - 2] > 1024) return false;  // the logit kernel keeps a hidden row in one wavefront
  for (int dt : {c.emb_dtype, c.dfv_dtype, c.mlp_dtype})
    if (dt != GEAR_F32 && dt != GEAR_BF16) return false;
  if (c.max_batch < 1 || c.max_nnz < 1) return false;
  if (!(c.emb_init_std >= 0.0f) || !isfinite(c.emb_init_std)) return false;
  return true;
}

bool make_layout(const gear_config &c, Layout *lay) {
  if (!config_ok(c)) return false;
  memset(lay, 0, sizeof(*lay));
  const int L = c.n_layers, F = 2 * c.emb_dim + c.dfv_dim;
  const size_t B = (size_t)c.max_batch, NNZ = (size_t)c.max_nnz;
  lay->F = F;
  lay->L = L;
  lay->act_bytes = dtype_bytes(c.mlp_dtype);
  int64_t off = 0;
  for (int l = 0; l < L; ++l) {
    lay->in_dim[l] = l == 0 ? F : c.layer_out[l - 1];
    lay->out_dim[l] = c.layer_out[l];
    lay->w_off[l] = off;
    off += (int64_t)lay->in_dim[l] * lay->out_dim[l];
    lay->b_off[l] = off;
    off += lay->out_dim[l];
  }
  lay->n_params = off;
  lay->colsum_chunks = (c.max_batch + kColsumRows - 1) / kColsumRows;

  size_t cur = 0;
  const size_t ab = lay->act_bytes;
  lay->x = take(&cur, B * F * ab);
  size_t max_partial = 0, max_h = 1;
  for (int l = 0; l < L; ++l) {
    const size_t wn = (size_t)lay->in_dim[l] * lay->out_dim[l];
    lay->wc[l] = take(&cur, wn * ab);
    lay->wct[l] = take(&cur, wn * ab);
    if (l < L - 1) {
      lay->h[l] = take(&cur, B * lay->out_dim[l] * ab);
      lay->relu_bits[l] = take(&cur, B * lay->out_dim[l] / 8);
      lay->delta[l] = take(&cur, B * lay->out_dim[l] * ab);
      lay->splitk[l] = gemm_splitk_max(c.mlp_dtype, lay->out_dim[l], lay->in_dim[l], c.max_batch);
      const size_t pb = (size_t)lay->splitk[l] * wn * sizeof(float);
      if (pb > max_partial) max_partial = pb;
    }
    if ((size_t)lay->out_dim[l] > max_h) max_h = lay->out_dim[l];
    if ((size_t)lay->in_dim[l] > max_h) max_h = lay->in_dim[l];
  }
  lay->logits = take(&cur, B * sizeof(float));
  lay->dz = take(&cur, B * sizeof(float));
  lay->loss_partial = take(&cur, logit_partial_floats(lay->in_dim[L - 1]) * sizeof(float));
  lay->dx_emb = take(&cur, B * 2 * c.emb_dim * sizeof(float));
  lay->dx_dfv = take(&cur, B * c.dfv_dim * ab);
  {
    // all hidden layers' partials at once when their products go out as one launch
    TnProblem wp[GEAR_MAX_LAYERS];
    size_t all = 0;
    for (int l = 0; l < L - 1; ++l) {
      wp[l] = TnProblem{nullptr, nullptr, nullptr, lay->out_dim[l], lay->in_dim[l]};
      all += (size_t)lay->in_dim[l] * lay->out_dim[l];
    }
    // the count of k-ranges grows with the batch, and only batches of a multiple of 32 rows take this
    // path: the largest such batch bounds what any step needs
    const size_t pb =
        (size_t)gemm_tn_batch_splits(c.mlp_dtype, wp, L - 1, c.max_batch / 32 * 32) * all * sizeof(float);
    if (pb > max_partial) max_partial = pb;
  }
  lay->wgrad_partial = take(&cur, max_partial);
  lay->wgrad_partial_bytes = max_partial;
  lay->colsum_stride = (size_t)lay->colsum_chunks * max_h;   // one buffer per hidden layer: they are reduced at the end of a step
  lay->colsum_partial = take(&cur, lay->colsum_stride * (size_t)(L > 1 ? L - 1 : 1) * sizeof(float));
  lay->emb_partial = take(&cur, embedding_partial_floats(c) * sizeof(float));
  lay->occ_view = take(&cur, NNZ * sizeof(int32_t));
  for (int s = 0; s < kMaxProblems; ++s) {
    const size_t n = s == 2 ? NNZ : B;
    const size_t tiles = (n + kSortTile - 1) / kSortTile;
    Layout::G &g = lay->g[s];
    for (int i = 0; i < 2; ++i) {
      g.keys[i] = take(&cur, n * sizeof(int32_t));
      g.vals[i] = take(&cur, n * sizeof(int32_t));
    }
    g.block_hist = take(&cur, (tiles + 1) * kMaxRadix * sizeof(int32_t));
    g.tile_heads = take(&cur, tiles * sizeof(int32_t));
    g.unique = take(&cur, n * sizeof(int32_t));
    g.segoff = take(&cur, (n + 1) * sizeof(int32_t));
    g.pos_seg = take(&cur, n * sizeof(int32_t));
    g.n_unique = take(&cur, sizeof(int32_t));
  }
  const size_t tiles = (NNZ + kSortTile - 1) / kSortTile;
  lay->tile_units = take(&cur, tiles * sizeof(int32_t));
  lay->tile_emits = take(&cur, tiles * sizeof(int32_t));
  lay->units = take(&cur, NNZ * sizeof(UnitDesc));
  lay->row_view = take(&cur, NNZ * sizeof(int32_t));
  lay->row_scale = take(&cur, NNZ * sizeof(float));
  lay->n_units = take(&cur, sizeof(int32_t));
  lay->expiry_marks = take(&cur, (size_t)expiry_words(c.n_images) * sizeof(uint32_t));
  lay->expiry_tiles = take(&cur, (size_t)expiry_tiles(c.n_images) * sizeof(int32_t));
  lay->total = cur;
  return true;
}

}  // namespace gear

using namespace gear;

// Scratch memory of gear_step_static: one array per device, inside the code object, so that the call
// needs no allocation.  In host code the array's name only stands for the symbol; the address of a
// device's copy comes from hipGetSymbolAddress with that device current, and that address is what
// the kernels are given.
#define GEAR_STATIC_SCRATCH_BYTES (64u << 20)
static __device__ __align__(256) unsigned char scratch[GEAR_STATIC_SCRATCH_BYTES];

namespace {
void *g_scratch_ptr[64];
std::mutex g_scratch_mutex;

// address of the current device's copy of `scratch` (looked up once per device); nullptr on failure
void *static_scratch() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    if ((uintptr_t)ptr & 255u) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

// One helper stream and three events per device, created on first use and kept for the life of the
// process: the integer grouping of a step runs beside its gather and forward pass.
namespace {
struct SideLane {
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, join = nullptr, checked = nullptr;
  bool ready = false;
  std::mutex busy;  // held while a step enqueues: two host threads never interleave their forks and joins
};
SideLane g_side[64];
std::mutex g_side_mutex;

// multiply-adds of the DFV-slot part of the dLoss/dx product from which it is worth an extra launch
// and event to let the embedding update run beside it (about 10 us of work on the device)
constexpr double kSplitDxMacs = 5e9;

// the helper lane of the current device; nullptr when one of its objects cannot be created (nothing
// half-made is kept: the next call starts over)
SideLane *side_lane() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(g_side_mutex);
  SideLane &l = g_side[dev];
  if (!l.ready) {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr, checked = nullptr;
    bool ok = hipStreamCreateWithFlags(&stream, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&fork, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&join, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&checked, hipEventDisableTiming) == hipSuccess;
    if (!ok) {
      if (checked) (void)hipEventDestroy(checked);
      if (join) (void)hipEventDestroy(join);
      if (fork) (void)hipEventDestroy(fork);
      if (stream) (void)hipStreamDestroy(stream);
      return nullptr;
    }
    l.stream = stream;
    l.fork = fork;
    l.join = join;
    l.checked = checked;
    l.ready = true;
  }
  return &l;
}

// A step's use of the helper lane.  Holds the lane for the whole enqueue, so that steps issued from
// several host threads on one device use the lane's events one after the other, and makes sure
// that whatever was forked to the helper stream is joined back into the caller's stream however the
// enqueue ends: after an early return (a failed launch) the next call on the caller's stream must
// not run beside kernels this call left on the helper stream.
class LaneScope {
 public:
  LaneScope(SideLane *side, hipStream_t caller) : side_(side), s_(caller) {
    if (side_) side_->busy.lock();
  }
  ~LaneScope() {
    if (!side_) return;
    if (forked_ && !joined_) {
      if (hipEventRecord(side_->join, side_->stream) == hipSuccess) (void)hipStreamWaitEvent(s_, side_->join, 0);
    }
    side_->busy.unlock();
  }
  LaneScope(const LaneScope &) = delete;
  LaneScope &operator=(const LaneScope &) = delete;
  // what the caller's stream has done so far happens before whatever the helper stream is given next
  hipError_t fork() {
    if (!side_) return hipSuccess;
    hipError_t e = hipEventRecord(side_->fork, s_);
    if (e != hipSuccess) return e;
    forked_ = true;
    joined_ = false;
    return hipStreamWaitEvent(side_->stream, side_->fork, 0);
  }
  // marks the point of the helper stream that a later wait() refers to
  hipError_t mark() { return side_ ? hipEventRecord(side_->join, side_->stream) : hipSuccess; }
  // the same for the end of the helper's first part (ids checked, plan made): the status word is final
  hipError_t mark_checked() { return side_ ? hipEventRecord(side_->checked, side_->stream) : hipSuccess; }
  hipError_t wait_checked() { return side_ ? hipStreamWaitEvent(s_, side_->checked, 0) : hipSuccess; }
  // the caller's stream continues after the last mark(); final = nothing is given to the helper after it
  hipError_t wait(bool final) {
    if (!side_) return hipSuccess;
    hipError_t e = hipStreamWaitEvent(s_, side_->join, 0);
    if (e == hipSuccess && final) joined_ = true;
    return e;
  }

 private:
  SideLane *side_;
  hipStream_t s_;
  bool forked_ = false, joined_ = false;
};
}  // namespace

// Test hook: the n-th launch of this thread's next steps reports failure instead of being enqueued
// (0 = off).  Lets a test walk the error paths of a step without a failing device.
thread_local int g_fail_at = 0;
inline bool fail_injected() { return g_fail_at > 0 && --g_fail_at == 0; }

#define GEAR_HIP(expr)                             \
  do {                                             \
    if ((expr) != hipSuccess) return GEAR_ERR_HIP; \
  } while (0)
// a launch bracketed by profile events (when a profile is attached)
#define GEAR_RUN(name, expr)    \
  do {                          \
    if (fail_injected()) return GEAR_ERR_HIP; \
    Span span_(prof, name, s);  \
    GEAR_HIP(expr);             \
  } while (0)

extern "C" {

size_t gear_workspace_bytes(const gear_config *cfg) {
  Layout lay;
  if (!cfg || !make_layout(*cfg, &lay)) return 0;
  return lay.total;
}

int64_t gear_mlp_param_count(const gear_config *cfg) {
  Layout lay;
  if (!cfg || !make_layout(*cfg, &lay)) return -1;
  return lay.n_params;
}

int64_t gear_mlp_param_offset(const gear_config *cfg, int32_t layer, int32_t which) {
  Layout lay;
  if (!cfg || !make_layout(*cfg, &lay) || layer < 0 || layer >= lay.L || which < 0 || which > 1) return -1;
  return which == 0 ? lay.w_off[layer] : lay.b_off[layer];
}

gear_status gear_workspace_region(const gear_config *cfg, const char *name, size_t *offset, size_t *bytes) {
  Layout lay;
  if (!cfg || !name || !offset || !bytes || !make_layout(*cfg, &lay)) return GEAR_ERR_INVALID;
  const size_t B = (size_t)cfg->max_batch;
  if (!strcmp(name, "x")) {
    *offset = lay.x;
    *bytes = B * lay.F * lay.act_bytes;
  } else if (!strcmp(name, "logits")) {
    *offset = lay.logits;
    *bytes = B * sizeof(float);
  } else if (!strcmp(name, "dx_emb")) {
    *offset = lay.dx_emb;
    *bytes = B * 2 * cfg->emb_dim * sizeof(float);
  } else if (!strcmp(name, "dx_dfv")) {
    *offset = lay.dx_dfv;
    *bytes = B * cfg->dfv_dim * lay.act_bytes;
  } else if (name[0] == 'h' && name[1] >= '0' && name[1] < '0' + GEAR_MAX_LAYERS && !name[2] &&
             name[1] - '0' < lay.L - 1) {
    const int l = name[1] - '0';
    *offset = lay.h[l];
    *bytes = B * lay.out_dim[l] * lay.act_bytes;
  } else {
    return GEAR_ERR_INVALID;
  }
  return GEAR_OK;
}

gear_status gear_fill_normal(void *dst, int32_t dtype, int64_t n_rows, int32_t dim, uint64_t seed,
                             uint32_t stream_id, float std, void *stream) {
  if (!dst || n_rows < 0 || dim < 1 || (dtype != GEAR_F32 && dtype != GEAR_BF16) || !(std >= 0.0f) || !isfinite(std))
    return GEAR_ERR_INVALID;
  GEAR_HIP(launch_fill_normal(dst, dtype, n_rows * dim, seed, stream_id, std, (hipStream_t)stream));
  return GEAR_OK;
}

gear_status gear_init_tables(const gear_config *cfg, gear_tables *t, float *grad_accum, int32_t *counts,
                             void *stream) {
  Layout lay;
  if (!cfg || !t || !t->user_emb || !t->url_emb || !t->mlp_params || !grad_accum || !counts) return GEAR_ERR_INVALID;
  if (!make_layout(*cfg, &lay) || !aligned16(grad_accum) || !aligned16(counts) || !aligned16(t->mlp_params))
    return GEAR_ERR_INVALID;
  hipStream_t s = (hipStream_t)stream;
  if (!static_scratch()) return GEAR_ERR_HIP;  // looked up here so that a later gear_step_static need not
  GEAR_HIP(launch_fill_normal(t->user_emb, cfg->emb_dtype, cfg->n_users * cfg->emb_dim, cfg->seed, 1u,
                              cfg->emb_init_std, s));
  GEAR_HIP(launch_fill_normal(t->url_emb, cfg->emb_dtype, cfg->n_urls * cfg->emb_dim, cfg->seed, 2u,
                              cfg->emb_init_std, s));
  GEAR_HIP(launch_fill_zero(t->mlp_params, (size_t)lay.n_params * sizeof(float), s));
  for (int l = 0; l < lay.L; ++l)
    GEAR_HIP(launch_fill_normal(t->mlp_params + lay.w_off[l], GEAR_F32, (int64_t)lay.in_dim[l] * lay.out_dim[l],
                                cfg->seed, 16u + (uint32_t)l, sqrtf(2.0f / (float)lay.in_dim[l]), s));
  GEAR_HIP(launch_fill_zero(grad_accum, (size_t)cfg->n_images * cfg->dfv_dim * sizeof(float), s));
  GEAR_HIP(launch_fill_zero(counts, (size_t)cfg->n_images * sizeof(int32_t), s));
  return GEAR_OK;
}

gear_status gear_step(const gear_config *cfg, const gear_batch *b, gear_tables *t, const void *dfv_cache,
                      float *grad_accum, int32_t *counts, int32_t M, float lr, void *workspace,
                      size_t workspace_bytes, gear_step_out *out, void *stream) {
  return gear_step_adam(cfg, b, t, dfv_cache, grad_accum, counts, M, lr, nullptr, workspace, workspace_bytes, out,
                        stream);
}

gear_status gear_step_static(const gear_config *cfg, const gear_batch *b, gear_tables *t, const void *dfv_cache,
                             float *grad_accum, int32_t *counts, int32_t M, float lr, gear_step_out *out,
                             void *stream) {
  Layout lay;
  if (!cfg || !out || !make_layout(*cfg, &lay)) return GEAR_ERR_INVALID;
  if (lay.total > GEAR_STATIC_SCRATCH_BYTES) return GEAR_ERR_CAPACITY;
  void *ws = static_scratch();
  if (!ws) return GEAR_ERR_HIP;
  // every kernel on the caller's stream: no helper stream or event has to exist
  gear_step_out o = *out;
  o.one_stream = 1;
  return gear_step_adam(cfg, b, t, dfv_cache, grad_accum, counts, M, lr, nullptr, ws, GEAR_STATIC_SCRATCH_BYTES, &o,
                        stream);
}

gear_status gear_step_adam(const gear_config *cfg, const gear_batch *b, gear_tables *t, const void *dfv_cache,
                           float *grad_accum, int32_t *counts, int32_t M, float lr, const gear_adam *adam,
                           void *workspace, size_t workspace_bytes, gear_step_out *out, void *stream) {
  Layout lay;
  if (!cfg || !b || !t || !dfv_cache || !grad_accum || !counts || !workspace || !out) return GEAR_ERR_INVALID;
  if (!make_layout(*cfg, &lay)) return GEAR_ERR_INVALID;
  if (!t->user_emb || !t->url_emb || !t->mlp_params) return GEAR_ERR_INVALID;
  if (!out->loss || !out->n_ready || !out->ready_ids || !out->ready_grads || !out->status || out->ready_cap < 0)
    return GEAR_ERR_INVALID;
  if (M < 1 || !isfinite(lr)) return GEAR_ERR_INVALID;
  if (b->B < 0 || b->nnz < 0 || b->B > cfg->max_batch || b->nnz > cfg->max_nnz) return GEAR_ERR_INVALID;
  if (b->B > 0 && (!b->user_id || !b->url_id || !b->img_off || !b->label)) return GEAR_ERR_INVALID;
  if (b->nnz > 0 && (!b->img_id || b->B == 0)) return GEAR_ERR_INVALID;
  if (((uintptr_t)workspace & (kAlign - 1)) || !aligned16(grad_accum) || !aligned16(out->ready_grads) ||
      !aligned16(dfv_cache) || !aligned16(t->user_emb) || !aligned16(t->url_emb) || !aligned16(t->mlp_params))
    return GEAR_ERR_INVALID;
  if (workspace_bytes < lay.total) return GEAR_ERR_CAPACITY;

  // the update rule and where each parameter array keeps its moments
  Optim opt = {lr, 0.0f, 0.0f, 0.0f, 1.0f, 0};
  Moments mom_mlp = {nullptr, nullptr}, mom_user = {nullptr, nullptr}, mom_url = {nullptr, nullptr};
  if (adam) {
    if (!(adam->beta1 >= 0.0f && adam->beta1 < 1.0f) || !(adam->beta2 >= 0.0f && adam->beta2 < 1.0f) ||
        !(adam->eps > 0.0f) || adam->t < 1)
      return GEAR_ERR_INVALID;
    if (!adam->user_m || !adam->user_v || !adam->url_m || !adam->url_v || !adam->mlp_m || !adam->mlp_v)
      return GEAR_ERR_INVALID;
    if (!aligned16(adam->user_m) || !aligned16(adam->user_v) || !aligned16(adam->url_m) || !aligned16(adam->url_v) ||
        !aligned16(adam->mlp_m) || !aligned16(adam->mlp_v))
      return GEAR_ERR_INVALID;
    opt.adam = 1;
    opt.beta1 = adam->beta1;
    opt.beta2 = adam->beta2;
    opt.eps = adam->eps;
    opt.lr = (float)((double)lr / (1.0 - pow((double)adam->beta1, (double)adam->t)));
    opt.inv_bc2 = (float)(1.0 / sqrt(1.0 - pow((double)adam->beta2, (double)adam->t)));
    mom_mlp = {adam->mlp_m, adam->mlp_v};
    mom_user = {adam->user_m, adam->user_v};
    mom_url = {adam->url_m, adam->url_v};
  }

  hipStream_t s = (hipStream_t)stream;
  char *ws = (char *)workspace;
  const int B = b->B, L = lay.L, F = lay.F, dt = cfg->mlp_dtype;
  int32_t *status = out->status;

  gear_profile *prof = (gear_profile *)out->profile;
  if (prof) prof->used = 0;
  static const char *const kFwd[GEAR_MAX_LAYERS] = {"fwd_gemm_l0", "fwd_gemm_l1", "fwd_gemm_l2", "fwd_gemm_l3",
                                                    "fwd_gemm_l4", "fwd_gemm_l5", "fwd_gemm_l6", "fwd_gemm_l7"};
  static const char *const kDgrad[GEAR_MAX_LAYERS] = {"dgrad_gemm_l0", "dgrad_gemm_l1", "dgrad_gemm_l2",
                                                      "dgrad_gemm_l3", "dgrad_gemm_l4", "dgrad_gemm_l5",
                                                      "dgrad_gemm_l6", "dgrad_gemm_l7"};
  static const char *const kWgrad[GEAR_MAX_LAYERS] = {"wgrad_gemm_l0", "wgrad_gemm_l1", "wgrad_gemm_l2",
                                                      "wgrad_gemm_l3", "wgrad_gemm_l4", "wgrad_gemm_l5",
                                                      "wgrad_gemm_l6", "wgrad_gemm_l7"};

  GEAR_RUN("begin", launch_begin(status, out->n_ready, out->loss, s));
  if (B == 0) return GEAR_OK;
  int32_t *occ_view = (int32_t *)(ws + lay.occ_view);

  // grouping of the three id lists and the plan of the per-image accumulation
  GroupBatch gb;
  gb.count = 3;
  gb.p[0] = make_problem(lay, ws, 0, b->user_id, B, cfg->n_users);
  gb.p[1] = make_problem(lay, ws, 1, b->url_id, B, cfg->n_urls);
  gb.p[2] = make_problem(lay, ws, 2, b->img_id, b->nnz, cfg->n_images);
  AccumPlan plan;
  plan.tile_units = (int32_t *)(ws + lay.tile_units);
  plan.tile_emits = (int32_t *)(ws + lay.tile_emits);
  plan.units = (UnitDesc *)(ws + lay.units);
  plan.row_view = (int32_t *)(ws + lay.row_view);
  plan.row_scale = (float *)(ws + lay.row_scale);
  plan.n_units = (int32_t *)(ws + lay.n_units);
  // What depends only on ids and counters runs on the helper stream while the main stream gathers and
  // runs the forward pass: the check of the ids, the grouping, the accumulation plan and the counter update.  The
  // main stream waits for it before the first kernel that changes caller state, so the status word
  // is final by then; until then its kernels write the workspace only, and the gather clamps what it
  // uses as an index.
  const bool one_stream = out->one_stream != 0;
  SideLane *side = one_stream ? nullptr : side_lane();
  if (!one_stream && !side) return GEAR_ERR_HIP;
  hipStream_t helper = one_stream ? s : side->stream;
  LaneScope lane(side, s);
  GEAR_HIP(lane.fork());
  {
    // operand copies of the weights (all layers in one launch), ahead of the gather on the caller's
    // stream: the first product then needs no event, and behind the gather's many workgroups the
    // copies would not get onto the device before it ends anyway
    const float *cw[GEAR_MAX_LAYERS];
    void *cwc[GEAR_MAX_LAYERS], *cwct[GEAR_MAX_LAYERS];
    for (int l = 0; l < L; ++l) {
      cw[l] = t->mlp_params + lay.w_off[l];
      cwc[l] = ws + lay.wc[l];
      cwct[l] = ws + lay.wct[l];
    }
    GEAR_RUN("cast_weights", launch_cast_weights(L, cw, lay.out_dim, lay.in_dim, dt, cwc, cwct, status, s));
  }
  // forward
  void *x = ws + lay.x;
  // the weight-gradient products of the hidden layers, and whether they go out as one launch
  TnProblem wp[GEAR_MAX_LAYERS];
  int n_wp = 0;
  for (int l = L - 2; l >= 0; --l)
    wp[n_wp++] = TnProblem{ws + lay.delta[l], l == 0 ? x : ws + lay.h[l - 1], nullptr, lay.out_dim[l], lay.in_dim[l]};
  const int batch_splits = gemm_tn_batch_splits(dt, wp, n_wp, B);
  GEAR_RUN("gather_pool", launch_gather_pool(*cfg, *b, *t, dfv_cache, x, s));
  // A hidden layer below the last one also leaves the sign bitmap of its activations when both its
  // own product and the dgrad product that masks with it run in the kernel that knows bitmaps: the
  // backward pass then reads one bit per unit instead of the activation.
  uint8_t *relu_bits[GEAR_MAX_LAYERS] = {};
  for (int l = 0; l + 2 < L; ++l)
    if (gemm_nt_has_bits(dt, lay.in_dim[l]) && gemm_nt_has_bits(dt, lay.out_dim[l + 1]))
      relu_bits[l] = (uint8_t *)(ws + lay.relu_bits[l]);
  for (int l = 0; l < L - 1; ++l)
    GEAR_RUN(kFwd[l], launch_gemm_nt(dt, l == 0 ? x : ws + lay.h[l - 1], ws + lay.wc[l], B, lay.out_dim[l],
                                     lay.in_dim[l], EPI_BIAS_RELU, t->mlp_params + lay.b_off[l], nullptr,
                                     ws + lay.h[l], 0, nullptr, relu_bits[l], status, s));
  // The helper stream's launches are issued after the forward pass's: where the host is not ahead of the
  // device (a caller that waits for every step), the gather then starts as soon as the step does, not
  // after the host has issued the grouping's many small launches.
  {
    hipStream_t s = helper;  // the launches of this block go to the helper stream
    GEAR_RUN("validate", launch_validate(*cfg, *b, occ_view, status, s));
    GEAR_RUN("group_ids", launch_group(gb, status, s));
    GEAR_RUN("accum_plan", launch_accum_plan(gb.p[2], plan, occ_view, b->img_off, counts, M, out->ready_cap,
                                             out->n_ready, status, s));
    GEAR_RUN("count_update", launch_count_update(gb.p[2], counts, status, s));
  }
  GEAR_HIP(lane.mark_checked());

  float *logits = (float *)(ws + lay.logits), *dz = (float *)(ws + lay.dz);
  // Until its first kernel that changes caller state (the first SGD on a hidden layer's weights), the
  // caller's stream writes the workspace only and need not know whether the ids were in range or the
  // ready list fits.  Just before that kernel the stream waits for the helper's first part, so that the
  // status word is final.
  GEAR_RUN("logit_loss", launch_logit_loss(dt, ws + lay.h[L - 2], ws + lay.wc[L - 1], t->mlp_params + lay.b_off[L - 1],
                                           b->label, B, lay.in_dim[L - 1], logits, dz, ws + lay.delta[L - 2],
                                           (float *)(ws + lay.loss_partial), status, s));

  // backward through the hidden layers down to dLoss/dx (all from the pre-step operand copies)
  // Each product that makes the delta of a hidden layer also leaves that layer's bias gradient (column
  // sums of the delta) as per-row-tile partials; they are added in tile order at the end of the step.
  float *dx_emb = (float *)(ws + lay.dx_emb);
  void *dx_dfv = ws + lay.dx_dfv;
  float *cpart = (float *)(ws + lay.colsum_partial), *wpart = (float *)(ws + lay.wgrad_partial);
  // Small reductions whose results nothing in the step reads (the loss, SGD on the logit layer and on
  // the biases): they go to the helper stream, ahead of the embedding update.
  auto small_reductions = [&](hipStream_t s) -> gear_status {
    GEAR_RUN("logit_sgd", launch_logit_finish((float *)(ws + lay.loss_partial), B, lay.in_dim[L - 1],
                                              t->mlp_params + lay.w_off[L - 1], t->mlp_params + lay.b_off[L - 1],
                                              t->mlp_params + lay.b_off[L - 2], out->loss, opt,
                                              moments_at(mom_mlp, lay.w_off[L - 1]), moments_at(mom_mlp, lay.b_off[L - 1]),
                                              moments_at(mom_mlp, lay.b_off[L - 2]), status, s));
    for (int l = L - 2; l > 0; --l) {
      // bias gradient of layer l - 1: column sums of its delta, left as per-row-tile partials by the
      // product that made it where that kernel does so, otherwise summed here
      const int parts = gemm_nt_colsum_parts(dt, B, lay.in_dim[l], lay.out_dim[l]);
      if (parts)
        GEAR_RUN("bias_sgd", launch_partial_sgd(cpart + (size_t)l * lay.colsum_stride, parts, lay.out_dim[l - 1],
                                                t->mlp_params + lay.b_off[l - 1], opt,
                                                moments_at(mom_mlp, lay.b_off[l - 1]), status, s));
      else
        GEAR_RUN("bias_sgd", launch_colsum_sgd(dt, ws + lay.delta[l - 1], B, lay.out_dim[l - 1], cpart,
                                               t->mlp_params + lay.b_off[l - 1], opt,
                                               moments_at(mom_mlp, lay.b_off[l - 1]), status, s));
    }
    return GEAR_OK;
  };
  bool embedding_updated = false;
  for (int l = L - 2; l >= 0; --l) {
    if (l > 0) {
      const int parts = gemm_nt_colsum_parts(dt, B, lay.in_dim[l], lay.out_dim[l]);
      const bool by_bits = relu_bits[l - 1] != nullptr;
      GEAR_RUN(kDgrad[l], launch_gemm_nt(dt, ws + lay.delta[l], ws + lay.wct[l], B, lay.in_dim[l], lay.out_dim[l],
                                         by_bits ? EPI_MASK_BITS : EPI_MASK, nullptr,
                                         by_bits ? (const void *)relu_bits[l - 1] : (const void *)(ws + lay.h[l - 1]),
                                         ws + lay.delta[l - 1], 0, parts ? cpart + (size_t)l * lay.colsum_stride : nullptr, nullptr,
                                         status, s));
    } else {
      // dLoss/dx: the embedding slots stay fp32, the DFV slot is kept in the MLP's operand type.
      // When the product is long enough to hide it, it is made in two parts: the embedding slots
      // first, and as soon as they are there the SGD on the touched embedding rows starts on the
      // helper stream, beside the larger product that makes the DFV slot.  Every element is computed
      // the same way in both forms.
      const int E2 = 2 * cfg->emb_dim;
      if ((double)B * (F - E2) * lay.out_dim[0] >= kSplitDxMacs) {
        GEAR_RUN("dgrad_gemm_emb", launch_gemm_nt(dt, ws + lay.delta[0], ws + lay.wct[0], B, E2, lay.out_dim[0], EPI_DX,
                                                  nullptr, dx_dfv, dx_emb, E2, nullptr, nullptr, status, s));
        GEAR_HIP(lane.fork());
        {
          hipStream_t s = helper;
          if (gear_status st = small_reductions(s)) return st;
          GEAR_RUN("embedding_update",
                   launch_embedding_update(*cfg, gb.p[0], gb.p[1], dx_emb, t->user_emb, t->url_emb,
                                           (float *)(ws + lay.emb_partial), opt, mom_user, mom_url, status, s));
        }
        embedding_updated = true;
        GEAR_RUN(kDgrad[0], launch_gemm_nt(dt, ws + lay.delta[0],
                                           ws + lay.wct[0] + (size_t)E2 * lay.out_dim[0] * lay.act_bytes, B, F - E2,
                                           lay.out_dim[0], EPI_DX, nullptr, dx_dfv, dx_emb, 0, nullptr, nullptr, status, s));
      } else {
        GEAR_RUN(kDgrad[0], launch_gemm_nt(dt, ws + lay.delta[0], ws + lay.wct[0], B, F, lay.out_dim[0], EPI_DX,
                                           nullptr, dx_dfv, dx_emb, E2, nullptr, nullptr, status, s));
      }
    }
  }

  // The per-image gradient bookkeeping only needs dLoss/dx and is bound by memory traffic: it runs on
  // the helper stream beside the weight-gradient products, which are not.  The products are
  // launched first and, where they can, as one launch of at most one round of workgroups, so that
  // they hold their CUs before the bookkeeping's many small workgroups arrive and fill what is
  // left; a product arriving later would wait until all of those have been placed.
  GEAR_HIP(lane.fork());
  {
    hipStream_t s = helper;
    if (!embedding_updated) {
      if (gear_status st = small_reductions(s)) return st;
      GEAR_RUN("embedding_update",
               launch_embedding_update(*cfg, gb.p[0], gb.p[1], dx_emb, t->user_emb, t->url_emb,
                                       (float *)(ws + lay.emb_partial), opt, mom_user, mom_url, status, s));
    }
    GEAR_RUN("accumulate", launch_accumulate(*cfg, gb.p[2], plan, dx_dfv, grad_accum, M, out->ready_ids,
                                             out->ready_grads, status, s));
  }
  GEAR_HIP(lane.mark());
  // SGD on the hidden layers' weights: split-K wgrad (the logit layer and all biases are done on the helper stream)
  bool joined = false;
  if (batch_splits > 0) {
    float *next = wpart;
    for (int i = 0; i < n_wp; ++i) {
      wp[i].partial = next;
      next += (size_t)batch_splits * wp[i].M * wp[i].N;
    }
    if ((size_t)(next - wpart) * sizeof(float) > lay.wgrad_partial_bytes) return GEAR_ERR_CAPACITY;  // cannot happen: sized for the largest batch
    GEAR_RUN("wgrad_gemm", launch_gemm_tn_batch(wp, n_wp, B, batch_splits, status, s));
    SplitkProblem sp[GEAR_MAX_LAYERS];
    for (int i = 0; i < n_wp; ++i) {
      const int l = L - 2 - i;
      sp[i] = SplitkProblem{wp[i].partial, t->mlp_params + lay.w_off[l], moments_at(mom_mlp, lay.w_off[l]),
                            (int64_t)wp[i].M * wp[i].N};
    }
    // The sums of the partials and the SGD change caller state, so the status word has to be final: the
    // stream waits for the helper's first part (long done by now), not for the bookkeeping.  Their
    // workgroups get onto the device as the bookkeeping's leave room and are done before it is, so the
    // step ends with the bookkeeping and the join.
    GEAR_HIP(lane.wait_checked());
    GEAR_RUN("splitk_sgd", launch_splitk_sgd_batch(sp, n_wp, batch_splits, opt, status, s));
    GEAR_HIP(lane.wait(true));
    joined = true;
  } else {
    for (int l = L - 2; l >= 0; --l) {
      const int splits = gemm_splitk_for(dt, lay.out_dim[l], lay.in_dim[l], B);
      if ((size_t)splits * lay.out_dim[l] * lay.in_dim[l] * sizeof(float) > lay.wgrad_partial_bytes)
        return GEAR_ERR_CAPACITY;  // cannot happen: sized for the largest count any batch can ask for
      GEAR_RUN(kWgrad[l], launch_gemm_tn_splitk(dt, ws + lay.delta[l], l == 0 ? x : ws + lay.h[l - 1], lay.out_dim[l],
                                                lay.in_dim[l], B, splits, wpart, status, s));
      if (l == L - 2) GEAR_HIP(lane.wait_checked());
      GEAR_RUN("splitk_sgd", launch_splitk_sgd(wpart, splits, (int64_t)lay.out_dim[l] * lay.in_dim[l],
                                               t->mlp_params + lay.w_off[l], opt, moments_at(mom_mlp, lay.w_off[l]),
                                               status, s));
    }
  }
  if (!joined) GEAR_HIP(lane.wait(true));  // the step ends on the caller's stream
  if (out->dbg_img_unique && b->nnz > 0)
    GEAR_HIP(hipMemcpyAsync(out->dbg_img_unique, gb.p[2].unique, (size_t)b->nnz * 4, hipMemcpyDeviceToDevice, s));
  if (out->dbg_img_segoff)
    GEAR_HIP(hipMemcpyAsync(out->dbg_img_segoff, gb.p[2].segoff, ((size_t)b->nnz + 1) * 4, hipMemcpyDeviceToDevice, s));
  if (out->dbg_img_perm && b->nnz > 0)
    GEAR_HIP(hipMemcpyAsync(out->dbg_img_perm, gb.p[2].perm, (size_t)b->nnz * 4, hipMemcpyDeviceToDevice, s));
  if (out->dbg_n_img_unique)
    GEAR_HIP(hipMemcpyAsync(out->dbg_n_img_unique, gb.p[2].n_unique, 4, hipMemcpyDeviceToDevice, s));
  return GEAR_OK;
}

gear_status gear_refresh_dfv(const gear_config *cfg, void *dfv_cache, const int32_t *image_ids, const void *new_dfv,
                             int64_t n, int32_t *status, void *stream) {
  if (!cfg || !config_ok(*cfg) || !dfv_cache || n < 0 || (n > 0 && !new_dfv)) return GEAR_ERR_INVALID;
  if (!aligned16(dfv_cache) || !aligned16(new_dfv)) return GEAR_ERR_INVALID;
  if (!image_ids && n > cfg->n_images) return GEAR_ERR_INVALID;
  GEAR_HIP(launch_refresh(cfg->dfv_dtype, dfv_cache, cfg->n_images, cfg->dfv_dim, image_ids, new_dfv, n, status,
                          (hipStream_t)stream));
  return GEAR_OK;
}

gear_status gear_refresh_dfv_n(const gear_config *cfg, void *dfv_cache, const int32_t *image_ids, const void *new_dfv,
                               const int32_t *n_rows, int64_t max_rows, int32_t *status, void *stream) {
  if (!cfg || !config_ok(*cfg) || !dfv_cache || !image_ids || !n_rows || max_rows < 0 || (max_rows > 0 && !new_dfv))
    return GEAR_ERR_INVALID;
  if (!aligned16(dfv_cache) || !aligned16(new_dfv)) return GEAR_ERR_INVALID;
  GEAR_HIP(launch_refresh(cfg->dfv_dtype, dfv_cache, cfg->n_images, cfg->dfv_dim, image_ids, new_dfv, max_rows, status,
                          (hipStream_t)stream, n_rows));
  return GEAR_OK;
}

gear_status gear_stamp_dfv_n(const gear_config *cfg, int32_t *dfv_stamp, const int32_t *image_ids, const int32_t *n_rows,
                             int64_t max_rows, int32_t now, int32_t *status, void *stream) {
  if (!cfg || !config_ok(*cfg) || !dfv_stamp || !image_ids || !n_rows || max_rows < 0) return GEAR_ERR_INVALID;
  GEAR_HIP(launch_stamp(dfv_stamp, cfg->n_images, image_ids, max_rows, now, status, (hipStream_t)stream, n_rows));
  return GEAR_OK;
}

gear_status gear_group_ids(const gear_config *cfg, const int32_t *keys, int32_t n, int64_t key_range, void *workspace,
                           size_t workspace_bytes, int32_t *unique, int32_t *segoff, int32_t *perm, int32_t *n_unique,
                           void *stream) {
  Layout lay;
  if (!cfg || !make_layout(*cfg, &lay) || !workspace || !unique || !segoff || !perm || !n_unique)
    return GEAR_ERR_INVALID;
  if (n < 0 || n > cfg->max_nnz || (n > 0 && !keys) || key_range < 1 || key_range > ((int64_t)1 << 31))
    return GEAR_ERR_INVALID;
  if ((uintptr_t)workspace & (kAlign - 1)) return GEAR_ERR_INVALID;
  if (workspace_bytes < lay.total) return GEAR_ERR_CAPACITY;
  hipStream_t s = (hipStream_t)stream;
  char *ws = (char *)workspace;
  int32_t *status = (int32_t *)(ws + lay.n_units);  // a spare word, cleared below: nothing can fail here
  GEAR_HIP(launch_fill_zero(status, sizeof(int32_t), s));
  GroupBatch gb;
  gb.count = 1;
  gb.p[0] = make_problem(lay, ws, 2, keys, n, key_range);
  gb.p[0].pos_seg = nullptr;
  GEAR_HIP(launch_group(gb, status, s));
  if (n > 0) {
    GEAR_HIP(hipMemcpyAsync(unique, gb.p[0].unique, (size_t)n * 4, hipMemcpyDeviceToDevice, s));
    GEAR_HIP(hipMemcpyAsync(perm, gb.p[0].perm, (size_t)n * 4, hipMemcpyDeviceToDevice, s));
  }
  GEAR_HIP(hipMemcpyAsync(segoff, gb.p[0].segoff, ((size_t)n + 1) * 4, hipMemcpyDeviceToDevice, s));
  GEAR_HIP(hipMemcpyAsync(n_unique, gb.p[0].n_unique, 4, hipMemcpyDeviceToDevice, s));
  return GEAR_OK;
}

gear_status gear_expired_ids(const gear_config *cfg, const int32_t *image_ids, int32_t n, const int32_t *dfv_stamp,
                             int32_t now, int32_t expiry, void *workspace, size_t workspace_bytes,
                             int32_t *expired_ids, int32_t *n_expired, int32_t *status, void *stream) {
  Layout lay;
  if (!cfg || !make_layout(*cfg, &lay) || !workspace || !dfv_stamp || !expired_ids || !n_expired || !status)
    return GEAR_ERR_INVALID;
  if (n < 0 || n > cfg->max_nnz || (n > 0 && !image_ids) || expiry < 0) return GEAR_ERR_INVALID;
  if ((uintptr_t)workspace & (kAlign - 1)) return GEAR_ERR_INVALID;
  if (workspace_bytes < lay.total) return GEAR_ERR_CAPACITY;
  hipStream_t s = (hipStream_t)stream;
  char *ws = (char *)workspace;
  GEAR_HIP(launch_fill_zero(status, sizeof(int32_t), s));
  GEAR_HIP(launch_expired(image_ids, n, dfv_stamp, cfg->n_images, now, expiry, (uint8_t *)(ws + lay.expiry_marks),
                          (int32_t *)(ws + lay.expiry_tiles), expired_ids, n_expired, status, s));
  return GEAR_OK;
}

gear_status gear_stamp_dfv(const gear_config *cfg, int32_t *dfv_stamp, const int32_t *image_ids, int64_t n,
                           int32_t now, int32_t *status, void *stream) {
  if (!cfg || !config_ok(*cfg) || !dfv_stamp || n < 0) return GEAR_ERR_INVALID;
  if (!image_ids && n > cfg->n_images) return GEAR_ERR_INVALID;
  GEAR_HIP(launch_stamp(dfv_stamp, cfg->n_images, image_ids, n, now, status, (hipStream_t)stream));
  return GEAR_OK;
}

gear_status gear_gemm(int32_t dtype, int32_t form, const void *A, const void *B, int32_t M, int32_t N, int32_t K,
                      int32_t epilogue, const float *bias, const void *aux, void *out, int32_t splits,
                      float *partial, int32_t *status, void *stream) {
  if ((dtype != GEAR_F32 && dtype != GEAR_BF16) || !A || !B || !out || !status || M < 1 || N < 1 || K < 1)
    return GEAR_ERR_INVALID;
  const int vec = dtype == GEAR_BF16 ? 8 : 4;
  if (!aligned16(A) || !aligned16(B) || !aligned16(out)) return GEAR_ERR_INVALID;
  hipStream_t s = (hipStream_t)stream;
  if (form == 0) {
    if (K % vec || N % vec || epilogue < EPI_BIAS_RELU || epilogue > EPI_F32) return GEAR_ERR_INVALID;
    if ((epilogue == EPI_BIAS_RELU && !bias) || (epilogue == EPI_MASK && (!aux || !aligned16(aux))))
      return GEAR_ERR_INVALID;
    GEAR_HIP(launch_gemm_nt(dtype, A, B, M, N, K, epilogue, bias, aux, out, 0, nullptr, nullptr, status, s));
  } else if (form == 1) {
    if (M % vec || N % vec || splits < 1 || splits > 64 || !partial) return GEAR_ERR_INVALID;
    GEAR_HIP(launch_gemm_tn_splitk(dtype, A, B, M, N, K, splits, partial, status, s));
    GEAR_HIP(launch_fill_zero(out, (size_t)M * N * sizeof(float), s));
    const Optim minus = {-1.0f, 0.0f, 0.0f, 0.0f, 1.0f, 0};   // out = 0 - (-1) * sum of the partials
    const Moments none = {nullptr, nullptr};
    GEAR_HIP(launch_splitk_sgd(partial, splits, (int64_t)M * N, (float *)out, minus, none, status, s));
  } else {
    return GEAR_ERR_INVALID;
  }
  return GEAR_OK;
}

void gear_debug_fail_launch(int32_t nth) { g_fail_at = nth > 0 ? nth : 0; }

int32_t gear_debug_helper_idle(void) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -1;
  std::lock_guard<std::mutex> lock(g_side_mutex);
  if (!g_side[dev].ready) return 1;
  const hipError_t e = hipStreamQuery(g_side[dev].stream);
  return e == hipSuccess ? 1 : (e == hipErrorNotReady ? 0 : -1);
}

gear_profile *gear_profile_create(void) {
  gear_profile *p = new (std::nothrow) gear_profile;
  if (!p) return nullptr;
  p->used = 0;
  int made = 0;  // events created so far, start[0], stop[0], start[1], ...
  for (; made < 2 * gear_profile::kMaxSpans; ++made) {
    const int i = made / 2;
    p->name[i] = "";
    if (hipEventCreate(made % 2 ? &p->stop[i] : &p->start[i]) != hipSuccess) break;
  }
  if (made < 2 * gear_profile::kMaxSpans) {
    for (int e = 0; e < made; ++e) (void)hipEventDestroy(e % 2 ? p->stop[e / 2] : p->start[e / 2]);
    delete p;
    return nullptr;
  }
  return p;
}

void gear_profile_destroy(gear_profile *p) {
  if (!p) return;
  for (int i = 0; i < gear_profile::kMaxSpans; ++i) {
    (void)hipEventDestroy(p->start[i]);
    (void)hipEventDestroy(p->stop[i]);
  }
  delete p;
}

int32_t gear_profile_count(const gear_profile *p) { return p ? p->used : 0; }

gear_status gear_profile_span(const gear_profile *p, int32_t i, const char **name, float *ms) {
  if (!p || !name || !ms || i < 0 || i >= p->used) return GEAR_ERR_INVALID;
  *name = p->name[i];
  GEAR_HIP(hipEventElapsedTime(ms, p->start[i], p->stop[i]));
  return GEAR_OK;
}

const char *gear_status_string(gear_status st) {
  switch (st) {
    case GEAR_OK: return "ok";
    case GEAR_ERR_INVALID: return "invalid argument";
    case GEAR_ERR_RANGE: return "id out of range or offsets not a CSR index";
    case GEAR_ERR_CAPACITY: return "workspace or ready list too small";
    case GEAR_ERR_HIP: return "HIP call failed";
  }
  return "unknown status";
}

}  // extern "C"
