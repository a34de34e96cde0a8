/*
 * libgear - the Gear Training sparse-part step on one MI355X (gfx950).
 *
 * "Gear Training: A new way to implement high-performance model-parallel
 * training" splits a model into a Sparse Part (user id, URL, ...) trained every
 * step by a Fastgear Worker and a Dense Part (image CNN) owned by a Slowgear
 * Worker.  The Dense Part is neither run forward nor backward in a training
 * step: its outputs, the Dense Feature Vectors (DFVs), are fetched from a cache
 * by image id (Section 1, second point; Section 3, steps 1-3), and the
 * gradients with respect to the DFVs are collected per image until M have
 * arrived and are then averaged (Section 1, third point; Section 3, step 6).
 *
 * This library is that per-step work.  All pointers named "device" are device
 * memory owned by the caller; the library allocates no device memory and keeps
 * no state between calls except one helper stream and three events per device,
 * created at the first gear_step (default priority; part of a step runs on it,
 * forked from and joined back into the caller's stream).  Calls enqueue their
 * kernels on the given hipStream_t (passed as void*) and return without
 * synchronising.  Results are valid once the caller has synchronised that
 * stream.  The stream must belong to the current device.  The entry points may
 * be called from several host threads; steps issued on one device are enqueued
 * one after the other (a per-device lock is held while a step enqueues) and
 * share the helper stream, so they run in the order they were issued.  Each
 * step needs a workspace of its own while it is in flight.  If a call returns
 * GEAR_ERR_HIP part-way through its enqueue, whatever it had put on the helper
 * stream is still joined back into the caller's stream before it returns.
 *
 * Errors.  Everything the host can check (NULL pointers, dimensions, M < 1,
 * sizes over the configured maxima, a workspace that is too small) is reported
 * through the return value and nothing is enqueued.  What only the device can
 * see (an id outside its table, offsets that are not a CSR index, a ready list
 * longer than ready_cap) is written to the device word `status`, and the step
 * then leaves every table, accumulator and counter as it was.
 */
#ifndef GEAR_H
#define GEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GEAR_MAX_LAYERS 8

typedef enum gear_status {
  GEAR_OK = 0,
  GEAR_ERR_INVALID = 1,  /* host-checked: NULL, bad dims, M < 1, lr not finite, B or nnz over max */
  GEAR_ERR_RANGE = 2,    /* device-checked: id out of range, offsets not a CSR index            */
  GEAR_ERR_CAPACITY = 3, /* workspace too small (host) or ready list over ready_cap (device)    */
  GEAR_ERR_HIP = 4       /* a HIP call failed                                                    */
} gear_status;

typedef enum gear_dtype { GEAR_F32 = 0, GEAR_BF16 = 1 } gear_dtype;

/* Shape of the Sparse Part and of the tables.  Plain data, read by every call.
 * The Sparse Part is x = [user row | URL row | mean of the view's DFVs] of width
 * F = 2*emb_dim + dfv_dim, followed by n_layers affine layers of output widths
 * layer_out[0..n_layers-1] with ReLU between them; the last width must be 1 (the
 * logit).  Requirements: 2 <= n_layers <= GEAR_MAX_LAYERS, emb_dim % 8 == 0,
 * dfv_dim % 8 == 0, hidden widths % 8 == 0, last hidden width <= 1024, table sizes below 2^31. */
typedef struct gear_config {
  int64_t n_users, n_urls, n_images;
  int32_t emb_dim, dfv_dim;
  int32_t n_layers;
  int32_t layer_out[GEAR_MAX_LAYERS];
  int32_t emb_dtype;     /* gear_dtype of user_emb / url_emb rows                              */
  int32_t dfv_dtype;     /* gear_dtype of dfv_cache rows                                       */
  int32_t mlp_dtype;     /* operand type of the MLP contractions; accumulation is always fp32  */
  int32_t max_batch;     /* largest B a step may carry                                         */
  int32_t max_nnz;       /* largest number of (view, image) occurrences a step may carry       */
  uint64_t seed;         /* seed of gear_init_tables                                           */
  float emb_init_std;    /* standard deviation of the initial embedding rows                   */
} gear_config;

/* Trainable state of the Sparse Part (device).  mlp_params packs, layer after layer,
 * W_l [layer_out[l] x in_l] row-major then b_l [layer_out[l]], all fp32 (master copy). */
typedef struct gear_tables {
  void *user_emb;        /* [n_users x emb_dim], emb_dtype, row-major */
  void *url_emb;         /* [n_urls  x emb_dim], emb_dtype, row-major */
  float *mlp_params;     /* gear_mlp_param_count(cfg) floats          */
} gear_tables;

/* One batch of page views (Section 1, Table 1: user id, URL, several image ids).
 * All arrays are device memory.  View b owns img_id[img_off[b] .. img_off[b+1]);
 * img_off[0] = 0, img_off[B] = nnz.  A view may have no image (its pooled DFV is 0
 * and it produces no DFV gradient).  The same image may occur several times, also
 * inside one view; every occurrence counts. */
typedef struct gear_batch {
  int32_t B, nnz;
  const int32_t *user_id; /* [B]   in [0, n_users)        */
  const int32_t *url_id;  /* [B]   URL hash bucket in [0, n_urls) */
  const int32_t *img_off; /* [B+1]                         */
  const int32_t *img_id;  /* [nnz] in [0, n_images)        */
  const float *label;     /* [B]   click label in {0, 1}   */
} gear_batch;

/* Outputs of one step (device memory, caller-owned). */
typedef struct gear_step_out {
  float *loss;            /* [1] mean sigmoid cross-entropy of the batch                         */
  int32_t *n_ready;       /* [1] number of emitted averages (0 when status is not 0)             */
  int32_t *ready_ids;     /* [ready_cap] image ids, ascending; an image that completed several
                             groups of M in this step appears once per group, oldest first       */
  float *ready_grads;     /* [ready_cap x dfv_dim] fp32, row r = average for ready_ids[r]        */
  int32_t ready_cap;      /* rows available; max_nnz is always enough                            */
  int32_t *status;        /* [1] 0, GEAR_ERR_RANGE or GEAR_ERR_CAPACITY                          */
  /* Optional exports of the image grouping (NULL = skip).  Sizes: [max_nnz], [max_nnz+1],
   * [max_nnz], [1].  unique = distinct image ids ascending; segment s of the stable
   * permutation perm is perm[segoff[s] .. segoff[s+1]), flat CSR positions ascending. */
  int32_t *dbg_img_unique, *dbg_img_segoff, *dbg_img_perm, *dbg_n_img_unique;
  /* Optional timing (NULL = off): a gear_profile from gear_profile_create.  Every kernel launch of
   * the step is then bracketed by HIP events on the stream it is launched on (the caller's or the
   * helper stream); read them with gear_profile_span after synchronising the caller's stream. */
  void *profile;
  /* Nonzero: every kernel of the step is launched on the caller's stream, one after another, and
   * the helper stream is not used.  Same results; for timing each kernel alone, or for callers
   * that want no second stream. */
  int32_t one_stream;
} gear_step_out;

/* Bytes of scratch device memory gear_step needs for this configuration (0 on a bad config). */
size_t gear_workspace_bytes(const gear_config *cfg);

/* Number of floats in gear_tables.mlp_params, and the float offset of W_l (which = 0) or
 * b_l (which = 1) inside it; -1 on a bad argument. */
int64_t gear_mlp_param_count(const gear_config *cfg);
int64_t gear_mlp_param_offset(const gear_config *cfg, int32_t layer, int32_t which);

/* Byte offset and size, inside the workspace, of an intermediate of the last gear_step, for
 * inspection by tests: "x" [max_batch x F] mlp_dtype, "logits" [max_batch] f32, and dLoss/dx in two
 * pieces: "dx_emb" [max_batch x 2*emb_dim] f32 (user and URL slots) and "dx_dfv" [max_batch x dfv_dim]
 * in mlp_dtype (the DFV slot), and "h0", "h1", ... [max_batch x layer_out[l]] mlp_dtype, the stored
 * activations of the hidden layers (zero where the unit is off).
 * Returns GEAR_ERR_INVALID for an unknown name. */
gear_status gear_workspace_region(const gear_config *cfg, const char *name, size_t *offset, size_t *bytes);

/* Fill dst [n_rows x dim] (device, `dtype`) with zero-mean noise of standard deviation `std`:
 * element (r, c) is a fixed function of (seed, stream_id, r*dim + c) - Philox4x32-10 with counter
 * (idx_lo, idx_hi, stream_id, 0) and key (seed_lo, seed_hi); the eight 16-bit halves of its output
 * are summed, centred, and scaled by one fp32 multiply.  (Section 4.1 fixes only a standard
 * deviation for the initial values.) */
gear_status gear_fill_normal(void *dst, int32_t dtype, int64_t n_rows, int32_t dim, uint64_t seed,
                             uint32_t stream_id, float std, void *stream);

/* Initial state: user_emb (stream 1) and url_emb (stream 2) ~ N(0, emb_init_std^2); W_l (stream
 * 16+l) ~ N(0, 2/in_l), b_l = 0; grad_accum [n_images x dfv_dim] f32 and counts [n_images] i32
 * zeroed (no gradient has arrived yet: Section 1, third point). */
gear_status gear_init_tables(const gear_config *cfg, gear_tables *tables, float *grad_accum,
                             int32_t *counts, void *stream);

/* One Fastgear training step (Section 3, steps 4 and 5) plus the Slowgear gradient bookkeeping
 * (Section 1, third point; Section 3, step 6; Eq. 1, left factor):
 *   x_b   = [user_emb[user_b] | url_emb[url_b] | mean_j dfv_cache[img_j]]
 *   loss  = mean_b BCE(sigmoid(MLP(x_b)), label_b)
 *   MLP parameters and the touched embedding rows take one SGD step with rate lr, gradients
 *     of a row summed over its views in batch order;
 *   every occurrence j of image i in view b contributes g_j = dLoss/dx_b[DFV slot] / n_b;
 *   the gradients of image i, in flat CSR order and continuing from earlier steps, are cut into
 *     groups of M: a completed group is emitted as (i, mean of the group) and forgotten, an
 *     unfinished one stays summed in grad_accum[i];  counts[i] += occurrences of i.
 * dfv_cache [n_images x dfv_dim] (dfv_dtype) is read only.  grad_accum [n_images x dfv_dim] f32 and
 * counts [n_images] i32 must be the arrays given to gear_init_tables and M must not change over
 * their life.  workspace: gear_workspace_bytes(cfg) bytes, 256-byte aligned; the tables,
 * mlp_params, dfv_cache, grad_accum and ready_grads 16-byte aligned.  Results do not depend on the
 * order in which the device schedules its work. */
gear_status gear_step(const gear_config *cfg, const gear_batch *batch, gear_tables *tables,
                      const void *dfv_cache, float *grad_accum, int32_t *counts, int32_t M, float lr,
                      void *workspace, size_t workspace_bytes, gear_step_out *out, void *stream);

/* gear_step for callers that cannot allocate device memory or must not see an allocation happen:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace
 * is a static device array inside the library (64 MiB = 67 108 864 bytes per GPU, held until the
 * process ends) instead of a caller's buffer, and every kernel is launched on the caller's stream
 * (no helper stream, no event).  The call allocates nothing.  Configurations whose
 * gear_workspace_bytes(cfg) exceeds 67 108 864 are rejected with GEAR_ERR_CAPACITY and nothing is
 * enqueued (of the workloads this library is measured on that admits batches of about 8 000 views
 * with 256-wide DFVs; the largest needs 760 MiB and has to bring its own workspace to gear_step).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two host threads) race on it and must be ordered by the caller; nothing in it has to survive
 * between calls and nothing in it has to be cleared beforehand.  Inputs, outputs, alignment, errors
 * and results (bit for bit) as for gear_step with one_stream set. */
gear_status gear_step_static(const gear_config *cfg, const gear_batch *batch, gear_tables *tables,
                             const void *dfv_cache, float *grad_accum, int32_t *counts, int32_t M, float lr,
                             gear_step_out *out, void *stream);

/* Adam for the Sparse Part (Section 4.1 trains with the Adam optimiser at rate 1e-4; its other
 * constants are not given).  Kingma & Ba, Algorithm 1, at step t = 1, 2, ...:
 *   m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2;
 *   w -= lr / (1 - beta1^t) * m / (sqrt(v) / sqrt(1 - beta2^t) + eps).
 * MLP parameters: every element every step; mlp_m, mlp_v are laid out like mlp_params.  Embedding
 * rows: only the rows a step touches move, moments included (their decay is applied per touch, not
 * per elapsed step), with the global t in the bias corrections; user_m/v and url_m/v are fp32 tables
 * [n x emb_dim] whatever emb_dtype is.  All moment arrays are device memory, caller-owned, 16-byte
 * aligned, zero before the first step. */
typedef struct {
  float beta1, beta2, eps;
  int32_t t;                  /* this step's number, from 1 */
  float *user_m, *user_v;     /* [n_users x emb_dim] */
  float *url_m, *url_v;       /* [n_urls x emb_dim] */
  float *mlp_m, *mlp_v;       /* [gear_mlp_param_count] */
} gear_adam;

/* gear_step with Adam instead of plain SGD for every parameter of the Sparse Part; adam = NULL is
 * gear_step.  Everything else as for gear_step. */
gear_status gear_step_adam(const gear_config *cfg, const gear_batch *batch, gear_tables *tables,
                           const void *dfv_cache, float *grad_accum, int32_t *counts, int32_t M, float lr,
                           const gear_adam *adam, void *workspace, size_t workspace_bytes,
                           gear_step_out *out, void *stream);

/* Overwrite cached DFVs (Section 1, second point: cached inference results are replaced after the
 * inference expired time).  Row image_ids[r] of dfv_cache becomes new_dfv[r] (device, dfv_dtype,
 * [n x dfv_dim]); image_ids = NULL means rows 0..n-1.  Ids must be distinct.  Gradient accumulators
 * and counters are a different table and are not touched.  status (device word, may be NULL) is
 * set to GEAR_ERR_RANGE if an id is outside [0, n_images); such rows are skipped. */
gear_status gear_refresh_dfv(const gear_config *cfg, void *dfv_cache, const int32_t *image_ids,
                             const void *new_dfv, int64_t n, int32_t *status, void *stream);

/* Which cached inference results a batch asks for have expired (Section 1, second point and
 * Section 3: a cache entry is recomputed once it is older than the inference expired time;
 * Section 4.1, Table 2: that time trades freshness for speed).  dfv_stamp [n_images] i32 (device,
 * caller-owned) holds the time each row was last written, in the caller's unit (steps, seconds).
 * expired_ids (device, room for n entries) receives, ascending, the distinct ids among
 * image_ids [n] (device, a batch's flat image list) with now - dfv_stamp[id] >= expiry, and
 * n_expired (device word) their number.  The caller recomputes those rows and hands them to
 * gear_refresh_dfv and gear_stamp_dfv.  expiry >= 0.  status (device word, not NULL) becomes
 * GEAR_ERR_RANGE if an id is outside [0, n_images); then n_expired is 0.  workspace as for
 * gear_step, with max_nnz >= n. */
gear_status gear_expired_ids(const gear_config *cfg, const int32_t *image_ids, int32_t n,
                             const int32_t *dfv_stamp, int32_t now, int32_t expiry, void *workspace,
                             size_t workspace_bytes, int32_t *expired_ids, int32_t *n_expired,
                             int32_t *status, void *stream);

/* dfv_stamp[image_ids[r]] = now for r < n; image_ids = NULL means rows 0..n-1.  status (device
 * word, may be NULL) becomes GEAR_ERR_RANGE if an id is outside [0, n_images); such ids are skipped. */
gear_status gear_stamp_dfv(const gear_config *cfg, int32_t *dfv_stamp, const int32_t *image_ids, int64_t n,
                           int32_t now, int32_t *status, void *stream);

/* gear_refresh_dfv and gear_stamp_dfv for a list whose length is only known on the device (the
 * output of gear_expired_ids, say): rows r < *n_rows are used, where n_rows is a device word read
 * when the kernels run, 0 <= *n_rows <= max_rows (a larger value is cut to max_rows); image_ids and
 * new_dfv hold max_rows entries.  The host need not read the count and can keep enqueuing.
 * Otherwise as the calls above (image_ids must be given). */
gear_status gear_refresh_dfv_n(const gear_config *cfg, void *dfv_cache, const int32_t *image_ids,
                               const void *new_dfv, const int32_t *n_rows, int64_t max_rows, int32_t *status,
                               void *stream);
gear_status gear_stamp_dfv_n(const gear_config *cfg, int32_t *dfv_stamp, const int32_t *image_ids,
                             const int32_t *n_rows, int64_t max_rows, int32_t now, int32_t *status, void *stream);

/* A stand-in Dense Part, so that the loop of the method can be closed on one device: a linear map
 * DFV[i] = Wd raw[i] from fixed per-image features raw [n_images x raw_dim] (f32, device) with
 * weights Wd [dfv_dim x raw_dim] (f32, device).  Not the paper's CNN: the smallest model that has
 * an inference pass feeding the cache (Section 3, steps 1-2) and a backward pass consuming the
 * averaged gradients (Section 3, step 6; Eq. 1, right factor).  raw_dim and dfv_dim are multiples
 * of 8; max_rows bounds n and n_ready of the calls below. */
typedef struct {
  int64_t n_images;
  int32_t raw_dim, dfv_dim;
  gear_dtype dfv_dtype; /* type of the rows gear_dense_infer writes (the cache's) */
  int32_t max_rows;
} gear_dense_config;

size_t gear_dense_workspace_bytes(const gear_dense_config *cfg);

/* out_rows [n x dfv_dim] (device, dfv_dtype) = Wd raw[image_ids[r]]; image_ids = NULL means images
 * 0..n-1.  The rows are what gear_refresh_dfv takes.  workspace: gear_dense_workspace_bytes(cfg)
 * bytes, 256-byte aligned.  status (device word, not NULL): GEAR_ERR_RANGE if an id is outside
 * [0, n_images) (that row is then computed from image 0). */
gear_status gear_dense_infer(const gear_dense_config *cfg, const float *raw, const float *wd,
                             const int32_t *image_ids, int32_t n, void *out_rows, void *workspace,
                             size_t workspace_bytes, int32_t *status, void *stream);

/* Back-propagation of a step's ready list through the stand-in (Eq. 1, right factor):
 * Wd -= lr * sum_e ready_grads[e] (outer) raw[ready_ids[e]], e < n_ready (a host count: the caller
 * reads n_ready back first), summed in a fixed shape that depends on n_ready only.  status (device
 * word, not NULL): GEAR_ERR_RANGE if an id is outside [0, n_images); Wd is then unchanged. */
gear_status gear_dense_backward(const gear_dense_config *cfg, const float *raw, float *wd,
                                const int32_t *ready_ids, const float *ready_grads, int32_t n_ready,
                                float lr, void *workspace, size_t workspace_bytes, int32_t *status,
                                void *stream);

/* The same with the number of emissions read from the device word n_ready when the kernels run
 * (a step's gear_step_out.n_ready; at most max_rows, which ready_ids and ready_grads must hold): the
 * host need not read it back.  The sum is split into a fixed number of ranges over *n_ready. */
gear_status gear_dense_backward_n(const gear_dense_config *cfg, const float *raw, float *wd,
                                  const int32_t *ready_ids, const float *ready_grads, const int32_t *n_ready,
                                  float lr, void *workspace, size_t workspace_bytes, int32_t *status,
                                  void *stream);

/* Sort-by-key grouping used for the embedding updates and the per-image accumulation, exposed
 * for tests: keys [n] in [0, key_range) -> distinct keys ascending (unique [n]), segment offsets
 * (segoff [n+1]), stable permutation (perm [n]) and the number of distinct keys (n_unique [1]).
 * All device memory; workspace as for gear_step with max_batch, max_nnz >= n. */
gear_status gear_group_ids(const gear_config *cfg, const int32_t *keys, int32_t n, int64_t key_range,
                           void *workspace, size_t workspace_bytes, int32_t *unique, int32_t *segoff,
                           int32_t *perm, int32_t *n_unique, void *stream);

/* The MLP's matrix products (Section 3, step 4: forward and back-propagation on the Sparse Part),
 * exposed for tests.  All device memory, 16-byte aligned; accumulation is fp32.
 *   form 0 (forward / dgrad): out[M x N] = A[M x K] * B[N x K]^T, operands of `dtype`, K and N
 *     multiples of 8; epilogue 0: out(dtype) = max(acc + bias[n], 0); 1: out(dtype) = aux[m,n] > 0
 *     ? acc : 0 with aux [M x N] of `dtype`; 2: out(f32) = acc.
 *   form 1 (wgrad): out[M x N] (f32) = A[K x M]^T * B[K x N], M and N multiples of 8, contracted in
 *     `splits` (1..64) ranges of K whose partial results (partial: [splits x M x N] f32) are added in
 *     ascending order.
 * status: device word, must be 0 on entry (a non-zero word makes the kernels return at once). */
gear_status gear_gemm(int32_t dtype, int32_t form, const void *A, const void *B, int32_t M, int32_t N, int32_t K,
                      int32_t epilogue, const float *bias, const void *aux, void *out, int32_t splits,
                      float *partial, int32_t *status, void *stream);

/* Per-kernel timing of a step, for benchmarks.  gear_profile_create allocates a fixed pool of HIP
 * events on the current device (host memory; NULL on failure), gear_profile_destroy releases it.
 * After a gear_step that was given the profile and after the stream has been synchronised,
 * gear_profile_count returns the number of timed launches and gear_profile_span the name of
 * launch i (a static string) and its duration in milliseconds. */
typedef struct gear_profile gear_profile;
gear_profile *gear_profile_create(void);
void gear_profile_destroy(gear_profile *p);
int32_t gear_profile_count(const gear_profile *p);
gear_status gear_profile_span(const gear_profile *p, int32_t i, const char **name, float *ms);

/* Test hooks for the error paths of a step (no device needs to fail for them to be walked).
 * gear_debug_fail_launch(n): on the calling thread, the n-th kernel launch counted from now (n >= 1)
 * is not enqueued and the step returns GEAR_ERR_HIP there, leaving caller state half-updated as any
 * failed launch would; 0 switches it off.  gear_debug_helper_idle(): 1 if the current device's helper
 * stream has nothing left to run (or was never created), 0 if it is still busy, -1 on a HIP error. */
void gear_debug_fail_launch(int32_t nth);
int32_t gear_debug_helper_idle(void);

const char *gear_status_string(gear_status s);

#ifdef __cplusplus
}
#endif
#endif /* GEAR_H */
