/*
 * abs_sgd.h -- C ABI of the MI355X (gfx950) library for the data-parallel hot
 * path of ABS-SGD (delayed synchronous SGD with adaptive batch size).
 *
 * Vocabulary (the paper's Algorithm 1 in brackets):
 *   P          number of parameters                      [n]
 *   K          number of workers                         [N]
 *   n_samples  samples in one micro-batch                [M_r, reference batch size]
 *   acc        a worker's running gradient accumulator   [G_t^i], fp32, P elements
 *   count      samples accumulated so far in acc         [M_t^i], int64, exact
 *   grad       MEAN gradient of one micro-batch, fp32 or bf16; the sum of its
 *              per-sample gradients is n_samples * grad
 *   params     x, fp32;  momentum  v, fp32
 *
 * Conventions for every entry point
 *   - Pointers marked DEVICE address memory of the current HIP device, owned by
 *     the caller; the library never allocates, frees or keeps P-sized memory.
 *     Pointers marked HOST are ordinary process memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Kernels are enqueued on it and the call returns without waiting.
 *   - fp32 buffers must be 4-byte aligned, bf16 buffers 2-byte aligned; 16-byte
 *     aligned bases take the 128-bit path, others a slower element-wise path
 *     with identical results.
 *   - Return value: ABS_OK (0); ABS_EMPTY (1): nothing to apply, no memory
 *     touched, not an error; ABS_EINVAL (-1): bad argument, nothing enqueued;
 *     ABS_EHIP (-2): a HIP runtime call failed, abs_last_hip_error() has its code.
 *     Nothing is thrown across this boundary.
 *   - Arithmetic is fp32 in one fixed order (stated per call) so results are
 *     reproducible bit for bit; sample counts are integers.
 *   - Threads: calls on different objects (layouts, tensor sets, contexts) and
 *     the stateless calls may run concurrently from several host threads; one
 *     object is used by one thread at a time (a layout uploads its tables on
 *     first use, a context keeps host counts), and the two tuning calls
 *     (abs_set_launch_tuning, abs_set_cache_policy) change process-wide settings
 *     and must not run while another thread is inside the library.
 *   - Devices: everything runs on the HIP device that is current at the call,
 *     on the caller's streams.  A layout keeps its tables on the device that was
 *     current at its first use in a ragged call; a ragged call with another
 *     device current returns ABS_EINVAL.  Create a layout's tensor sets with
 *     that same device current.
 */
#ifndef ABS_SGD_H
#define ABS_SGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ABS_MAX_K 64    /* most workers one sync-update may combine */
#define ABS_MAX_BATCH 8 /* most gradients one accumulate launch folds in */

enum { ABS_OK = 0, ABS_EMPTY = 1, ABS_EINVAL = -1, ABS_EHIP = -2 };

typedef enum { ABS_F32 = 0, ABS_BF16 = 1 } abs_dtype;

/* Library version (major*10000 + minor*100 + patch). */
int abs_version(void);
/* hipError_t of the last failed HIP call made by this thread through the library. */
int abs_last_hip_error(void);
/* Static, human-readable text for a return code. */
const char *abs_error_string(int rc);
/* Elements in one workgroup row (threads per workgroup x 4); every tile, and every
 * ragged chunk, is a whole number of rows. */
int64_t abs_row_elems(void);

/* Launch shape.  A launch gives each workgroup one tile of consecutive rows,
 * sized so the grid fills the GPU in whole rounds of resident workgroups.
 * blocks_per_cu: resident workgroups per CU to plan for (0 = default: what the
 * kernel's register use allows).  max_rows_per_tile: cap on the tile (default 4;
 * 0 = none: one round, each workgroup walks one long run).  Affects later launches and
 * later abs_layout_create calls; results never change.  Process-wide. */
int abs_set_launch_tuning(int blocks_per_cu, int max_rows_per_tile);

/* Cache policy of the kernels.  Accumulators, x and v are re-read soon after a
 * launch (next micro-batch, next iteration).  Each kernel has a cached flavour
 * and a streaming one (non-temporal accesses to those buffers); results are
 * identical.  Mode -1 (default) picks per launch from the buffer sizes: cached
 * while the working set fits the GPU's memory-side cache, streaming beyond.
 * 0 forces cached, 1 forces streaming.  Process-wide; not thread-safe against
 * concurrent launches.  EINVAL for other values. */
int abs_set_cache_policy(int accumulate_mode, int update_mode);

/* ------------------------------------------------------------------------
 * (1) Gradient accumulation -- Algorithm 1, Step 2 (inner loop and its
 *     initialisation G_t^i = 0, M_t^i = 0).
 *
 *   first = (*count == 0), i.e. first micro-batch since the accumulator was
 *           reset (creation or swap).  Then, for every i < P,
 *     acc[i] = first ? (float)n_samples * g[i]
 *                    : fmaf((float)n_samples, g[i], acc[i])
 *   with g[i] the fp32 value of grad[i] (bf16 widens exactly), and
 *     *count += n_samples.
 *   Overwriting on the first call is the paper's zero initialisation without a
 *   separate pass over memory.
 *
 *   acc   DEVICE, P floats, read (unless first) and written
 *   grad  DEVICE, P elements of grad_dtype, read only
 *   count HOST, read and updated before the call returns
 *   P = 0 is allowed (only the count moves).  EINVAL: null pointer, P < 0,
 *   n_samples <= 0, *count < 0, count overflow, misaligned base, bad dtype.
 * ---------------------------------------------------------------------- */
int abs_accumulate(float *acc, const void *grad, abs_dtype grad_dtype, int64_t P,
                   int64_t n_samples, int64_t *count, void *stream);

/* (1') Batched accumulation: the J micro-batch gradients a worker has ready are
 *     folded into its accumulator in ONE pass, in order j = 0..J-1, with exactly
 *     the roundings of J successive abs_accumulate calls (same bits), but the
 *     accumulator is read and written once: J*g_b + 8 bytes per parameter
 *     instead of J*(g_b + 8).  Launches fold at most ABS_MAX_BATCH gradients;
 *     a larger J is split into several launches.
 *
 *   grads      HOST array of J DEVICE pointers, each P elements of grad_dtype
 *   n_samples  HOST array of J sample counts (each > 0);  *count += their sum
 *   Errors as abs_accumulate; J < 1 is EINVAL.  If a HIP error stops a call that
 *   needed several launches, earlier launches have already been enqueued and
 *   *count is left unchanged: treat the accumulator as undefined. */
int abs_accumulate_batch(float *acc, const void *const *grads, abs_dtype grad_dtype, int J,
                         int64_t P, const int64_t *n_samples, int64_t *count, void *stream);

/* ------------------------------------------------------------------------
 * (2)+(3) Weighted combination of the K delayed accumulators and the delayed
 *     parameter update -- Algorithm 1, Step 1 (weighted gradient averaging)
 *     and the update line; momentum and weight decay wrap the paper's plain
 *     SGD step and vanish for mu = 0, wd = 0.
 *
 *   M = sum_k counts[k].  M == 0 -> ABS_EMPTY (the first iteration: G_{-1} = 0).
 *   Workers with counts[k] == 0 are skipped; their buffers are never read (they
 *   may hold stale data because accumulation overwrites instead of zeroing).
 *   For every i < P, over the non-empty workers in ascending k:
 *     s    = acc[k0][i];  s = s + acc[k][i] ...
 *     Gbar = s / (float)M              (correctly rounded divide)
 *     d    = fmaf(wd, x[i], Gbar)
 *     v[i] = fmaf(mu, v[i], d)
 *     x[i] = fmaf(-lr, v[i], x[i])
 *   One read pass over the K buffers, fused with the reads and writes of x, v.
 *
 *   params, momentum  DEVICE, P floats, read and written
 *   acc     HOST array of K DEVICE pointers (each P floats, read only)
 *   counts  HOST array of K int64
 *   EINVAL: null pointer, K < 1 or K > ABS_MAX_K, P < 0, a negative count,
 *   misaligned base.
 * ---------------------------------------------------------------------- */
int abs_sync_update(float *params, float *momentum, const float *const *acc,
                    const int64_t *counts, int K, int64_t P, float lr, float mu, float wd,
                    void *stream);

/* ------------------------------------------------------------------------
 * (3') The same with delayed gradient compensation -- Algorithm 1, "Compensate
 *     delayed gradients" (third mechanism of Section "Algorithm"):
 *       Gtilde = Gbar + lambda * Gbar (.) Gbar (.) (x_t - x_{t-1})   element-wise,
 *     used in place of Gbar.  The previous iterate x_{t-1} lives in a caller-owned
 *     buffer (the memory overhead the paper mentions): +8 B/param of traffic.
 *
 *   Order after Gbar: q = Gbar*Gbar; c = lambda*q; diff = x[i] - xp[i];
 *     Gtilde = fmaf(c, diff, Gbar); d = fmaf(wd, x[i], Gtilde); v[i] = fmaf(mu, v[i], d);
 *     xp[i] = x[i] (the value on entry); x[i] = fmaf(-lr, v[i], x[i]).
 *
 *   params_prev  DEVICE, P floats, read and written.  The caller initialises it
 *     to a copy of params before the first call (then x_t - x_{t-1} = 0 and the
 *     first applied step is uncompensated, as in the paper where x_{-1} does not
 *     exist).  When the total count is 0 the call copies params into params_prev
 *     (x_{t+1} = x_t, so the next difference is 0) and returns ABS_EMPTY; this is
 *     the one case in which ABS_EMPTY touches memory.
 *   Other arguments, errors: as abs_sync_update; params_prev must differ from
 *   params and momentum.
 * ---------------------------------------------------------------------- */
int abs_sync_update_dc(float *params, float *params_prev, float *momentum, const float *const *acc,
                       const int64_t *counts, int K, int64_t P, float lr, float mu, float wd,
                       float lambda, void *stream);

/* ------------------------------------------------------------------------
 * (3'm) The same compensation (Algorithm 1, "Compensate delayed gradients")
 *     without a stored x_{t-1}: every applied update of this family is
 *     x_t = x_{t-1} - lr_{t-1} * v_t, so x_t - x_{t-1} = -lr_{t-1} * v_t with v_t
 *     the momentum as it stands on entry.  Equal to abs_sync_update_dc in exact
 *     arithmetic (in fp32 it differs by the rounding of the previous write of x);
 *     traffic is that of abs_sync_update, 4K + 16 B/param.
 *
 *   Order after Gbar: q = Gbar*Gbar; c = lambda*q; diff = (-lr_prev) * v[i];
 *     Gtilde = fmaf(c, diff, Gbar); d = fmaf(wd, x[i], Gtilde); v[i] = fmaf(mu, v[i], d);
 *     x[i] = fmaf(-lr, v[i], x[i]).
 *
 *   lr_prev  the lr of the update that produced the current params from the
 *     previous ones through this family of calls; 0 when there was none, or when
 *     the previous iteration returned ABS_EMPTY (x_t = x_{t-1}).  Only valid while
 *     momentum is the v of that previous update, untouched since.
 *   Other arguments, errors, ABS_EMPTY (no memory touched): as abs_sync_update.
 * ---------------------------------------------------------------------- */
int abs_sync_update_dcm(float *params, float *momentum, const float *const *acc,
                        const int64_t *counts, int K, int64_t P, float lr, float mu, float wd,
                        float lambda, float lr_prev, void *stream);

/* ------------------------------------------------------------------------
 * (3'') Adam behind the delayed synchronous mechanism -- the update rule the
 *     paper's Section "Conclusions and Future Work" names as its next step.
 *     Same read pass over the K delayed accumulators; the state is the first
 *     and second moment instead of the momentum: 4K + 24 B/param.
 *
 *   step >= 1 is the index of this update among the APPLIED ones (the caller
 *   advances it when the call returns ABS_OK, not on ABS_EMPTY).  Order after Gbar:
 *     g = fmaf(wd, x, Gbar)                      (coupled weight decay)
 *     m = fmaf(beta1, m, (1-beta1)*g);  v = fmaf(beta2, v, (1-beta2)*(g*g))
 *       with (1-beta) rounded to fp32 once
 *     mh = m / bc1;  vh = v / bc2;   bc = (float)(1 - beta^step), evaluated in double
 *     x = fmaf(-lr, mh / (sqrtf(vh) + eps), x)    (correctly rounded divide and sqrt)
 *
 *   exp_avg, exp_avg_sq  DEVICE, P floats each, read and written (start at 0)
 *   EINVAL also for step < 1, beta outside [0, 1), eps < 0.
 * ---------------------------------------------------------------------- */
int abs_sync_update_adam(float *params, float *exp_avg, float *exp_avg_sq, const float *const *acc,
                         const int64_t *counts, int K, int64_t P, float lr, float beta1, float beta2,
                         float eps, float wd, int64_t step, void *stream);

/* ------------------------------------------------------------------------
 * Ragged (multi-tensor) layouts: the parameter vector of Section "Problem
 * definition" split into T separately allocated tensors of arbitrary sizes.
 * One launch covers all tensors.
 *
 * abs_layout    sizes only; built on the host (needs no GPU).  It cuts every
 *               tensor into chunks of abs_layout_tile() elements, one per
 *               workgroup; the chunk table is copied to the device the first
 *               time a launch needs it.
 * abs_tensorset T DEVICE base pointers for one logical vector (x, v, one
 *               worker's accumulator, one gradient) laid out per the layout;
 *               the pointer table is copied to device memory at creation.
 *               The tensors stay owned by the caller and must outlive the set.
 * ---------------------------------------------------------------------- */
typedef struct abs_layout abs_layout;
typedef struct abs_tensorset abs_tensorset;

/* sizes: HOST array of T element counts (each >= 0; T >= 1). */
int abs_layout_create(abs_layout **out, int T, const int64_t *sizes);
int abs_layout_destroy(abs_layout *layout);
int abs_layout_num_tensors(const abs_layout *layout);
int64_t abs_layout_total(const abs_layout *layout);
int64_t abs_layout_num_chunks(const abs_layout *layout);
/* Elements per chunk of this layout (a multiple of abs_row_elems()). */
int64_t abs_layout_tile(const abs_layout *layout);
/* Chunk c covers elements [*offset, *offset + *len) of tensor *tensor. */
int abs_layout_chunk(const abs_layout *layout, int64_t c, int *tensor, int64_t *offset,
                     int64_t *len);

/* ptrs: HOST array of T DEVICE pointers; elem: element type of the tensors.
 * A tensor of size 0 may have a null pointer. */
int abs_tensorset_create(abs_tensorset **out, const abs_layout *layout, void *const *ptrs,
                         abs_dtype elem);
int abs_tensorset_destroy(abs_tensorset *set);

/* Same arithmetic as abs_accumulate over every tensor of the layout; one count
 * for the whole vector.  acc must be an ABS_F32 set; grad may be F32 or BF16. */
int abs_accumulate_mt(abs_layout *layout, const abs_tensorset *acc,
                      const abs_tensorset *grad, int64_t n_samples, int64_t *count,
                      void *stream);

/* abs_accumulate_batch over every tensor of the layout.  grads: HOST array of J
 * sets of one element type. */
int abs_accumulate_batch_mt(abs_layout *layout, const abs_tensorset *acc,
                            const abs_tensorset *const *grads, int J, const int64_t *n_samples,
                            int64_t *count, void *stream);

/* Same arithmetic as abs_sync_update over every tensor of the layout.
 * acc: HOST array of K sets; counts: HOST array of K int64. */
int abs_sync_update_mt(abs_layout *layout, const abs_tensorset *params,
                       const abs_tensorset *momentum, const abs_tensorset *const *acc,
                       const int64_t *counts, int K, float lr, float mu, float wd,
                       void *stream);

/* abs_sync_update_dc over every tensor of the layout; params_prev an ABS_F32 set. */
int abs_sync_update_dc_mt(abs_layout *layout, const abs_tensorset *params,
                          const abs_tensorset *params_prev, const abs_tensorset *momentum,
                          const abs_tensorset *const *acc, const int64_t *counts, int K, float lr,
                          float mu, float wd, float lambda, void *stream);

/* abs_sync_update_dcm over every tensor of the layout. */
int abs_sync_update_dcm_mt(abs_layout *layout, const abs_tensorset *params,
                           const abs_tensorset *momentum, const abs_tensorset *const *acc,
                           const int64_t *counts, int K, float lr, float mu, float wd, float lambda,
                           float lr_prev, void *stream);

/* abs_sync_update_adam over every tensor of the layout. */
int abs_sync_update_adam_mt(abs_layout *layout, const abs_tensorset *params,
                            const abs_tensorset *exp_avg, const abs_tensorset *exp_avg_sq,
                            const abs_tensorset *const *acc, const int64_t *counts, int K, float lr,
                            float beta1, float beta2, float eps, float wd, int64_t step, void *stream);

/* LARS behind the delayed synchronous mechanism -- the other rule the paper's
 * Section "Conclusions and Future Work" names.  Layer = tensor of the layout.  Per
 * tensor l, with g_l the delayed weighted average Gbar restricted to it:
 *     rate_l = eta * ||x_l|| / (||g_l|| + wd * ||x_l||)      (1 if either norm is 0)
 *     v = fmaf(mu, v, step_l * fmaf(wd, x, Gbar)),  step_l = (float)(lr * rate_l);   x = x - v
 * Norms are accumulated in double in a fixed order (results do not depend on
 * timing).  Three launches: Gbar and the sums of squares (4K + 8 B/param), the
 * per-tensor rates, the update (20 B/param).
 *
 *   gbar  an ABS_F32 set over the layout, caller-owned workspace: it receives Gbar
 *         and must differ from every other set of the call.
 *   The per-chunk sums and per-tensor rates live in device memory owned by the
 *   layout (allocated on the first LARS call): two LARS calls on one layout must
 *   not overlap in time.  A flat vector is a layout of one tensor.
 *   Other arguments, ABS_EMPTY and errors: as abs_sync_update_mt. */
int abs_sync_update_lars_mt(abs_layout *layout, const abs_tensorset *params,
                            const abs_tensorset *momentum, const abs_tensorset *gbar,
                            const abs_tensorset *const *acc, const int64_t *counts, int K, float lr,
                            float mu, float wd, float eta, void *stream);

/* ------------------------------------------------------------------------
 * (4) Double buffer -- Algorithm 1, "Run Step 1 and Step 2 in parallel": two
 *     generations of (K accumulators, K counts).  Accumulation of batch t runs
 *     on stream_acc into the CURRENT generation while the sync-update of batch
 *     t-1 runs on stream_upd from the PREVIOUS one.
 *
 * The context owns only indices, the 2*K host counts and two HIP events; the
 * accumulators stay the caller's.  All counts start at 0 (G_{-1} = 0).
 * stream_acc == stream_upd gives the serial order on one stream.
 * ---------------------------------------------------------------------- */
typedef struct abs_ctx abs_ctx;

/* acc_A, acc_B: HOST arrays of K DEVICE pointers, P floats each. */
int abs_ctx_create(abs_ctx **out, int K, int64_t P, float *const *acc_A, float *const *acc_B,
                   void *stream_acc, void *stream_upd);
/* Ragged form: acc_A, acc_B are HOST arrays of K ABS_F32 sets over `layout`. */
int abs_ctx_create_mt(abs_ctx **out, int K, abs_layout *layout,
                      const abs_tensorset *const *acc_A, const abs_tensorset *const *acc_B,
                      void *stream_acc, void *stream_upd);
int abs_ctx_destroy(abs_ctx *ctx);

/* Optional: spread accumulation over n streams, worker k on streams[k % n]
 * (replaces stream_acc).  The K workers of Algorithm 1 compute at the same
 * time; their accumulators are independent, so their launches may overlap,
 * which hides launch ramp-up and drain when P is small.  A worker's own
 * launches of a step stay ordered on one stream.  With fewer streams than
 * workers, abs_swap_buffers re-places the workers for the next step so that the
 * streams carry about equal numbers of launches, forecasting from the step just
 * finished (initially worker k is on streams[k % n]).  Only before the first accumulate;
 * EINVAL afterwards, or for n < 1, n > ABS_MAX_K.  streams: HOST array. */
int abs_ctx_set_accumulate_streams(abs_ctx *ctx, void *const *streams, int n);

/* How many accumulate streams to give a context over K workers with P-element
 * accumulators (Algorithm 1's Step 2 of different workers is independent work):
 * 2 while 24 MiB <= 4*P <= 112 MiB and K >= 2, else 1.  Measured on MI355X with
 * the sync-update on a stream of its own: two streams hide launch ramp-up and
 * drain in that range (+3 to +12 % per step); below it the event joins cost
 * more than they hide (-3 to -25 %), above it concurrent launches push each
 * other out of the memory-side cache (-4 %); four streams never beat two.
 * With 1, accumulate and sync-update are best put on one stream too. */
int abs_suggest_accumulate_streams(int64_t P, int K);

/* abs_accumulate into worker k's CURRENT accumulator, on that worker's
 * accumulate stream. */
int abs_ctx_accumulate(abs_ctx *ctx, int k, const void *grad, abs_dtype grad_dtype,
                       int64_t n_samples);
int abs_ctx_accumulate_mt(abs_ctx *ctx, int k, const abs_tensorset *grad, int64_t n_samples);
/* Batched forms (abs_accumulate_batch) into worker k's CURRENT accumulator. */
int abs_ctx_accumulate_batch(abs_ctx *ctx, int k, const void *const *grads, abs_dtype grad_dtype,
                             int J, const int64_t *n_samples);
int abs_ctx_accumulate_batch_mt(abs_ctx *ctx, int k, const abs_tensorset *const *grads, int J,
                                const int64_t *n_samples);

/* abs_sync_update from the PREVIOUS generation, on stream_upd.  ABS_EMPTY in
 * the first iteration. */
int abs_ctx_sync_update(abs_ctx *ctx, float *params, float *momentum, float lr, float mu,
                        float wd);
int abs_ctx_sync_update_mt(abs_ctx *ctx, const abs_tensorset *params,
                           const abs_tensorset *momentum, float lr, float mu, float wd);

/* The same with delayed gradient compensation (abs_sync_update_dc). */
int abs_ctx_sync_update_dc(abs_ctx *ctx, float *params, float *params_prev, float *momentum,
                           float lr, float mu, float wd, float lambda);
int abs_ctx_sync_update_dc_mt(abs_ctx *ctx, const abs_tensorset *params,
                              const abs_tensorset *params_prev, const abs_tensorset *momentum,
                              float lr, float mu, float wd, float lambda);

/* Compensation from the momentum (abs_sync_update_dcm).  The context supplies
 * lr_prev: the lr of its last call of this pair that returned ABS_OK, 0 before
 * the first and after one that returned ABS_EMPTY.  Calls of the other update
 * rules on the same context are not tracked. */
int abs_ctx_sync_update_dcm(abs_ctx *ctx, float *params, float *momentum, float lr, float mu,
                            float wd, float lambda);
int abs_ctx_sync_update_dcm_mt(abs_ctx *ctx, const abs_tensorset *params,
                               const abs_tensorset *momentum, float lr, float mu, float wd,
                               float lambda);

/* Adam (abs_sync_update_adam) from the PREVIOUS generation. */
int abs_ctx_sync_update_adam(abs_ctx *ctx, float *params, float *exp_avg, float *exp_avg_sq, float lr,
                             float beta1, float beta2, float eps, float wd, int64_t step);
int abs_ctx_sync_update_adam_mt(abs_ctx *ctx, const abs_tensorset *params,
                                const abs_tensorset *exp_avg, const abs_tensorset *exp_avg_sq,
                                float lr, float beta1, float beta2, float eps, float wd, int64_t step);

/* LARS (abs_sync_update_lars_mt) from the PREVIOUS generation; ragged contexts only. */
int abs_ctx_sync_update_lars_mt(abs_ctx *ctx, const abs_tensorset *params,
                                const abs_tensorset *momentum, const abs_tensorset *gbar, float lr,
                                float mu, float wd, float eta);

/* End of an iteration (Algorithm 1, t = t + 1): stream_upd and every accumulate
 * stream wait for the work the other side has enqueued so far (the next sync-update reads what accumulation
 * wrote; the next accumulation overwrites what the sync-update read), the
 * generations trade places, and the new current counts become 0.  No memory is
 * cleared.  Does not block the host. */
int abs_swap_buffers(abs_ctx *ctx);

/* which: 0 = current generation, 1 = previous.  out: HOST, K int64. */
int abs_ctx_counts(const abs_ctx *ctx, int which, int64_t *out);

#ifdef __cplusplus
}
#endif
#endif /* ABS_SGD_H */
