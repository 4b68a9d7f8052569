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
 *   - No overlap: a buffer a call writes (an accumulator, params, momentum and
 *     the other state vectors) must not share a byte with any other buffer of
 *     the same call.  The flat calls check the ranges and return ABS_EINVAL; the
 *     ragged calls check only that the tensor sets are distinct objects, the
 *     tensors behind them are the caller's to keep apart.
 *   - Return value: ABS_OK (0); ABS_EMPTY (1): nothing to apply, no memory
 *     touched, not an error; ABS_EINVAL (-1): bad argument, nothing enqueued;
 *     ABS_EHIP (-2): a HIP runtime call failed, abs_last_hip_error() has its code.
 *     Nothing is thrown across this boundary.
 *   - Arithmetic is fp32 in one fixed order (stated per call) so results are
 *     reproducible bit for bit; sample counts are integers.
 *   - Threads: calls on different objects (layouts, tensor sets, contexts) and
 *     the stateless calls may run concurrently from several host threads; one
 *     object is used by one thread at a time (a context keeps host counts; a
 *     layout is uploaded by the first tensor set made over it).  The two
 *     process-wide tuning calls (abs_set_launch_tuning, abs_set_cache_policy)
 *     may run at any time: a call in flight works with the settings it read at
 *     its start.  A context can carry settings of its own.
 *   - Devices: everything runs on the HIP device that is current at the call,
 *     on the caller's streams.  A layout keeps its tables on the device that was
 *     current when it was uploaded (abs_layout_upload, or the first
 *     abs_tensorset_create over it); a ragged call with another device current
 *     returns ABS_EINVAL.
 *   - Allocation: only abs_layout_upload / abs_tensorset_create (device tables,
 *     blocking copies) and the abs_*_create calls (host objects, HIP events)
 *     allocate.  No accumulate, sync-update or swap call allocates, frees or
 *     waits for the device.
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
 * later abs_layout_create calls (a layout keeps the tile it was created with);
 * results never change.  Process-wide default; see abs_ctx_set_launch_tuning. */
int abs_set_launch_tuning(int blocks_per_cu, int max_rows_per_tile);

/* Launch length.  Very long launches move fewer bytes per second on this part than the
 * same work in shorter ones, so a call whose kernels would move n times `bytes` is
 * enqueued as n launches over consecutive ranges of its workgroups (one launch when
 * n < 2), on the same stream, in order.  Default 1 GiB; 0 = never cut.  Results never
 * change: every element is still written once, by the same arithmetic.  Process-wide,
 * read once per call; ABS_EINVAL for a negative value. */
int abs_set_launch_slice_bytes(int64_t bytes);
/* Kernel launches the calling thread has enqueued through the library so far (a
 * counter that only grows; the difference around a call is the launches of that call). */
int64_t abs_launch_count(void);
/* The rule itself, for callers that want to know how a call is enqueued: workgroups
 * per launch for a call of `workgroups` workgroups moving `bytes` bytes when
 * `resident_workgroups` of them run at once (every launch but the last is a whole number
 * of such rounds).  Equal to `workgroups` when the call is not cut.  ABS_EINVAL for a
 * negative count or fewer than one resident workgroup. */
int64_t abs_slice_workgroups(int64_t workgroups, int64_t bytes, int resident_workgroups);

/* Cache policy of the kernels.  Accumulators, x and v are re-read soon after a
 * launch (next micro-batch, next iteration).  Each kernel has a cached flavour
 * and a streaming one (non-temporal accesses to those buffers); results are
 * identical.  Mode -1 (default) picks per launch from the buffer sizes: cached
 * while the working set fits the GPU's memory-side cache, streaming beyond.
 * 0 forces cached, 1 forces streaming.  Process-wide default; see
 * abs_ctx_set_cache_policy.  EINVAL for other values. */
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
 *   needed several launches, *count has advanced by the samples of the launches
 *   already enqueued, so count and accumulator still agree. */
int abs_accumulate_batch(float *acc, const void *const *grads, abs_dtype grad_dtype, int J,
                         int64_t P, const int64_t *n_samples, int64_t *count, void *stream);

/* (1'') Job list: Step 2 of SEVERAL workers in one launch -- in Algorithm 1 all N
 *     workers run Step 2 at the same time, each into its own G_t^i.  Job w is one
 *     worker's share: its accumulator, its count and the J_w gradients it has
 *     ready (J_w >= 0; the adaptive batch size makes J_w differ from worker to
 *     worker).  For every job the result equals abs_accumulate_batch on that
 *     job alone, bit for bit.
 *
 *     fold (1..ABS_MAX_BATCH) is the most gradients of one job a launch folds in:
 *     launch r = 0, 1, ... carries, for every job that still has some, its
 *     gradients r*fold .. r*fold + fold - 1, so the call enqueues
 *     ceil(max_w J_w / fold) launches (times ceil(njobs / 16): a launch carries at
 *     most 16 jobs).  fold = 1 keeps the traffic of one abs_accumulate per
 *     gradient (g_b + 8 bytes per parameter and gradient, g_b + 4 for a first one)
 *     with max_w J_w launches instead of sum_w J_w; fold = 8 is the batched traffic
 *     (J*g_b + 8 per job) in one launch.  A launch streams its jobs through the
 *     GPU back to back, with no ramp-up or drain between workers.
 *
 *   jobs   HOST array of njobs (1..ABS_MAX_K) entries; the accumulators must be
 *          distinct buffers and the counts distinct integers
 *   Errors as abs_accumulate_batch, checked for all jobs before anything is
 *   enqueued; if a HIP error stops the call, every count has advanced by what
 *   was enqueued for its job. */
typedef struct abs_job {
    float *acc;               /* DEVICE, P floats */
    const void *const *grads; /* HOST array of J DEVICE pointers, P elements of grad_dtype each */
    const int64_t *n_samples; /* HOST array of J sample counts (each > 0) */
    int J;                    /* gradients ready for this worker; 0 = it sits this call out */
    int64_t *count;           /* HOST, read and advanced as by abs_accumulate */
} abs_job;
int abs_accumulate_jobs(const abs_job *jobs, int njobs, abs_dtype grad_dtype, int64_t P, int fold,
                        void *stream);

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
 * (3') The same with delayed gradient compensation -- Algorithm 1, the
 *     compensation line (third mechanism of Section "Algorithm"):
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
 * (3'm) The same compensation (Algorithm 1, the compensation line)
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
 *               workgroup.  abs_layout_upload copies the chunk table to the
 *               current device and allocates the small per-chunk scratch of the
 *               LARS rule (16 bytes per chunk); the first abs_tensorset_create
 *               over a layout does it if the caller has not.
 * abs_tensorset T DEVICE base pointers for one logical vector (x, v, one
 *               worker's accumulator, one gradient) laid out per the layout;
 *               the pointer table is copied to device memory at creation.
 *               The tensors stay owned by the caller and must outlive the set.
 * ---------------------------------------------------------------------- */
typedef struct abs_layout abs_layout;
typedef struct abs_tensorset abs_tensorset;

/* sizes: HOST array of T element counts (each >= 0; T >= 1). */
int abs_layout_create(abs_layout **out, int T, const int64_t *sizes);
/* Puts the layout's tables on the current device (blocking; allocates).  Idempotent;
 * ABS_EINVAL if the layout already lives on another device. */
int abs_layout_upload(const abs_layout *layout);
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

/* abs_accumulate_jobs over every tensor of the layout: one launch covers all
 * tensors of all jobs.  All gradient sets of a call have one element type. */
typedef struct abs_job_mt {
    const abs_tensorset *acc;           /* an ABS_F32 set */
    const abs_tensorset *const *grads;  /* HOST array of J sets */
    const int64_t *n_samples;           /* HOST array of J sample counts */
    int J;
    int64_t *count;                     /* HOST */
} abs_job_mt;
int abs_accumulate_jobs_mt(abs_layout *layout, const abs_job_mt *jobs, int njobs, int fold,
                           void *stream);

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
 *   layout (allocated by abs_layout_upload): two LARS calls on one layout must
 *   not overlap in time.  A flat vector is a layout of one tensor.
 *   Other arguments, ABS_EMPTY and errors: as abs_sync_update_mt. */
int abs_sync_update_lars_mt(abs_layout *layout, const abs_tensorset *params,
                            const abs_tensorset *momentum, const abs_tensorset *gbar,
                            const abs_tensorset *const *acc, const int64_t *counts, int K, float lr,
                            float mu, float wd, float eta, void *stream);

/* For callers that cannot allocate -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: abs_sync_update_lars_mt with its scratch
 * (per-chunk sums of squares, per-tensor step factors, the first-chunk table, which
 * the kernels rebuild from the chunk table) in a fixed device array inside the
 * library instead of memory owned by the layout.  The array is about 1.03 MiB; every
 * GPU the library runs on holds its own copy until the process ends.  The call never
 * allocates or frees, on the host side of the runtime or through it, and does not
 * wait for the device.  The array's address on a device is looked up once, when a
 * layout's tables go to that device (abs_layout_upload, or the first tensor set over
 * a layout), so the call itself asks the runtime for nothing but launches and may be
 * recorded into a HIP graph; a recorded call replays with the sample counts it was
 * recorded with.
 *
 *   Limits: abs_layout_num_chunks(layout) <= ABS_NOALLOC_MAX_CHUNKS and
 *   abs_layout_num_tensors(layout) <= ABS_NOALLOC_MAX_TENSORS, else ABS_EINVAL with
 *   nothing enqueued.  The layout must already be on the device (it is once a tensor
 *   set exists over it); ABS_EINVAL otherwise.
 *   All calls on one GPU, whatever their layout or context, share the one array,
 *   which keeps the last call's contents: calls that overlap in time on one GPU
 *   race; order them on one stream or with events.  Nothing in it needs clearing:
 *   a call writes every entry before it reads it.
 *   Arguments, arithmetic, results (bit for bit), ABS_EMPTY and the other errors:
 *   as abs_sync_update_lars_mt. */
#define ABS_NOALLOC_MAX_CHUNKS 65536
#define ABS_NOALLOC_MAX_TENSORS 4096
int abs_sync_update_lars_mt_noalloc(abs_layout *layout, const abs_tensorset *params,
                                    const abs_tensorset *momentum, const abs_tensorset *gbar,
                                    const abs_tensorset *const *acc, const int64_t *counts, int K,
                                    float lr, float mu, float wd, float eta, void *stream);

/* ------------------------------------------------------------------------
 * (4) Double buffer -- Algorithm 1, the line that runs Step 1 and Step 2 side
 *     by side: two generations of (K accumulators, K counts).  Accumulation of batch t runs
 *     on stream_acc into the CURRENT generation while the sync-update of batch
 *     t-1 runs on stream_upd from the PREVIOUS one.
 *
 * The context owns only indices, the 2*K host counts and two HIP events; the
 * accumulators stay the caller's.  All counts start at 0 (G_{-1} = 0).
 * stream_acc == stream_upd gives the serial order on one stream.
 * ---------------------------------------------------------------------- */
typedef struct abs_ctx abs_ctx;

/* acc_A, acc_B: HOST arrays of K DEVICE pointers, P floats each; the 2K buffers
 * must not overlap one another. */
int abs_ctx_create(abs_ctx **out, int K, int64_t P, float *const *acc_A, float *const *acc_B,
                   void *stream_acc, void *stream_upd);
/* Ragged form: acc_A, acc_B are HOST arrays of K ABS_F32 sets over `layout`. */
int abs_ctx_create_mt(abs_ctx **out, int K, abs_layout *layout,
                      const abs_tensorset *const *acc_A, const abs_tensorset *const *acc_B,
                      void *stream_acc, void *stream_upd);
int abs_ctx_destroy(abs_ctx *ctx);

/* Settings of this context's own calls, in place of the process-wide defaults
 * (abs_set_launch_tuning, abs_set_cache_policy; same arguments and errors).  A
 * ragged context's tile is its layout's; only the cache policy applies to it. */
int abs_ctx_set_launch_tuning(abs_ctx *ctx, int blocks_per_cu, int max_rows_per_tile);
int abs_ctx_set_cache_policy(abs_ctx *ctx, int accumulate_mode, int update_mode);

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

/* Step 2 of ALL K workers of an iteration in one call (abs_accumulate_jobs into
 * the CURRENT generation): worker k contributes m[k] >= 0 gradients.  grads and
 * n_samples list them worker by worker (worker 0's m[0] entries, then worker 1's,
 * ...; sum_k m[k] entries each).  With fold = 8 an iteration is this call, one
 * sync-update and the swap: two launches.  Runs on stream_acc; contexts that
 * spread accumulation over several streams return ABS_EINVAL. */
int abs_ctx_accumulate_step(abs_ctx *ctx, const void *const *grads, const int *m,
                            const int64_t *n_samples, abs_dtype grad_dtype, int fold);
int abs_ctx_accumulate_step_mt(abs_ctx *ctx, const abs_tensorset *const *grads, const int *m,
                               const int64_t *n_samples, int fold);

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
