/*
 * bsgd — the parameter-side step of synchronous SGD with backup workers,
 * for one AMD MI355X (gfx950).
 *
 * What one step computes (paper: "Revisiting Distributed Synchronous SGD",
 * Algorithm 4, and Sec. 3 "backup workers"):
 *
 *   1. N+b workers each send a gradient G_k for the current step.  The
 *      parameter side keeps the first N to arrive and drops the b slowest
 *      (Algorithm 4, collect loop).
 *   2. theta(t+1) = theta(t) - (gamma_t / N) * sum of the kept G_k
 *      (Algorithm 4, update line), i.e. one optimizer update on the mean of
 *      the kept mini-batch gradients (Sec. 1.1 notation: theta, G, gamma_t).
 *      Sec. 3 allows any first-order optimizer in place of plain SGD;
 *      Appendix A.2/A.3 use RMSProp with momentum.
 *   3. Optionally the aggregated gradient is first clipped by its global L2
 *      norm over all layers (Appendix A.3 describes global-norm clipping).
 *   4. Optionally an exponential moving average of theta is kept (Sec. 1.1;
 *      the last line of Algorithm 4).
 *
 * Conventions for every entry point
 *   - Pointers marked DEVICE are HIP device pointers valid on the current
 *     device; pointers marked HOST are ordinary host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls only enqueue work on `stream` and return; they never synchronise
 *     unless stated.  HOST arrays are consumed before the call returns.
 *   - The caller owns every buffer.  The library allocates nothing, frees
 *     nothing and keeps no pointer after a call returns.
 *   - Return value: BSGD_OK, or a negative BSGD_ERR_* for misuse detectable
 *     on the host (nothing is enqueued then).  The one condition only the
 *     device can see — fewer than N workers ever arrive — is reported
 *     through a device status word and leaves theta and state untouched.
 *   - All floating-point data is IEEE fp32, gradients row-major.
 */
#ifndef BSGD_H
#define BSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BSGD_OK            0
#define BSGD_ERR_ARG      (-1)  /* bad argument (host-detected)                     */
#define BSGD_ERR_TOO_FEW  (-2)  /* device status: fewer than N gradients arrive     */
#define BSGD_ERR_HIP      (-3)  /* a HIP runtime call failed                        */
#define BSGD_ERR_SCRATCH  (-4)  /* bsgd_step_noalloc: step too large for the static scratch */

#define BSGD_MAX_WORKERS  256   /* N + b may not exceed this                        */
#define BSGD_MAX_TENSORS  4096  /* T may not exceed this                            */
#define BSGD_STATIC_SCRATCH_BYTES 33554432  /* 32 MiB: scratch of bsgd_step_noalloc  */

/* Which update rule is applied to the aggregated gradient G (Sec. 3:
 * "Sync-Opt"; Sec. 1.1 gives SGD, Appendix A.2/A.3 name RMSProp with
 * momentum and its decay/momentum values).
 *   BSGD_SGD          theta <- theta - lr*G
 *   BSGD_MOMENTUM     v  <- momentum*v + G ;              theta <- theta - lr*v
 *   BSGD_RMSPROP_MOM  ms <- decay*ms + (1-decay)*G*G ;
 *                     m  <- momentum*m + lr*G/sqrt(ms+eps) ; theta <- theta - m   */
typedef enum { BSGD_SGD = 0, BSGD_MOMENTUM = 1, BSGD_RMSPROP_MOM = 2 } bsgd_opt;

/* Hyper-parameters of one step.  HOST; read during the call. */
typedef struct {
  int32_t opt;        /* bsgd_opt                                                   */
  float   lr;         /* gamma_t for THIS step (schedules belong to the caller)     */
  float   momentum;   /* mu   (BSGD_MOMENTUM, BSGD_RMSPROP_MOM)                     */
  float   decay;      /* rho  (BSGD_RMSPROP_MOM)                                    */
  float   eps;        /* epsilon, added inside the square root (BSGD_RMSPROP_MOM)   */
  float   clip_norm;  /* c: G <- G*min(1, c/||G||_2), norm over all tensors;
                         <= 0, NaN or +inf switches clipping off                    */
  float   ema_decay;  /* alpha in [0,1] of the moving average of theta (used when
                         the tensors carry an `ema` buffer)                         */
  float   worker_clip_norm; /* c_w: every kept gradient is first clipped on its own,
                         G_k <- G_k*min(1, c_w/||G_k||_2), norm over all tensors
                         (Appendix A.3 as printed); costs one more pass over the
                         kept rows; <= 0, NaN or +inf switches it off               */
} bsgd_hyper;

/* One parameter tensor.  The struct array itself is HOST memory; the
 * pointers inside are DEVICE pointers, 4-byte aligned, updated in place.
 * Tensors may be listed in any order and may leave gaps in the row, but two
 * tensors may not claim the same gradient columns. */
typedef struct {
  float*  theta;        /* numel parameters                                         */
  float*  s0;           /* v (BSGD_MOMENTUM) or ms (BSGD_RMSPROP_MOM); else NULL     */
  float*  s1;           /* m (BSGD_RMSPROP_MOM); else NULL                          */
  int64_t grad_offset;  /* where this tensor starts inside every gradient row       */
  int64_t numel;        /* >= 0                                                     */
  float*  ema;          /* thetabar, the exponential moving average of theta (Sec.
                           1.1; last line of Algorithm 4), or NULL.  Updated as
                           thetabar <- alpha*thetabar + (1-alpha)*theta(t) from the
                           value of theta BEFORE this step's update.  Either
                           every non-empty tensor has one or none has.            */
} bsgd_tensor;

/* Algorithm 4, collect loop: which N of the N+b gradients are kept.
 *
 *   arrival_t  DEVICE fp32[N+b]: arrival time of worker k's gradient in this
 *              step.  +inf or NaN = never arrives (also stands for a message
 *              carrying a stale step tag, which Algorithm 4 drops).
 *   sel_idx    DEVICE out int32[N]: kept workers, ascending index.
 *   t_step     DEVICE out fp32 (may be NULL): arrival time of the N-th kept
 *              gradient, i.e. how long the step waited.
 *   status     DEVICE out int32: BSGD_OK, or BSGD_ERR_TOO_FEW when fewer than
 *              N arrival times are finite (sel_idx contents are then unspecified).
 *
 * Workers are ordered by (arrival time, worker index): equal times go to the
 * lower index; -0 and +0 are the same instant.  Errors: BSGD_ERR_ARG for
 * N < 1, b < 0, N+b > BSGD_MAX_WORKERS or a NULL required pointer. */
int bsgd_select_first_n(const float* arrival_t, int32_t N, int32_t b,
                        int32_t* sel_idx, float* t_step, int32_t* status, void* stream);

/* Selection with Algorithm 4's tag test spelled out and an optional deadline.
 * HOST struct; `tags` inside is a DEVICE pointer.
 *
 * A message is eligible when its tag equals the current step (Algorithm 4
 * drops a gradient tagged t' != t: the previous step's stragglers), when it
 * arrives no later than `deadline` (Sec. 6 proposes time-outs in place of
 * backup workers), and when its arrival time is neither +inf nor NaN. */
typedef struct {
  const int32_t* tags;  /* DEVICE int32[N+b]: step tag of each message; NULL = all current */
  int32_t step_tag;     /* t, the step being collected                                 */
  float   deadline;     /* tau; +inf = no deadline; NaN is refused                     */
  int32_t n_min;        /* 0: keep the first N eligible messages (fewer than N eligible
                           = BSGD_ERR_TOO_FEW).  >= 1: keep EVERY eligible message,
                           any number from n_min to N+b (fewer than n_min =
                           BSGD_ERR_TOO_FEW); the mean then divides by the number kept */
  const int32_t* row_count; /* DEVICE int32[N+b] or NULL: row k already is the sum of
                           row_count[k] >= 1 worker gradients, added on the machine
                           those workers share before it was sent (Sec. 6; see
                           bsgd_precombine).  N, b and n_min keep counting messages
                           (rows); the mean divides by the number of worker gradients
                           the kept rows hold.  Only bsgd_step_ex takes it
                           (bsgd_select_ex refuses it), and not together with
                           worker_clip_norm.  A kept row with a count < 1 sets the
                           status word to BSGD_ERR_ARG and nothing is updated.      */
} bsgd_select_opts;

/* As bsgd_select_first_n, under `opts`.
 *   sel_idx  DEVICE out int32[N+b] (up to N+b workers can be kept when n_min >= 1)
 *   n_kept   DEVICE out int32: how many were kept (0 on BSGD_ERR_TOO_FEW); may be
 *            NULL only when n_min == 0
 *   t_step   arrival time of the last kept message                              */
int bsgd_select_ex(const float* arrival_t, int32_t N, int32_t b, const bsgd_select_opts* opts,
                   int32_t* sel_idx, int32_t* n_kept, float* t_step, int32_t* status, void* stream);

/* Algorithm 4, update line, for an already chosen set: sum the N kept rows,
 * take the mean, optionally clip, apply one optimizer update to every tensor.
 *
 *   grads     DEVICE fp32[(N+b) x ld], row k = worker k's gradient; only rows
 *             listed in sel_idx are read.  16-byte aligned.  Must not alias
 *             theta/state.
 *   ld        row stride in elements, a multiple of 4, >= every
 *             grad_offset + numel.  Any such stride is correct; a stride that is
 *             an exact power of two around 4 MiB makes the kept rows of a column
 *             collide in the memory system (measured: 2^20 elements, 50 rows:
 *             5.0 TB/s, with ld = 2^20 + 1024: 6.4 TB/s), so pad such rows by
 *             1024 elements.  Strides of 8 MiB and more showed no such effect.
 *   sel_idx   DEVICE int32[N] (as written by bsgd_select_first_n), values in [0, N+b).
 *   status    DEVICE int32 or NULL: when non-NULL and the word is non-zero at
 *             execution time the kernels do nothing.
 *   tensors   HOST array of T descriptors (T = 1 for one flat theta).
 *   workspace DEVICE scratch of at least bsgd_workspace_bytes(...) bytes,
 *             256-byte aligned; contents need not be preserved between calls.
 *
 * Rows are added in ascending worker index in fp32, the sum is multiplied by
 * 1/N once.  Errors: BSGD_ERR_ARG for bad sizes, NULL pointers, a missing
 * state pointer for the chosen optimizer, ld too small, tensors that overlap
 * in the gradient row, or a workspace too small. */
int bsgd_reduce_update(const float* grads, int64_t ld,
                       const int32_t* sel_idx, const int32_t* status, int32_t N,
                       const bsgd_tensor* tensors, int32_t T, const bsgd_hyper* hyper,
                       void* workspace, size_t workspace_bytes, void* stream);

/* One whole step of Algorithm 4: bsgd_select_first_n into the workspace,
 * then bsgd_reduce_update with that selection.  Arguments as above.  When
 * fewer than N gradients arrive, theta and state are left untouched and the
 * workspace status word holds BSGD_ERR_TOO_FEW (see bsgd_last_status). */
int bsgd_step(const float* grads, int64_t ld,
              const float* arrival_t, int32_t N, int32_t b,
              const bsgd_tensor* tensors, int32_t T, const bsgd_hyper* hyper,
              void* workspace, size_t workspace_bytes, void* stream);

/* bsgd_step with the selection taken under `opts` (tags, deadline).  With
 * opts->n_min >= 1 the number of kept gradients is decided on the device and
 * the mean divides by it (see bsgd_last_kept_count). */
int bsgd_step_ex(const float* grads, int64_t ld,
                 const float* arrival_t, int32_t N, int32_t b, const bsgd_select_opts* opts,
                 const bsgd_tensor* tensors, int32_t T, const bsgd_hyper* hyper,
                 void* workspace, size_t workspace_bytes, void* stream);

/* bsgd_step for callers that cannot allocate device memory or carry a
 * workspace around: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * bits in theta and state as bsgd_step, but the step's scratch (kept rows,
 * tensor table, partial sums, the stored mean of a clipped step) lives in a
 * device array of BSGD_STATIC_SCRATCH_BYTES bytes that is part of the library
 * itself; each GPU the library runs on holds its copy until the process ends.
 * The call allocates and frees nothing, on the device or through any library.
 *
 *   status   DEVICE out int32, required: BSGD_OK or BSGD_ERR_TOO_FEW (theta and
 *            state are then untouched), written by the step's first kernel.
 *   t_step   DEVICE out fp32 or NULL: arrival time of the N-th kept gradient.
 *
 * Limit: bsgd_workspace_bytes(span, N, b, T, hyper) must not exceed
 * BSGD_STATIC_SCRATCH_BYTES, else BSGD_ERR_SCRATCH is returned and nothing is
 * enqueued.  Steps without clipping always fit (under 0.4 MiB for 4096
 * tensors); a step clipped by the global norm fits up to about 8.2 M columns,
 * with per-worker clipping up to about 16 M, with both up to about 5.5 M.
 * All calls on one GPU share that GPU's array: two calls whose kernels can
 * overlap in time (different streams without an ordering between them, or
 * different host threads) race on it and must be serialised by the caller.
 * The array's address on the current device is looked up on the first call on
 * that device; make that call outside graph capture.  The bsgd_last_* getters
 * do not apply (there is no workspace pointer to give them). */
int bsgd_step_noalloc(const float* grads, int64_t ld,
                      const float* arrival_t, int32_t N, int32_t b,
                      const bsgd_tensor* tensors, int32_t T, const bsgd_hyper* hyper,
                      int32_t* status, float* t_step, void* stream);

/* Bytes of workspace bsgd_step / bsgd_reduce_update need.  span = the largest
 * grad_offset + numel over the tensors (the total parameter count when the
 * tensors are packed back to back).  Returns 0 for invalid arguments. */
size_t bsgd_workspace_bytes(int64_t span, int32_t N, int32_t b, int32_t T, const bsgd_hyper* hyper);

/* Synchronises `stream`, then copies out what the last bsgd_step on this
 * workspace recorded.  Any out pointer may be NULL.
 *   status_out  HOST int32: BSGD_OK or BSGD_ERR_TOO_FEW
 *   t_step_out  HOST fp32: arrival time of the N-th kept gradient, i.e. how
 *               long the step waited (the quantity Sec. 3.1 records)       */
int bsgd_last_status(const void* workspace, void* stream, int32_t* status_out, float* t_step_out);

/* Synchronises `stream`, then reports how many gradients the last bsgd_step /
 * bsgd_step_ex on this workspace kept (HOST out). */
int bsgd_last_kept_count(const void* workspace, void* stream, int32_t* n_kept_out);

/* Synchronises `stream`, then reports how many worker gradients the rows kept
 * by the last bsgd_step / bsgd_step_ex on this workspace hold: the divisor of
 * the mean (equal to the kept count unless row_count was given).  HOST out. */
int bsgd_last_gradient_count(const void* workspace, void* stream, int32_t* n_gradients_out);

/* Synchronises `stream`, then copies the N kept worker indices of the last
 * bsgd_step on this workspace to HOST int32[N]. */
int bsgd_last_selection(const void* workspace, void* stream, int32_t N, int32_t* sel_idx_out);

/* Synchronises `stream`, then reports the global norm ||G|| (before
 * clipping) and the scale applied by the last clipped step on this
 * workspace.  HOST out pointers, either may be NULL. */
int bsgd_last_clip(const void* workspace, void* stream, double* norm_out, float* scale_out);

/* Sec. 6 of the paper: gradients of workers that share a machine are added
 * on that machine before they are sent, so the parameter side receives one
 * message per machine.  This is that addition, for M machines at once;
 * machine m's workers are the next group_size[m] consecutive rows of `grads`.
 *
 *   grads       DEVICE fp32 [W x ld], W = sum of group_size; 16-byte aligned,
 *               ld a multiple of 4 and >= cols.
 *   cols        columns to combine (the gradient length).
 *   arrival_t   DEVICE fp32 [W]: when each worker finished (+inf/NaN: never).
 *   group_size  HOST int32 [M], every entry >= 1, 1 <= M <= W <= BSGD_MAX_WORKERS.
 *   combined    DEVICE out fp32 [M x ld_out]: row m = sum of machine m's rows,
 *               added in ascending worker index in fp32; same alignment rules;
 *               must not overlap grads.
 *   arrival_m   DEVICE out fp32 [M]: when machine m's message leaves: the
 *               latest of its workers' times (+inf if one never finishes).
 *   row_count   DEVICE out int32 [M]: group_size, for bsgd_select_opts.row_count.
 *
 * Only enqueues on `stream`; allocates nothing.  BSGD_OK, BSGD_ERR_ARG or BSGD_ERR_HIP. */
int bsgd_precombine(const float* grads, int64_t ld, int64_t cols, const float* arrival_t,
                    const int32_t* group_size, int32_t M,
                    float* combined, int64_t ld_out, float* arrival_m, int32_t* row_count, void* stream);

/* ---------------------------------------------------------------------------
 * Straggler analysis (Sec. 3.1 of the paper, "Straggler effects")
 * ------------------------------------------------------------------------- */

/* Time to collect k gradients, for B recorded iterations at once.
 *
 * arrival_t  DEVICE, fp32 [B x W] row-major: row i holds the arrival times of
 *            the W workers' gradients in iteration i (+inf or NaN: never
 *            arrives).  1 <= W <= BSGD_MAX_WORKERS, B >= 1.
 * kth_time   DEVICE out, fp32 [B x W], or NULL: row i = row i of arrival_t in
 *            ascending order, so column k-1 is the time at which the
 *            parameter side held k gradients; never-arriving ones come last
 *            as +inf.
 * mean_kth   DEVICE out, fp64 [W], or NULL: mean over the B iterations of
 *            each column of kth_time (the mean time to collect k gradients),
 *            accumulated in fp64 in a fixed order (deterministic).
 * workspace  DEVICE scratch of bsgd_straggler_workspace_bytes(W, B) bytes,
 *            256-byte aligned; needed only when mean_kth is given.
 *
 * Only enqueues on `stream`.  Returns BSGD_OK or BSGD_ERR_ARG / BSGD_ERR_HIP. */
size_t bsgd_straggler_workspace_bytes(int32_t W, int64_t B);
int bsgd_kth_arrival_times(const float* arrival_t, int32_t W, int64_t B, float* kth_time, double* mean_kth,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Estimated running time to convergence for every split of W machines into
 * N kept workers and W-N backups (Sec. 3.1): iterations(N) x mean time to
 * collect N gradients, where iterations(N) joins the measured points
 * (measured_N[i], measured_iters[i]) by straight lines and is unknown outside
 * their range.  HOST arithmetic on HOST arrays, nothing is enqueued.
 *
 * mean_kth       HOST, fp64 [W], as written by bsgd_kth_arrival_times.
 * measured_N/_iters  HOST, fp64 [n_measured], any order, N values distinct.
 * est            HOST out, fp64 [W]: est[N-1] for N = 1..W, NaN where
 *                iterations(N) is unknown.
 * best_N         HOST out: the N with the smallest finite estimate (the larger
 *                N among equals), 0 if there is none.
 * Returns BSGD_OK or BSGD_ERR_ARG. */
int bsgd_time_to_converge(const double* mean_kth, int32_t W, const double* measured_N, const double* measured_iters,
                          int32_t n_measured, double* est, int32_t* best_N);

/* Human-readable text for a BSGD_* code. */
const char* bsgd_strerror(int code);

/* Library version string, e.g. "bsgd 0.1 (gfx950)". */
const char* bsgd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BSGD_H */
