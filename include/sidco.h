/*
 * sidco.h - C ABI of the MI355X (gfx950) implementation of the SIDCo gradient
 * sparsifier (arXiv 2101.10761, "An Efficient Statistical-based Gradient
 * Compression Technique for Distributed Training Systems").
 *
 * What one call computes, on one worker's flat fp32 gradient g of d elements:
 *   1. error compensation  acc = g + residual           (App. B.2, memory-based compression)
 *   2. stage-1 fit of a sparsity-inducing distribution to |acc| from the sums
 *      sum|x|, sum x^2, sum log|x|                        (Corollary 1 / eq. (6); Corollaries 1.2, 1.3)
 *   3. threshold eta_1 in closed form, refined over M peak-over-threshold
 *      stages on the exceedances                          (Sec. 2.4: Lemma 2 / eqs. (7)-(9),
 *                                                          Corollary 2 / eqs. (10)-(11))
 *   4. C_eta: the pairs (j, acc_j) with |acc_j| > eta_M, their number, and the
 *      residual update residual_j = 0 for selected j      (Sec. 2.3; Algorithm 1, Sparsify)
 *
 * All pointers named "device" are HIP device pointers on the current device;
 * "host" pointers are ordinary host memory.  No torch types cross this boundary.
 * Every enqueueing call is asynchronous on `stream` and returns after enqueue;
 * outputs are valid once the stream reaches that point.  The library never
 * spins on the device, and an enqueueing call synchronises with the host in
 * one case only: when the stream's workspace has to grow (first use, or a
 * longer vector than before), it is freed and allocated again, which waits for
 * the device.  sidco_reserve moves that out of the enqueueing calls, and
 * sidco_compress_static never allocates at all.  (sidco_controller_compress also
 * reads one counter back on every Q-th call; that is its contract.)
 *
 * Results are deterministic for a given history of calls on a workspace: the
 * same inputs after the same previous calls give the same bits.  Across
 * different histories the exceedance statistics of the stages after the first
 * are summed in a different order (the candidate lists follow the previous
 * call's thresholds, see sidco_set_speculation), so a threshold can differ in
 * its last bit, far inside the 1e-5 the fitted values are specified to; given
 * the threshold, the selected set, its values and the residual are exact.  The
 * order of the output pairs is fixed for a single-stage call and may vary
 * between runs for M >= 2.
 *
 * Return value: 0 on success, a negative SIDCO_ERR_* otherwise.  Argument
 * errors are detected on the host before any HIP call is made.  Conditions
 * that depend on the data (NaN/Inf input, degenerate fits, output overflow)
 * never cause out-of-bounds accesses; they are reported in sidco_diag.status.
 *
 * Workspaces.  The library keeps one workspace per (device, stream), so calls
 * on different streams do not share state and may overlap; calls on one stream
 * are ordered by the stream.  A caller-provided workspace (sidco_set_workspace)
 * replaces them all on its device: calls that use it must not overlap.  The
 * diagnostics calls that take a stream (sidco_read_diag, sidco_fit_result, ...)
 * report the last call made on that stream.
 */
#ifndef SIDCO_H
#define SIDCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SIDCO_MAX_STAGES 8

/* `dist`: the first-stage law and with it the chain of later stages
 * (Sec. 2.4, last paragraph; naming as in App. E/F).                          */
#define SIDCO_DIST_EXP        0 /* SIDCo-E : exponential, then exponential PoT stages   */
#define SIDCO_DIST_GAMMA_GPD  1 /* SIDCo-GP: gamma first stage, then GPD PoT stages     */
#define SIDCO_DIST_GPD        2 /* SIDCo-P : generalized Pareto in every stage          */

/* error codes */
#define SIDCO_OK              0
#define SIDCO_ERR_NULL       -1 /* a required pointer is NULL                           */
#define SIDCO_ERR_SIZE       -2 /* d < 1 or d > 2^31-1, or a capacity < 1               */
#define SIDCO_ERR_DELTA      -3 /* a ratio is not in (0,1)                              */
#define SIDCO_ERR_STAGES     -4 /* stages < 1 or > SIDCO_MAX_STAGES                     */
#define SIDCO_ERR_DIST       -5 /* unknown dist                                         */
#define SIDCO_ERR_WORKSPACE  -6 /* caller-provided workspace too small or misaligned    */
#define SIDCO_ERR_HIP        -7 /* a HIP runtime call failed (see sidco_last_hip_error) */
#define SIDCO_ERR_ALIGN      -8 /* a float/int32 pointer is not 4-byte aligned          */
#define SIDCO_ERR_ARG        -9 /* any other invalid argument                           */

/* status bits of sidco_diag.status (data-dependent conditions) */
#define SIDCO_ST_NONFINITE    (1u << 0) /* a stage-1 sum was NaN/Inf: eta = NaN, nothing selected     */
#define SIDCO_ST_VAR_ZERO     (1u << 1) /* a GPD fit saw variance <= 0: increment = mean             */
#define SIDCO_ST_GAMMA_S      (1u << 2) /* gamma fit had s <= 0: threshold 0                          */
#define SIDCO_ST_GAMMA_CLAMP  (1u << 3) /* gamma closed form negative, clamped to 0                    */
#define SIDCO_ST_STOPPED      (1u << 4) /* an exceedance set was empty: later stages keep eta         */
#define SIDCO_ST_OVERFLOW     (1u << 5) /* more pairs selected than the output capacity; the excess
                                           stays in the residual and is not reported                  */
#define SIDCO_ST_FALLBACK     (1u << 6) /* performance only: a stage found the candidate lists of the
                                           stage before it too short for its threshold and read the
                                           dense vector again (see sidco_set_speculation); the result
                                           is the same either way                                     */

/* Per-call diagnostics, filled on the device by the kernels of the last call. */
typedef struct sidco_diag {
    float    eta[SIDCO_MAX_STAGES];      /* eta_m, fp32, m = 1..M (Lemma 2: absolute thresholds)      */
    int64_t  n[SIDCO_MAX_STAGES];        /* number of elements the stage-m fit ran over (n[0] = d)    */
    double   stats[SIDCO_MAX_STAGES][3]; /* stage 1: mean|x|, variance (GPD only), mean log|x| (gamma
                                            only); stage m>=2: mean and variance of |x|-eta_{m-1}
                                            (variance for GPD chains only); unused entries are 0      */
    int64_t  selected;                   /* |{j : |acc_j| > eta_M}| before capacity clipping          */
    int32_t  count;                      /* pairs written = min(selected, capacity)                   */
    int32_t  stages;                     /* M of the call                                             */
    uint32_t status;                     /* OR of SIDCO_ST_*                                          */
    uint32_t reserved;
} sidco_diag;

/*
 * The sparsifier (Algorithm 1, function Sparsify, with error compensation).
 *
 *  stream     hipStream_t as void*; NULL = the default stream
 *  grad       device, d floats, read only
 *  residual   device, d floats, in/out, or NULL.  On entry the error carried
 *             from the previous iteration; on exit acc = grad + residual with
 *             zeros at the selected positions (so the next call's step 1 is
 *             App. B.2's update).  NULL = memoryless variant: acc = grad and
 *             nothing but out_* is written.  Must not alias grad.
 *  d          1 <= d <= 2^31-1
 *  delta      target ratio k/d, 0 < delta < 1 (Sec. 2.3)
 *  dist       SIDCO_DIST_*
 *  stages     M, 1..SIDCO_MAX_STAGES.  The ratios are delta_1 = 0.25 (the
 *             paper's setting, Sec. 4.1; see sidco_set_delta1) and delta_m = (delta/delta_1)^(1/(M-1))
 *             for m >= 2, so that their product is delta (Sec. 2.4); if
 *             delta_1 <= delta or M = 1 a single stage at delta is used.
 *  out_idx    device, int32, capacity sidco_out_capacity(d, delta)
 *  out_val    device, float, same capacity: out_val[i] = acc[out_idx[i]]
 *  out_count  device, 1 int32: number of pairs written (khat)
 *  out_eta    device, 1 float: eta_M
 * The pairs are not sorted by index.  Buffers are owned by the caller; the library owns only
 * its workspaces, which it allocates on first use per stream (hipMalloc) and
 * grows when d grows, unless sidco_set_workspace was called.
 * Explicit stage ratios are an argument of sidco_compress_ex rather than state
 * set by a separate call (sidco_set_delta1 exists for callers that must stay on
 * this signature); the diagnostics of a call are read with sidco_read_diag
 * (sidco_get_diag is exported as another name of the same function).
 */
int sidco_compress(void *stream, const float *grad, float *residual, int64_t d,
                   double delta, int dist, int stages,
                   int32_t *out_idx, float *out_val, int32_t *out_count, float *out_eta);

/*
 * sidco_compress for callers that cannot allocate device memory or must not
 * trigger an allocation: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results, same kernels;
 * the workspace is a fixed array inside the library's device code (about 34 MB,
 * resident in every GPU the library is loaded on until the process ends), so the
 * call makes no hipMalloc / hipFree and nothing that allocates, on any call,
 * the first included.  Limits: d <= sidco_static_max_elements() = 2,097,152
 * (SIDCO_ERR_SIZE beyond it, with the limit in sidco_last_hip_error), fp32
 * gradients, the default stage schedule, no per-kernel profiling.  All calls
 * on a GPU share that GPU's one array, on whatever stream: calls that overlap
 * in time race and must be serialised by the caller.  The array keeps what the
 * previous call left; the first kernel of every call resets the per-call
 * counters, and the lists are always written before they are read, so nothing
 * carries over except the threshold hints of a repeated shape (performance only).
 * sidco_read_diag does not cover these calls.
 * sidco_static_init looks the array's address up on the current device (the HIP
 * runtime maps the array into the device on that first access); the first
 * sidco_compress_static on a device does the same if it has not been called, so
 * a caller that captures or forbids allocation from the start calls it once
 * per device beforehand.
 */
int sidco_compress_static(void *stream, const float *grad, float *residual, int64_t d,
                          double delta, int dist, int stages,
                          int32_t *out_idx, float *out_val, int32_t *out_count, float *out_eta);
int64_t sidco_static_max_elements(void);
int sidco_static_init(void);

/*
 * Same computation with explicit stage ratios delta_1..delta_M (host array,
 * each in (0,1); the target ratio is their product, Sec. 2.4) and an explicit
 * capacity of out_idx / out_val in elements.
 */
int sidco_compress_ex(void *stream, const float *grad, float *residual, int64_t d,
                      int dist, const double *ratios, int n_ratios,
                      int32_t *out_idx, float *out_val, int64_t out_capacity,
                      int32_t *out_count, float *out_eta);

/*
 * The sparsifier on a gradient stored in 16 bits (fp16 or bf16, the types
 * mixed-precision training produces).  The gradient is widened to fp32 as it is
 * read - exactly - and everything else is sidco_compress: acc = fp32(grad) +
 * residual in fp32, fits in fp64, fp32 thresholds, fp32 residual and values.
 *
 *  grad        device, d elements of grad_dtype, read only, aligned to its
 *              element size (8-byte alignment enables the vector path)
 *  grad_dtype  SIDCO_GRAD_F32 (then this is sidco_compress), _F16 or _BF16
 *  residual    device, d floats, in/out, or NULL.  Without a residual the
 *              widened vector is kept in the workspace, which then needs
 *              sidco_workspace_bytes_typed(d, grad_dtype, 0) bytes.
 * Everything else as in sidco_compress.
 */
#define SIDCO_GRAD_F32  0
#define SIDCO_GRAD_F16  1
#define SIDCO_GRAD_BF16 2
int sidco_compress_typed(void *stream, const void *grad, int grad_dtype, float *residual, int64_t d,
                         double delta, int dist, int stages,
                         int32_t *out_idx, float *out_val, int32_t *out_count, float *out_eta);
size_t sidco_workspace_bytes_typed(int64_t d, int grad_dtype, int has_residual);

/* The other calls on a gradient of element type grad_dtype (SIDCO_GRAD_*): the
 * batched call, the stage controller, and the two comparators.  Everything but
 * the gradient's element type is as in the call of the same name without
 * "_typed"; the residual, all arithmetic and the outputs stay fp32 / fp64.
 * Without a residual a 16-bit gradient's widened copy lives in the workspace
 * (sidco_workspace_bytes_typed / sidco_workspace_bytes_batched_typed); the DGC
 * comparator needs none.                                                      */
int sidco_compress_batched_typed(void *stream, const void *grad, int grad_dtype, float *residual,
                                 const int64_t *offsets, int n, double delta, int dist, int stages,
                                 int32_t *out_idx, float *out_val, const int64_t *out_offsets,
                                 int32_t *out_counts, float *out_etas);
size_t sidco_workspace_bytes_batched_typed(const int64_t *offsets, int n, int grad_dtype, int has_residual);
struct sidco_controller;
int sidco_controller_compress_typed(struct sidco_controller *c, void *stream, const void *grad, int grad_dtype,
                                    float *residual, int64_t d, int32_t *out_idx, float *out_val,
                                    int32_t *out_count, float *out_eta);
int sidco_topk_typed(void *stream, const void *grad, int grad_dtype, float *residual, int64_t d, int64_t k,
                     int32_t *out_idx, float *out_val, int32_t *out_count, float *out_kth);
int sidco_dgc_typed(void *stream, const void *grad, int grad_dtype, float *residual, int64_t d, double delta,
                    double sample_ratio, uint64_t seed,
                    int32_t *out_idx, float *out_val, int32_t *out_count, float *out_eta);

/*
 * Several vectors in one launch sequence: the tensors of one flat gradient
 * buffer, each sparsified on its own exactly as sidco_compress would (the cost of
 * the compressor depends only on the vector's size, App. A, so layer-wise
 * compression is n independent problems; here they share every kernel launch).
 *
 *  grad, residual  device, flat buffers; tensor t is the elements
 *                  [offsets[t], offsets[t+1]) of both (residual may be NULL)
 *  offsets         host, n+1 ascending int64; every tensor has 1..2^31-1 elements
 *  n               1..512 tensors per call
 *  delta, dist, stages   as in sidco_compress, the same for every tensor
 *  out_idx, out_val      device; tensor t's pairs start at out_offsets[t] and have room
 *                  for out_offsets[t+1] - out_offsets[t] >= 1 pairs; indices are
 *                  relative to the tensor's first element
 *  out_offsets     host, n+1 int64 (sidco_batched_out_offsets fills the default:
 *                  sidco_out_capacity per tensor)
 *  out_counts, out_etas  device, n int32 / n floats
 * A call with a layout other than the previous call's uploads a table of a few
 * kilobytes in stream order; nothing waits for the device.
 */
int sidco_compress_batched(void *stream, const float *grad, float *residual, const int64_t *offsets,
                           int n, double delta, int dist, int stages,
                           int32_t *out_idx, float *out_val, const int64_t *out_offsets,
                           int32_t *out_counts, float *out_etas);
int sidco_batched_out_offsets(const int64_t *offsets, int n, double delta, int64_t *out_offsets);
size_t sidco_workspace_bytes_batched(const int64_t *offsets, int n);
/* Diagnostics of tensor t of the last batched call on `stream`.  Synchronises `stream`. */
int sidco_read_diag_batched(void *stream, int t, sidco_diag *host_out);

/*
 * Adapt_Stages (Algorithm 1; Sec. 3): the number of stages for the next Q
 * iterations from the average number of selected elements over the last Q.
 * One stage fewer if khat_avg > k (1 + eps_high), one more if
 * khat_avg < k (1 - eps_low), clamped to [1, max_stages].  Pure host function.
 * Returns the new number of stages, or a negative error code.
 */
int sidco_adapt_stages(int stages, double khat_avg, double k, double eps_high, double eps_low,
                       int max_stages);

/*
 * The sparsifier with its stage controller (Algorithm 1 as a whole): one
 * controller per gradient vector, one sidco_controller_compress per training
 * iteration.  Each call is sidco_compress with the controller's current number
 * of stages (ratios as described there, with the controller's delta_1); the
 * device keeps the running count of reported pairs, and every Q-th call
 * synchronises `stream` once, reads the count back and applies
 * sidco_adapt_stages with k = delta * d.  All Q counts of a window enter the
 * average (the pseudo-code drops the count of the adapting iteration yet divides
 * by Q; Sec. 3 describes an average over the past Q steps).  The paper's
 * settings are delta_1 = 0.25, eps_high = eps_low = 0.2, Q = 5 (Sec. 4.1).
 * A controller belongs to one stream.  Its running count lives in that
 * stream's workspace: if any other call of this library uses the same
 * workspace inside a window of Q calls, the window's count is not this
 * vector's alone; the controller then leaves the number of stages as it is
 * and counts the window in sidco_controller_disturbed.
 */
typedef struct sidco_controller sidco_controller;
int sidco_controller_create(sidco_controller **out, double delta, int dist, int stages,
                            int max_stages, int Q, double eps_high, double eps_low, double delta1);
void sidco_controller_destroy(sidco_controller *c);
int sidco_controller_stages(const sidco_controller *c);             /* current M               */
int64_t sidco_controller_iteration(const sidco_controller *c);      /* calls made so far       */
double sidco_controller_last_average(const sidco_controller *c);    /* khat average at the last
                                                                       adaptation, -1 before it */
int64_t sidco_controller_disturbed(const sidco_controller *c);      /* windows skipped because another
                                                                       caller used the workspace   */
int sidco_controller_compress(sidco_controller *c, void *stream, const float *grad, float *residual,
                              int64_t d, int32_t *out_idx, float *out_val, int32_t *out_count,
                              float *out_eta);

/*
 * Decompression / aggregation, the step that follows the sparsifier in the
 * distributed algorithm (Algorithm 2: the workers' sparsified gradients are
 * averaged): dense[idx[i]] += scale * val[i] for i < min(*count, capacity).
 *
 *  dense     device, d floats, in/out (the caller zeroes it before the first list)
 *  idx, val  device, one worker's output pairs as sidco_compress wrote them
 *            (indices distinct within one list)
 *  count     device, 1 int32: the list's length (so no host read-back is needed)
 *  capacity  elements idx / val have room for
 *  scale     e.g. 1/N for the average over N workers
 * One list per call; lists of several workers are added by consecutive calls on
 * the stream, so the sum is formed in a fixed order.  An index outside [0, d)
 * is skipped and remembered; sidco_scatter_check (synchronises `stream`)
 * returns 1 if that happened since the last check, else 0.
 */
int sidco_scatter_add(void *stream, float *dense, int64_t d, const int32_t *idx, const float *val,
                      const int32_t *count, int64_t capacity, float scale);
int sidco_scatter_check(void *stream);

/*
 * Exact Top-k by magnitude, the operator the paper compares its threshold
 * estimators with (Sec. 1: Top-k keeps the k entries of largest magnitude; a GPU
 * finds them with a radix select; footnote of Sec. 2.3: C_eta equals Top-k at
 * k = khat).  Same buffers and error-compensation semantics as sidco_compress:
 * acc = grad + residual is formed and stored back into residual (App. B.2), the
 * k entries of largest |acc| are written as (index, value) pairs, and residual
 * is zeroed at their positions.
 *
 *  k          1 <= k <= d
 *  out_idx, out_val  device, capacity k
 *  out_count  device, 1 int32: k
 *  out_kth    device, 1 float: the k-th largest magnitude
 * A NaN counts as larger than every number (its bit pattern is).  The k-th
 * largest magnitude, the selected entries above it and all values are
 * deterministic; which of the entries EQUAL to the k-th largest magnitude
 * complete the set may differ between runs.  The pairs are not sorted.
 */
int sidco_topk(void *stream, const float *grad, float *residual, int64_t d, int64_t k,
               int32_t *out_idx, float *out_val, int32_t *out_count, float *out_kth);

/*
 * DGC's sampling threshold, one of the threshold methods the paper compares
 * with (Sec. 1, related work and its footnote): a random subset of the
 * gradient is drawn, Top-k of the subset at the target ratio gives a
 * threshold, the threshold selects from the whole vector, and a second Top-k
 * trims the selection when it exceeds the target.  Same buffers and
 * error-compensation semantics as sidco_compress.
 *
 *  delta         target ratio, 0 < delta < 1; k = ceil(delta * d)
 *  sample_ratio  size of the subset relative to d, 0 < sample_ratio <= 1
 *                (DGC's example is 0.01): n_s = ceil(sample_ratio * d) draws
 *                with replacement; draw j is element floor(u_j * d / 2^32),
 *                u_j = upper 32 bits of output j of the splitmix64 sequence
 *                started at `seed`
 *  out_idx, out_val  device, capacity k
 *  out_count     device, 1 int32: entries written, min(k, first-pass count)
 *  out_eta       device, 1 float: the subset's threshold, i.e. its k_s-th
 *                largest magnitude, k_s = ceil(delta * n_s)
 * The first pass keeps |acc| > threshold (strict, fp32).  If that is more than
 * k entries, the k of largest magnitude stay (which of the entries tied with the
 * smallest one stay may differ between runs); otherwise all of them stay.
 * sidco_dgc_sizes fills sizes[0..2] = n_s, k_s, k (host only).
 * sidco_dgc_result fills host_out[0..3] = n_s, k_s, first-pass count and
 * entries written of the last sidco_dgc on `stream`; it synchronises `stream`.
 */
int sidco_dgc(void *stream, const float *grad, float *residual, int64_t d, double delta,
              double sample_ratio, uint64_t seed,
              int32_t *out_idx, float *out_val, int32_t *out_count, float *out_eta);
int sidco_dgc_sizes(int64_t d, double delta, double sample_ratio, int64_t *sizes);
int sidco_dgc_result(void *stream, int64_t *host_out);

/*
 * Steps 1-2 alone: the error-compensation add (App. B.2; skipped when residual
 * is NULL) fused with the sums of the stage-1 fit (Corollary 1 / eq. (6),
 * Corollaries 1.2 and 1.3).  This is the kernel that dominates a call; it is
 * exported so that it can be timed and checked on its own.  On return of the
 * stream, residual holds acc = grad + residual.  The sums stay in the
 * workspace until the next call on the device.
 */
int sidco_fit(void *stream, const float *grad, float *residual, int64_t d, int dist);
/* The same on a gradient of element type grad_dtype (SIDCO_GRAD_*), as in sidco_compress_typed. */
int sidco_fit_typed(void *stream, const void *grad, int grad_dtype, float *residual, int64_t d, int dist);

/* Sums of the last sidco_fit on `stream`, reduced on the host in a
 * fixed order.  host_sums (host, 4 doubles) receives sum|acc|, sum acc^2
 * (GPD law only, else 0), sum log max(|acc|, 2^-126) (gamma law only, else 0)
 * and d.  Synchronises `stream`.                                              */
int sidco_fit_result(void *stream, double *host_sums);

/* Host helper: the default split of delta over `stages` stages described at
 * sidco_compress, for a given delta_1.  Writes the ratios to `ratios` (host,
 * room for SIDCO_MAX_STAGES doubles) and returns their number (>= 1), or a
 * negative error code.                                                        */
int sidco_stage_ratios(double delta, int stages, double delta1, double *ratios);

/* Host helper: capacity sidco_compress assumes for out_idx / out_val:
 * min(d, 4*ceil(delta*d) + 4096).  The paper reports khat/k ~ 1 on average
 * and at most ~2 for the gamma-GPD chain (App. E); a worse overshoot sets
 * SIDCO_ST_OVERFLOW and the excess stays in the residual.  Returns a negative
 * error code for invalid arguments.                                           */
int64_t sidco_out_capacity(int64_t d, double delta);

/* delta_1 of the default stage schedule used by sidco_compress,
 * sidco_compress_static, sidco_compress_typed and sidco_compress_batched, for the
 * calls that follow on every device: 0 < delta1 < 1, initially 0.25 (Sec. 4.1).
 * Explicit ratios per call: sidco_compress_ex.                                */
int sidco_set_delta1(double delta1);

/* Host helper: bytes of device workspace a call with this d needs.  It depends
 * on d alone (room for one list slot per element in two buffers, whatever
 * delta and the number of stages are); the 16-bit and batched variants have
 * their own helpers.                                                          */
size_t sidco_workspace_bytes(int64_t d);

/* Give the library a caller-owned device workspace (256-byte aligned) for the
 * current device instead of letting it allocate; NULL/0 returns to library
 * allocation.  The buffer must outlive every call that uses it; it serves the
 * calls of every stream, which therefore must not overlap.                    */
int sidco_set_workspace(void *device_ptr, size_t bytes);

/* Make sure that the library's own workspace of `stream` on the current device
 * has at least `bytes` (see the sidco_workspace_bytes helpers), so that the
 * enqueueing calls that follow on that stream neither allocate nor wait for
 * the device.  This call itself may do both.  sidco_release frees the
 * workspace of `stream` (it waits for work that still uses it).              */
int sidco_reserve(void *stream, size_t bytes);
int sidco_release(void *stream);

/* Status bits without a host round trip: the sparsifier calls that follow on
 * `stream` (single-vector calls; not the batched one) also OR the call's
 * SIDCO_ST_* bits, SIDCO_ST_OVERFLOW included, into *device_word (device, one
 * uint32, cleared at the start of each call), so that a consumer on the device,
 * or a copy the caller already makes, sees them next to out_count.  NULL
 * switches it off.                                                            */
int sidco_set_status_word(void *stream, uint32_t *device_word);

/*
 * Tuning knob, no effect on results.  A stage m < M that reads the dense vector
 * (Sec. 2.4: every stage after the first only needs the exceedances of the stage
 * before it) hands the next stage a list of candidates instead of all its
 * exceedances: the entries above the quantile of stage m's fitted law at
 * log(1/ratio) = log(1/delta_m) + theta * log(1/delta_{m+1}).  The next stage
 * uses the list if its own threshold, computed from the exact statistics of all
 * exceedances, is at or above the candidate threshold, and reads the dense
 * vector again otherwise (SIDCO_ST_FALLBACK).  theta in [0, 1]; 0 = the list
 * holds all exceedances of eta_m and is always usable; default 0.5.  Applies
 * to the calls that follow, on every device.
 */
int sidco_set_speculation(double theta);

/* Copy the diagnostics of the last call on `stream` (current device) to host
 * memory.  Synchronises `stream`.  sidco_get_diag is the same function.       */
int sidco_read_diag(void *stream, sidco_diag *host_out);
int sidco_get_diag(void *stream, sidco_diag *host_out);

/* Per-kernel timing of the calls that follow (HIP events recorded on the
 * call's stream around every kernel).  sidco_get_profile synchronises on the
 * last event and returns the number of kernels of the last call, writing up to
 * `cap` durations in milliseconds to `ms` and, if names != NULL, pointers to
 * static kernel-name strings.                                                 */
int sidco_set_profiling(int enable);
int sidco_get_profile(float *ms, const char **names, int cap);

/* Text for an error code; the HIP error string of the last SIDCO_ERR_HIP.     */
const char *sidco_strerror(int code);
const char *sidco_last_hip_error(void);

/* Library version (major*100 + minor).                                        */
int sidco_version(void);

/* Free the library-owned workspaces and events of every device.               */
void sidco_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* SIDCO_H */
