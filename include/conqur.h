/*
 * conqur.h -- C ABI of the MI355X (gfx950) hot path of ConQuR's online rotation
 * calibration: rotate -> row-normalise -> hypercube-corner assign -> accumulate
 * the cross-covariance -> closed-form orthogonal Procrustes (polar) update, plus
 * the per-token symmetric fake-quantisation error of the rotated activations.
 *
 * Conventions (all matrices row-major, activations are rows, App. A "X_hat = X R"):
 *   y_i  = x_i R                      the rotation maps row vectors; it is the
 *                                     transpose of the R of Sec. 3 (which writes R x)
 *   M    = sum_i (x_i/||x_i||)^T c_i  c_i = sgn(y_i)/sqrt(dh), sgn(0) = +1 (Eq. 2);
 *                                     the transpose of Sec. 3.3's C = Z^T X~
 *   R    <- polar(M) = U V^T          Sec. 3.3, for M = U S V^T
 * With heads = h > 1 the row of width d is h independent blocks of width dh = d/h,
 * each with its own rotation, statistics and update (App. A: the block-diagonal
 * per-head rotation; Sec. 3.4 "a Procrustes problem per head").
 *
 * Pointers are tagged HOST or DEVICE below.  Every call returns a conqur_status;
 * nothing throws across the boundary.  Calls enqueue their kernels on the stream
 * given at init and return without waiting unless a HOST output is requested.
 * A context is not thread safe.  The library never falls back to the CPU: every
 * step below runs in HIP kernels, and a call fails with CONQUR_EHIP if the device
 * or a launch fails.
 */
#ifndef CONQUR_H
#define CONQUR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct conqur_ctx conqur_ctx; /* opaque; owns R, the rotate operand, M and all workspaces (device) */

typedef enum {
  CONQUR_OK = 0,
  CONQUR_EINVAL = 1,    /* bad argument, shape, stride or alignment; nothing was enqueued        */
  CONQUR_ESTATE = 2,    /* call not valid in this state (update with no accumulated row)         */
  CONQUR_ENOMEM = 3,    /* device or host allocation failed                                      */
  CONQUR_EHIP = 4,      /* a HIP call failed; conqur_last_error() holds the HIP error string      */
  CONQUR_ENOCONV = 5,   /* polar iteration hit polar_max_iters; R holds the last iterate and the
                           reported orthogonality error says how far it is from orthogonal        */
  CONQUR_ENONFINITE = 6 /* (reported by update) rows with NaN/Inf were met and skipped           */
} conqur_status;

typedef enum { CONQUR_F32 = 0, CONQUR_BF16 = 1 } conqur_dtype;

typedef struct {
  uint32_t d;               /* row width of X; d % heads == 0, (d/heads) % 16 == 0, d/heads <= 8192 */
  uint32_t heads;           /* 1 = one d x d rotation; h > 1 = h independent (d/h) x (d/h) problems */
  uint32_t act_dtype;       /* conqur_dtype of X; the rotate operand is R rounded to this type      */
  uint32_t max_tokens;      /* largest T passed to step_batch / quant_error (sizes the workspaces);
                               (d/heads) * round_up(max_tokens, 64) < 2^30                           */
  float prox_lambda;        /* R <- polar(M + lambda * tau * R_prev), tau = ||M||_F / sqrt(dh): the proximal
                               reading that makes the update unique when M is rank deficient.  0 asks for
                               the paper's update R <- polar(M) (Sec. 3.3) and is taken as the limit
                               lambda -> 0+ at fp32 resolution: values below 2^-20 are raised to 2^-20
                               (that ties R to R_prev on the null space of M, where every completion is
                               optimal, and breaks exact degeneracies a polynomial iteration would keep;
                               it moves <R, M> by less than 1e-6 relative)                            */
  float polar_tol;          /* stop when ||X^T X - I||_F <= tol; 0 selects 9.5e-5                    */
  uint32_t polar_max_iters; /* 0 selects 200                                                        */
  uint32_t polar_precision; /* arithmetic of the main polar iterations: 0 = single fp16 operands (fast; 11
                               significant bits: meets the orthogonality and objective tolerances, R itself
                               deviates a little on directions with small singular values, where a step's
                               rounding is amplified by 1/sigma), 1 = two bf16 planes per operand (about 16
                               significant bits), 2 = three planes (fp32-equivalent products).
                               The closing iterations always run fp32-equivalent.                     */
  uint32_t polar_verify;    /* orthogonality of the final iterate: 0 = bounded from the last measured
                               residual (exact-arithmetic residual of the closing step, from ||D^3||_F,
                               plus a rounding allowance; one bf16 GEMM), 1 = measured by one more
                               fp32-equivalent Gram matrix (costs about six bf16 GEMMs)               */
  int32_t device;           /* HIP device ordinal                                                   */
  void* stream;             /* hipStream_t the caller owns (NULL = the device's default stream)      */
} conqur_config;

/* Per-head statistics of the rows accumulated since the last update (HOST struct). */
typedef struct {
  uint64_t rows;    /* rows that entered M                                                         */
  uint64_t skipped; /* rows skipped: all-zero or non-finite head slice                             */
  double l1;        /* L = sum_i ||y_i||_1 / ||x_i||_2                                               */
  double objective; /* Eq. 1 summed over those rows, sum_i || y_i/||x_i|| - c_i ||^2, evaluated through
                       the l1 identity of Sec. 3.2 as 2*rows - 2*L/sqrt(dh)                          */
} conqur_batch_stats;

/* Per-head result of one Procrustes update (HOST struct). */
typedef struct {
  uint32_t iters;       /* polar iterations run (main + closing)                                   */
  uint32_t accurate;    /* how many of them were closing iterations (fp32-equivalent Gram)         */
  double orth_err;      /* ||R^T R - I||_F of the stored fp32 R: measured on the device, or an upper
                           estimate of it (see polar_verify)                                         */
  double inner;         /* <R_new, M>, the Procrustes objective value (nuclear norm at the optimum)  */
  double m_fro;         /* ||M||_F                                                                  */
  double ms;            /* device time of this update in milliseconds (all heads together)          */
  uint32_t orth_measured; /* 1: orth_err was measured; 0: it is the estimate                          */
  uint32_t reserved;
  double l1;            /* L of the rows this update consumed (as conqur_batch_stats.l1 just before it)   */
  double mfma_flop;     /* multiply-add work the update's matrix products issued, in FLOP, all heads
                           together (tiles that ran x tile area x contraction length x 2: symmetric
                           products run on the tiles on and above the diagonal only, split-plane
                           products count once per plane pair); the algorithmic figure is
                           4 dh^3 heads per iteration                                                 */
} conqur_update_stats;

/*
 * Create a context (Alg. 1 "initial rotation").  R0_host: HOST, heads*dh*dh floats,
 * head-major, each block row-major and orthogonal (not checked).  Copied; the caller
 * keeps ownership.  On success *out receives the context.  Allocates all device
 * memory the other calls need; those calls allocate nothing.
 */
conqur_status conqur_init(const conqur_config* cfg, const float* R0_host, conqur_ctx** out);

/*
 * One batch of the statistics loop (Alg. 1 inner loop; Sec. 3.4): for every row
 * x_i of X and every head, rotate with the operand copy of R, take the corner of
 * the rotated row (Eq. 2), and add (x_i/||x_i||)^T c_i to M.  May be called many
 * times before one update (Alg. 1 pools all sites of a mini-batch).
 * X_dev: DEVICE, T rows of row_stride_elems elements of act_dtype, of which the
 * first d are used; 16-byte aligned base and row pitch.  1 <= T <= max_tokens,
 * T * row_stride_elems < 2^30 (CONQUR_EINVAL otherwise).  The caller keeps ownership of X and may reuse it once the stream has passed
 * this call's kernels.  Asynchronous; never touches the host.
 */
conqur_status conqur_step_batch(conqur_ctx* ctx, const void* X_dev, uint64_t T, uint64_t row_stride_elems);

/*
 * The same for the heads [head0, head0 + nheads) only: X_dev holds T rows whose first
 * nheads * dh columns belong to those heads.  One context can so carry the per-head
 * rotations of several layers (Alg. 1 keeps one R_2 per layer, App. A one block per
 * head): every layer's batch goes to its own range, and a single
 * conqur_update_rotation then updates all of them in batched launches that fill the
 * device, which one layer's heads alone do not.  A partial range needs heads of width
 * 128 and bf16 activations (CONQUR_EINVAL otherwise); the full range is
 * conqur_step_batch.  Every head must have received rows before the update
 * (CONQUR_ESTATE otherwise).  After a partial range conqur_get_last_corners has nothing
 * to return (CONQUR_ESTATE).
 */
conqur_status conqur_step_batch_heads(conqur_ctx* ctx, const void* X_dev, uint64_t T, uint64_t row_stride_elems,
                                      uint32_t head0, uint32_t nheads);

/*
 * Read the per-head statistics accumulated since the last update.  stats_host:
 * HOST array of `heads` entries.  Synchronises the stream.
 */
conqur_status conqur_get_batch_stats(conqur_ctx* ctx, conqur_batch_stats* stats_host);

/*
 * Orthogonal Procrustes update (Sec. 3.3): R <- polar(M + prox_lambda*tau*R) per
 * head, computed on the device by a GEMM-only Newton-Schulz iteration; refreshes
 * the rotate operand and clears M and the batch statistics (Alg. 1 starts every
 * mini-batch with empty statistics).  stats_host: HOST array of `heads` entries or
 * NULL.  Synchronises the stream (the iteration count is data dependent).
 * Returns CONQUR_ESTATE if no row was accumulated, CONQUR_ENOCONV if the cap was
 * hit (R is still replaced; stats->orth_err tells how good it is), and
 * CONQUR_ENONFINITE (after a successful update) if rows were skipped as non-finite.
 */
conqur_status conqur_update_rotation(conqur_ctx* ctx, conqur_update_stats* stats_host);

/*
 * Score the current rotation (App. B symmetric quantiser; Sec. 4.3 error metric):
 * Y = X R_op per head, stored in act_dtype, then per token (one scale over the whole
 * row of width d) D = max|y| / (2^(bits-1) - 1), q = D * round_half_even(y / D)
 * clamped to the level range.  sse_host = sum (y - q)^2, energy_host = sum y^2
 * (both HOST doubles).  X_dev as in conqur_step_batch.  bits in [2, 8].  Does not
 * change the calibration state.  Synchronises the stream.
 */
conqur_status conqur_quant_error(conqur_ctx* ctx, const void* X_dev, uint64_t T, uint64_t row_stride_elems,
                                 uint32_t bits, double* sse_host, double* energy_host);

/*
 * The same score with the per-token asymmetric (zero-point) quantiser (App. B, "zeropoint
 * quantizer"; App. C evaluates activations with clipping ratio 0.9): per token, over the
 * whole row, lo = clip_ratio * min_j y_j, hi = clip_ratio * max_j y_j, D = (hi - lo) /
 * (2^bits - 1), integer zero point zeta = -round_half_even(lo / D), code = round_half_even(y / D)
 * + zeta clamped to [0, 2^bits - 1], q = D * (code - zeta); a constant row has the single
 * level lo.  clip_ratio in (0, 1] (1: the appendix's quantiser).  Arguments, outputs,
 * synchronisation and errors as conqur_quant_error.
 */
conqur_status conqur_quant_error_zp(conqur_ctx* ctx, const void* X_dev, uint64_t T, uint64_t row_stride_elems,
                                    uint32_t bits, float clip_ratio, double* sse_host, double* energy_host);

/*
 * The rotated rows themselves: Y = X R_op per head (R_op = R rounded to act_dtype;
 * fp32-equivalent products for fp32), stored in act_dtype -- Eq. 1's R x~ before
 * normalisation; with the rows of a weight matrix as X this folds the learned rotation
 * into that matrix (App. A).  X_dev as in conqur_step_batch (T <= max_tokens rows per
 * call).  Y_dev: DEVICE, T rows of y_row_stride_elems elements of act_dtype
 * (d <= y_row_stride_elems < 2^21, else CONQUR_EINVAL), owned by the caller, must not
 * overlap X.  Asynchronous on the context's stream; does not change the calibration
 * state.
 */
conqur_status conqur_rotate(conqur_ctx* ctx, const void* X_dev, uint64_t T, uint64_t row_stride_elems, void* Y_dev,
                            uint64_t y_row_stride_elems);

/*
 * The fake-quantised rotated rows: Yq = Q(X R_op), what a linear layer receives when its
 * input is quantised after the current rotation has been applied (quantisation-aware
 * calibration, Sec. 3.4).  Y = X R_op as in conqur_rotate; each row of width d is then
 * quantised per token with the symmetric quantiser of conqur_quant_error (zero_point =
 * 0; clip_ratio ignored) or the zero-point quantiser of conqur_quant_error_zp
 * (zero_point = 1, clip_ratio in (0, 1]) and written as the level values q (not the
 * integer codes), rounded once into act_dtype.  Yq_dev: DEVICE, T rows of
 * yq_row_stride_elems >= d elements of act_dtype, base and row pitch multiples of 16
 * bytes, owned by the caller, must not overlap X.  Asynchronous on the context's stream;
 * does not change the calibration state.  Errors: CONQUR_EINVAL (bits outside [2, 8],
 * zero_point > 1, clip_ratio outside (0, 1], NULL / misaligned Yq_dev, bad X
 * arguments), CONQUR_EHIP.
 */
conqur_status conqur_rotate_quant(conqur_ctx* ctx, const void* X_dev, uint64_t T, uint64_t row_stride_elems, uint32_t bits,
                                  uint32_t zero_point, float clip_ratio, void* Yq_dev, uint64_t yq_row_stride_elems);

/*
 * Quantisation-aware calibration (Sec. 3.4, second paragraph: during calibration the input of every
 * linear layer is quantised after the current rotation has been applied, so that later sites see
 * the activations inference will give them): conqur_step_batch and conqur_rotate_quant of the same
 * batch in ONE call and from ONE rotation of X.  The site's statistics are accumulated exactly as
 * conqur_step_batch does, and Yq_dev receives Q(X R_op) exactly as conqur_rotate_quant writes it --
 * the quantised input of the layer behind the site.  Arguments and errors as for those two calls.
 * (Heads of width 128 with bf16 activations rotate twice internally: their fused step keeps the
 * rotated rows on the compute unit.)  Asynchronous on the context's stream.
 */
conqur_status conqur_step_batch_quant(conqur_ctx* ctx, const void* X_dev, uint64_t T, uint64_t row_stride_elems, uint32_t bits,
                                      uint32_t zero_point, float clip_ratio, void* Yq_dev, uint64_t yq_row_stride_elems);

/*
 * Per-row diagnostics of the rotated activations: Y = X R_op per head, stored in
 * act_dtype, then per token over the whole row of width d
 *   pr  = ||y||_2^4 / (d ||y||_4^4)   normalised participation ratio (Sec. 4.2), in [1/d, 1]
 *   rho = ||y||_inf^2 / ||y||_2^2     dynamic-range ratio of the SQNR bound (App. B), in [1/d, 1]
 * pr_host / rho_host: HOST, T floats each, either may be NULL; a row with zero or
 * non-finite energy gets 0.  X_dev as in conqur_step_batch.  Does not change the
 * calibration state.  Synchronises the stream.
 */
conqur_status conqur_row_diagnostics(conqur_ctx* ctx, const void* X_dev, uint64_t T, uint64_t row_stride_elems,
                                     float* pr_host, float* rho_host);

/*
 * Copy state to the host / replace it (checkpointing, and teacher-forced parity
 * tests).  R_host, M_host: HOST, heads*dh*dh floats or NULL.  n_rows_host: HOST,
 * `heads` entries or NULL: the rows that entered M since the last update (as
 * conqur_batch_stats.rows).  set_state(R) also refreshes the rotate operand;
 * set_state(M) marks the statistics as holding rows, so that an update may follow; the
 * row and skipped counters and the l1 term then still describe the rows stepped through
 * the library, not the M that was written.  Both synchronise the stream.
 */
conqur_status conqur_get_state(conqur_ctx* ctx, float* R_host, float* M_host, uint64_t* n_rows_host);
conqur_status conqur_set_state(conqur_ctx* ctx, const float* R_host, const float* M_host);

/*
 * Keep (enable != 0) or drop (0, the default) the corner signs of every later
 * conqur_step_batch for conqur_get_last_corners.  Only the fused per-head step
 * (heads of width 128, bf16 activations) honours the switch -- there the signs never
 * leave the compute unit otherwise and storing them doubles the step's HBM traffic;
 * the general path produces them anyway as an operand of the accumulate GEMM.
 */
conqur_status conqur_set_taps(conqur_ctx* ctx, int enable);

/*
 * Debug / parity taps of the last conqur_step_batch: the corner signs as int8
 * (+1 / -1; HOST, T*d, row-major like X) and the per-row norms (HOST, heads*T,
 * head-major; 0 marks a skipped row).  Either may be NULL.  Synchronises.
 * CONQUR_ESTATE if the signs are asked for and the last step did not keep them
 * (see conqur_set_taps).
 */
conqur_status conqur_get_last_corners(conqur_ctx* ctx, int8_t* signs_host, float* norms_host);

/*
 * For callers that cannot allocate device memory or wait for the stream (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the score of
 * conqur_quant_error (zero_point = 0; clip_ratio ignored) or conqur_quant_error_zp (zero_point
 * = 1) on rows that are ALREADY rotated -- Y_dev is what conqur_rotate wrote -- with the two
 * results left in device memory.  No context: the per-row results the score kernels exchange
 * live in a static device array of the library (2 floats per row, 512 KiB, held by every GPU
 * the library has run on until the process ends), so the call allocates nothing, copies
 * nothing to the host and returns without waiting.  Runs on the CURRENT device; `stream` must
 * belong to it (NULL = its default stream).  The array's address is looked up once per device,
 * by conqur_init or by the first call on that device: make that first call outside any graph
 * capture.  Y_dev: DEVICE, T rows of row_stride_elems >= d elements of dtype (conqur_dtype),
 * 16-byte aligned base and row pitch; 1 <= T <= 65536 rows per call (more: CONQUR_EINVAL, split
 * the rows over several calls and add the results); d a multiple of 16, at most 65536.
 * out_dev: DEVICE, 2 doubles, overwritten with { sum (y - q)^2, sum y^2 } once the stream has
 * passed the call's kernels.  All calls on one GPU share the array, which keeps the last
 * call's per-row values: calls that overlap in time on one GPU (different streams) race; calls
 * on one stream are ordered and safe.  Errors: CONQUR_EINVAL (arguments as above, bits outside
 * [2, 8], zero_point > 1, clip_ratio outside (0, 1]), CONQUR_EHIP.
 */
conqur_status conqur_score_rows_static(const void* Y_dev, uint32_t dtype, uint64_t T, uint64_t d, uint64_t row_stride_elems,
                                       uint32_t bits, uint32_t zero_point, float clip_ratio, double* out_dev, void* stream);

/* Device times (ms) of the most recent call of each kind, measured with HIP events on the
 * context's stream.  level 0: off.  level 1: one event pair around each whole call (what a
 * caller's pipeline sees: the call's kernels run back to back).  level 2: additionally one
 * pair per stage -- the records between the kernels keep one kernel's launch from
 * overlapping the previous kernel's tail, so the stages sum to more than the whole call --
 * and the clock probes of conqur_get_clock_probe.  out_host: HOST, 12 floats:
 * [0] step: prepare (norms + transposed operand)  [1] step: rotate+corner GEMM
 * [2] step: accumulate GEMM                       [3] step: statistics reduction
 * [4] update: whole polar update                  [5] quant: rotate GEMM
 * [6] quant: error kernel                         [7] whole conqur_step_batch
 * [8] whole conqur_quant_error (device part)      [9..11] reserved (0)
 * Entries whose events were not recorded at the current level are 0.                       */
conqur_status conqur_set_timing(conqur_ctx* ctx, int level);
conqur_status conqur_get_timing(conqur_ctx* ctx, float* out_host);

/* Clock probe of the two GEMM launches of the most recent conqur_step_batch that ran with timing
 * level 2: means over the launch's workgroups.  out_host: HOST, 8 floats:
 * [0] shader clock (MHz) sustained during the rotate+corner GEMM's main loop  [1] its main-loop time (us)
 * [2] its prologue (first operand tiles arriving) (us)      [3] its epilogue (us)
 * [4..7] the same for the accumulate GEMM.  Zeros if no probe was taken.  Synchronises.           */
conqur_status conqur_get_clock_probe(conqur_ctx* ctx, float* out_host);

/* Environment: CONQUR_TRACE (set to anything) makes conqur_update_rotation print one line per polar step to stderr
 * (interval, coefficients, measured and predicted residuals) and measure a few quantities it otherwise skips; results
 * are unchanged.  Nothing else is read from the environment. */

/* Last error text of this context (HOST string owned by the context; "" if none). */
const char* conqur_last_error(const conqur_ctx* ctx);

/* Release the context and all device memory it owns.  NULL is allowed. */
void conqur_destroy(conqur_ctx* ctx);

/* Library version string, e.g. "conqur-gfx950 0.1". */
const char* conqur_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CONQUR_H */
