// Non-GEMM kernels of the calibration path: row norms, scaled/transposed operand
// preparation, bf16 split packing, statistics reductions, polar start/finish and
// the bandwidth-bound fake-quantisation error kernel.  Launch wrappers only; each
// returns the launch status.
#pragma once
#include "common.h"

namespace conqur {

// n_i = ||x_i||_2 over each head slice; w_i = kXhatScale / n_i, or 0 for a row that is
// all zero or holds a non-finite value (then nrm = 0 and *nonfinite is raised for NaN/Inf).
hipError_t launch_row_norms(const void* X, int x_is_f32, int64_t T, int64_t stride, int heads, int dh,
                            float* nrm, float* w, int64_t ldn, int* nonfinite, hipStream_t s);

// Xt[p][k][i] = x_ik * w_{head(k), i} for i < T, 0 for T <= i < Tk.  np = 1 (bf16 activations):
// one fp16 plane; np = 3 (fp32 activations): three bf16 split planes (exact).
// Also counts the rows (w != 0: entered M, w == 0: skipped) into cnt [heads][kCountSlots][2], the token block b
// into slot b % kCountSlots.
constexpr int kCountSlots = 64;
hipError_t launch_transpose_scale(const void* X, int x_is_f32, int64_t T, int64_t Tk, int64_t stride, int d, int dh,
                                  const float* w, int64_t ldn, bf16_bits* Xt, int64_t pitch, int64_t plane, int np,
                                  unsigned long long* cnt, hipStream_t s);

// Xs[p][i][k] = split_p(x_ik), fp32 activations only (3 planes).
hipError_t launch_split_rows(const float* X, int64_t T, int64_t stride, int d, bf16_bits* Xs, int64_t plane,
                             hipStream_t s);

// Split an fp32 matrix batch [batch][rows][cols] into np bf16 planes, in natural
// layout (outN[p][b][r][c]) and/or transposed (outT[p][b][c][r]); either may be null.
// out_f16 (np = 1 only): the plane holds the values rounded to fp16 instead of bf16.
hipError_t launch_pack(const float* src, int batch, int rows, int cols, int np, bf16_bits* outN, bf16_bits* outT,
                       int64_t plane, hipStream_t s, int out_f16 = 0);

// out[h] = <R_op,h , M_h> over n elements per head, R_op = R rounded to bf16 if round_bf16 else R (the l1 term of
// the accumulated rows is sqrt(dh) times this).  part: heads * dot_rm_partials(n) doubles of scratch.
int dot_rm_partials(int64_t n);
hipError_t launch_dot_rm(const float* R, const float* M, int heads, int64_t n, int round_bf16, double* part, double* out,
                         hipStream_t s);

// fro2[h] = sum M_h^2 (overwritten).  part: heads * dot_rm_partials(n) doubles of scratch.
hipError_t launch_fro2(const float* M, int heads, int64_t n, double* part, double* fro2, hipStream_t s);

// Start of the polar iteration, fused with the operand packing: X0 = (M + lambda*tau*R) / alpha with
// tau = ||M||_F/sqrt(dh), alpha = ||M||_F (1 + lambda) (a head with M = 0 starts from R itself), written as np bf16
// split planes in natural (outN) and transposed (outT) layout and, if X32 is not null, in fp32.
// If dot_part is not null (heads * pack_dot_partials(dh) doubles), also dot_out[h] = <R_op,h , M_h> (R_op = R rounded to bf16 if
// round_bf16), the quantity of launch_dot_rm, from the same pass.
hipError_t launch_polar_start_pack(const float* M, const float* R, int heads, int dh, float lambda, const double* fro2, int np,
                                   float* X32, bf16_bits* outN, bf16_bits* outT, int64_t plane, int round_bf16,
                                   double* dot_part, double* dot_out, hipStream_t s, int out_f16 = 0);

// X += kappa * R over n elements (all heads).
hipError_t launch_axpy(float* X, const float* R, int64_t n, float kappa, hipStream_t s);

// End of the polar iteration, one pass over X: inner[h] = <X_h, M_h> (overwritten), the rotate operand outT =
// np bf16 split planes of X^T, and, if R32 is not null, R32 = X.  dot_part: heads * pack_dot_partials(dh) doubles.
int pack_dot_partials(int dh);
hipError_t launch_polar_finish_pack(const float* X, const float* M, int heads, int dh, int np, float* R32, bf16_bits* outT,
                                    int64_t plane, double* dot_part, double* inner, hipStream_t s);

// Fused statistics step for heads of width 128 with bf16 activations (head_step.hip): one kernel rotates, normalises,
// takes the corners and accumulates; every workgroup (head, share of the tokens) stores a partial M_h into
// Mpart [nsplit][heads][128][128], adds its share of L / rows / skipped, writes the row norms and, if St is not null,
// the corner signs (+-1 as fp16, transposed [heads*128][pitch]).  launch_head_reduce then sets or adds the shares to M.
// The partial M_h already carry the factor 1 / (kXhatScale sqrt(128)).
int head_step_splits(int heads, int64_t T);
hipError_t launch_head_step128(const bf16_bits* X, int64_t T, int64_t stride, int heads, const bf16_bits* RopT, float* Mpart,
                               int nsplit, float* nrm, int64_t ldn, double* L, unsigned long long* rows,
                               unsigned long long* skipped, int* nonfinite, bf16_bits* St, int64_t pitch, hipStream_t s);
// fro2_part non-null: also 16 partial sums of squares per head of the resulting M (kHeadReduceParts doubles per head, in
// head order), whose sum per head is ||M_h||_F^2.
// The same sum for any matrix of n_total floats (a multiple of 1024) held as nsplit shares [nsplit][n_total], fixed order.
hipError_t launch_sum_shares(const float* part, int nsplit, int64_t n_total, float* M, int accumulate, hipStream_t s);
constexpr int kHeadReduceParts = 16;
hipError_t launch_head_reduce(const float* Mpart, int nsplit, int heads, float* M, int accumulate, double* fro2_part, hipStream_t s);

// Main phase of the polar iteration for heads of width 128 in one launch (head_polar.hip): runs the composed cubics
// X <- X (a_k I + b_k X^T X), k < nsteps, on single fp16 operand planes held in LDS (11 significant bits).  Xn0 / Xt0:
// the start iterate as one natural and one transposed fp16 plane [heads][128][128].  Outputs, as the last step of the
// general path writes them: the result rounded to bf16, as X32 (fp32), Pt (one transposed bf16 plane) and Pn (one
// natural bf16 plane).
constexpr int kPolarScheduleMax = 64;
struct PolarSchedule {
  int nsteps;
  float a[kPolarScheduleMax], b[kPolarScheduleMax];
};
// close non-null: each head whose residual ||I - X^T X||_F at the hand-over is at most res_max also takes the closing
// step X <- X + X (D + 1.5 D^2), D = (I - X^T X)/2, in the same launch and writes R (fp32), RopT (bf16 plane of R^T) and
// inner_out[h] = <R, M>; res_out[h] = ||I - X^T X||_F^2 at the hand-over, sq_out[h] = ||D^2||_F^2, or < 0 if the head did
// not take the step (then R, RopT and inner_out of that head are untouched).  The hand-over outputs are written either way.
struct HeadPolarClose {
  float* R;
  bf16_bits* RopT;
  const float* M;
  double* res_out;
  double* sq_out;
  double* inner_out;
  float res_max;
};
// start non-null: the launch forms the start iterate itself, X0 = (M + lambda tau R) / alpha per head (Xn0 / Xt0 unused,
// may be null), from M, R (fp32 [heads][128][128]) and ||M_h||_F^2 = the sum of nparts partial sums per head
// (fro2_parts[h * nparts + p]); it also stores that sum to fro2_out[h] and, if ldot is non-null, copies L[h] to ldot[h].
struct HeadPolarStart {
  const float* M;
  const float* R;
  const double* fro2_parts;
  int nparts;
  double* fro2_out;
  float lambda;
  const double* L;
  double* ldot;
};
hipError_t launch_head_polar128(const bf16_bits* Xn0, const bf16_bits* Xt0, int heads, const PolarSchedule& sched, float* X32,
                                bf16_bits* Pn, bf16_bits* Pt, const HeadPolarClose* close, const HeadPolarStart* start,
                                hipStream_t s);

// Per-row fake-quantisation error of Y [T][ld] (bf16 or fp32) into row_sse / row_en, then their sums over rows:
// out[0] = SSE, out[1] = energy (skipped if out is null).  zero_point = 0: symmetric quantiser; 1: zero-point quantiser on [clip*min, clip*max].
// Q non-null: the quantised rows are also written to Q [T][ldq] in Y's element type (Q must not overlap Y).
hipError_t launch_quant_error(const void* Y, int y_is_f32, int64_t T, int64_t ld, int d, int bits, int zero_point, float clip,
                              float* row_sse, float* row_en, double* out, void* Q, int64_t ldq, hipStream_t s);

// Per-row diagnostics of Y [T][ld] (bf16 or fp32): row_pr = ||y||_2^4 / (d ||y||_4^4), row_rho = ||y||_inf^2 / ||y||_2^2
// (0, 0 for a row with zero or non-finite energy).
hipError_t launch_row_diag(const void* Y, int y_is_f32, int64_t T, int64_t ld, int d, float* row_pr, float* row_rho,
                           hipStream_t s);

// out[h] = sum of part[h][0..n) for h < heads, fixed order.
hipError_t launch_sum_partials(const double* part, int n, int heads, double* out, hipStream_t s);

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);

// Device address, on the current device, of the static array conqur_score_rows_static keeps its per-row results in
// (static_score.hip); looked up once per device.
hipError_t static_scratch_for_current_device(float** out);

}  // namespace conqur
