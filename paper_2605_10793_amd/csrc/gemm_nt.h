// bf16 MFMA GEMM for gfx950, "NT" form: both operands are K-contiguous,
//   acc[m][n] = sum_seg sum_k A[seg.a + m*lda + k] * B[seg.b + n*ldb + k]    (fp32 accumulate)
// followed by one of a few fused epilogues.  Every dense contraction of the
// calibration path (rotate, accumulate, Gram, polynomial apply) is this kernel:
// operands that are K-strided in their natural layout are produced transposed by
// the kernel that writes them, and fp32-accurate products are obtained by feeding
// bf16 split planes as several K-segments (hi*hi, hi*mid, mid*hi, ...).
#pragma once
#include "common.h"

namespace conqur {

enum GemmEpilogue : int {
  EPI_SIGN = 0,  // corner signs, transposed: St[n][m] = +-1 (bf16 or fp16)
  EPI_ACT = 1,   // Y[m][n] = acc, stored as bf16 or fp32 (rotated activations for the quantiser score)
  EPI_F32 = 2,   // C[m][n] = out_scale * acc (+ C[m][n] if accumulate), fp32
  EPI_GRAMW = 3, // acc = Gram matrix G: W = coef_i*I + coef_g*G (+ the planes Padd) written as np_out bf16 split
                 // planes (natural layout) and per-wavefront partial sums of (G - I)^2
  EPI_XOUT = 4,  // acc = X' (+ Xadd): written as fp32 (C32) and/or np_out bf16 split planes in natural (Pn)
                 // and transposed (Pt) layout -- the operands of the next Gram / apply GEMMs
  EPI_SQUARE = 5, // acc = D^2 (D symmetric, given as two planes Padd): writes acc as one bf16 plane (Pacc) and
                  // coef_g * acc + D as two split planes (Pn); per-wavefront partial sums of acc^2 (resid_part) if asked
  EPI_FRO2 = 6,   // per-wavefront partial sums of acc^2 only (resid_part): a Frobenius norm, nothing stored
  EPI_XLAST = 7,  // acc = X' rounded to np_out (1 or 2) bf16 split planes: exactly that value goes to C32 (fp32), to
                  // np_out natural planes (Pn) and to np_out transposed planes (Pt) -- the hand-over from the
                  // low-precision polar steps to the closing ones, whose Gram matrix is then exact with 1 or 4 plane
                  // products instead of the 6 a 24-bit iterate needs
  EPI_SIGN_ACT = 8, // EPI_SIGN and EPI_ACT of the same accumulators: St as for EPI_SIGN, and Y[m][n] = acc stored as bf16 or
                  // fp32 (Yact): one rotation of a batch serves the corner statistics and the quantiser that follows
  EPI_SIGN_XT = 9, // EPI_SIGN, and the accumulate GEMM's other operand on the way (square problems, N == K, bf16 A): every
                  // wavefront also takes the block of A that lies under its output block (rows = its tokens, columns = its
                  // output columns read as input channels), scales each row by w, converts to fp16 and stores it
                  // transposed, Xt[channel][token], through the same LDS staging as the signs; the first tile column
                  // counts the rows (w != 0 / w == 0) into cnt.  Saves the separate transposing launch.
};

constexpr int kMaxSegments = 6;

struct GemmArgs {
  const bf16_bits* A;
  const bf16_bits* B;
  int64_t lda, ldb;        // row pitch in elements (multiples of 8)
  int64_t batchA, batchB;  // element offset between batch entries (grid.z)
  int M, N, K;             // K per segment, a multiple of 8
  int ab_f16;              // operands hold fp16 instead of bf16 (EPI_F32; EPI_GRAMW / EPI_XOUT with one output plane,
                           // which is then fp16 as well: the single-plane polar steps; EPI_XLAST, whose outputs stay bf16)
  int nseg;
  int64_t a_seg[kMaxSegments];  // element offsets of each K-segment
  int64_t b_seg[kMaxSegments];
  // epilogue
  void* C;                 // EPI_SIGN: bf16 St; EPI_ACT: bf16/f32 Y; EPI_F32: fp32
  int64_t ldc, batchC;     // pitch / batch offset of every output of the epilogue (elements)
  int c_is_f32;            // EPI_ACT: element type of C
  int accumulate;          // EPI_F32: add to C instead of overwriting
  float out_scale;         // EPI_F32: C = out_scale * acc (+ C)
  int64_t st_rows_valid;   // EPI_SIGN: St rows hold this many m entries (padded pitch), multiple of 4
  int sign_f16;            // EPI_SIGN: write +-1 as fp16 instead of bf16
  const float* xt_w;       // EPI_SIGN_XT: row weights [batch][ldw] (0: the row is skipped and contributes zeros)
  int64_t xt_ldw;
  bf16_bits* Xt;           // EPI_SIGN_XT: fp16 [batch][N][ldc] (pitch and batch offset of C), columns m < st_rows_valid written
  unsigned long long* cnt; // EPI_SIGN_XT: [batch][cnt_slots][2] row counters (entered, skipped); tile row tm adds to slot tm % cnt_slots
  int cnt_slots;
  void* Yact;              // EPI_SIGN_ACT: bf16/f32 Y (element type by c_is_f32), pitch ldy, batch offset batchY
  int64_t ldy, batchY;
  double* resid_part;      // EPI_GRAMW: [batch][gemm_num_partials()] per-wavefront sums of (acc - I)^2, or null.
                           // (No atomics: same-address atomics from all XCDs serialise at the memory side.)
  float coef_i, coef_g;    // EPI_GRAMW
  int np_out;              // EPI_GRAMW: planes of W written; EPI_XOUT: transposed planes (Pt) written (1..3);
                           // plane p holds the p-th bf16 split term
  int np_out_n;            // EPI_XOUT: natural planes (Pn) written (<= 3)
  const bf16_bits* Padd;   // EPI_GRAMW: np_add planes [m][n] (same pitch / plane offset) whose sum is added to W,
  int np_add;              //            or null: W = coef_i*I + coef_g*acc + sum_p Padd[p]
  int64_t plane_out;       //   element offset between output planes
  bf16_bits* Pn;           // EPI_GRAMW: W planes; EPI_XOUT: X' planes, natural [m][n] (may be null)
  bf16_bits* Pt;           // EPI_XOUT: X' planes, transposed [n][m] (may be null)
  float* C32;              // EPI_XOUT: X' in fp32 [m][n] (may be null)
  const float* Xadd;       // EPI_XOUT: fp32 [m][n] added to acc before writing (may be null)
  bf16_bits* Pacc;         // EPI_SQUARE: the accumulator itself as one bf16 plane [m][n]
  int symmetric;           // EPI_GRAMW / EPI_SQUARE, A and B the same matrix (so M == N and the result is symmetric):
                           // only the tiles on and above the diagonal are computed, each also stored mirrored
                           // (EPI_FRO2: A, B two commuting symmetric matrices; tiles above the diagonal count twice).  With
                           // half the workgroups the chip's power limit allows a higher clock: at 4096^3 the
                           // launch takes 0.8 of the full one's time; with more tiles than CUs it saves tile rounds.
                           // Used when the chosen tile is square and there are at least 8 tiles per side.
  unsigned long long* clk; // optional clock probe, 4 values per workgroup (see gemm_num_workgroups): main-loop
                           // shader cycles, then 100 MHz ticks of main loop, prologue, epilogue (may be null)
};

// Enqueue the GEMM on `stream`.  Returns hipSuccess or the launch error.
hipError_t launch_gemm_nt(const GemmArgs& args, GemmEpilogue epi, int batch, hipStream_t stream);

// Multiply-add work launch_gemm_nt issues for these arguments, in FLOP: workgroups that run x tile area x K x segments
// x 2 (a symmetric launch runs the tiles on and above the diagonal only).
double gemm_issued_flop(const GemmArgs& args, GemmEpilogue epi, int batch);

// Number of workgroups launch_gemm_nt uses for an M x N problem with `batch` entries (size of the clock probe / 4).
int gemm_num_workgroups(int M, int N, int batch);

// Per-batch-entry count of the partial sums the EPI_GRAMW / EPI_FRO2 epilogues write for an M x N problem launched
// with the given `symmetric` flag (the flag can select another tile).
int gemm_num_partials(int M, int N, int batch, int symmetric);


}  // namespace conqur
