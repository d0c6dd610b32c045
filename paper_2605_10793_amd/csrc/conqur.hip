// Host side of libconqur: context, argument checks, kernel sequencing and the
// polar-iteration control loop.  All arithmetic of the method runs in the HIP
// kernels of gemm_nt.hip / kernels.hip; there is no CPU fallback.
#include "../../include/conqur.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "gemm_nt.h"
#include "kernels.h"

using namespace conqur;

namespace {

// K-segment schedules for products of bf16 split planes.  (a, b) multiplies plane a
// of the left operand with plane b of the right one; smallest terms first.
struct SegList { int n; int a[kMaxSegments]; int b[kMaxSegments]; };
constexpr SegList kSeg1 = {1, {0}, {0}};
constexpr SegList kSeg3 = {3, {1, 0, 0}, {0, 1, 0}};                     // two planes each: hi*hi + hi*lo + lo*hi
constexpr SegList kSeg6 = {6, {2, 1, 0, 1, 0, 0}, {0, 1, 2, 0, 1, 0}};  // all terms down to 2^-24 relative
constexpr SegList kSeg4 = {4, {1, 1, 0, 0}, {1, 0, 1, 0}};              // both operands exactly two planes: every term
constexpr SegList kSeg2 = {2, {0, 0}, {1, 0}};                          // exact one-plane left operand, two-plane right
constexpr SegList kSeg3x1 = {3, {2, 1, 0}, {0, 0, 0}};                   // 3-plane left operand, exact right operand

constexpr int kResidSlots = 512;
// Rounding share of ||X^T X - I||_F after a closing step, per unit of dh (correction product from two-plane
// operands, fp32 iterate): used where the residual is predicted instead of measured.
constexpr double kOrthFloorPerDim = 1e-8;
constexpr double kCubeFactor = 5.5;
constexpr int kClkMaxWorkgroups = 8192;    // clock probes are taken for GEMM launches of at most this many workgroups
constexpr int64_t kHostSumRows = 16384;    // quant_error: up to this many rows the host adds the per-row results

enum Stage { ST_PREP = 0, ST_ROTATE, ST_ACCUM, ST_STATS, ST_UPDATE, ST_QROT, ST_QERR, ST_STEP, ST_QUANT, ST_COUNT };
constexpr int kTimingSlots = 12;

}  // namespace

struct conqur_ctx {
  conqur_config cfg{};
  int d = 0, heads = 0, dh = 0, np = 1;  // np: bf16 planes per activation operand (1 bf16, 3 fp32)
  bool f32 = false;
  int64_t tmax = 0, pitch = 0;            // pitch: token pitch of the transposed operands
  hipStream_t stream = nullptr;
  std::string err;

  float* R = nullptr;          // [heads][dh][dh] fp32 master rotation
  bf16_bits* RopT = nullptr;   // [np][heads][dh][dh] planes of R^T in the activation dtype (rotate operand)
  float* M = nullptr;          // [heads][dh][dh]
  bool m_empty = true;         // M holds no rows: the next accumulate overwrites it
  bool have_rows = false;
  // Heads of width 128 may be stepped in ranges (conqur_step_batch_heads): the same two facts per head.
  std::vector<uint8_t> h_empty, h_rows;
  bf16_bits* Xt = nullptr;     // [np][d][pitch] scaled, transposed activations (fp16 plane, or 3 bf16 planes for fp32 input)
  bf16_bits* St = nullptr;     // [d][pitch] corner signs +-1, transposed (fp16, or bf16 for fp32 input)
  bf16_bits* Xs = nullptr;     // fp32 activations only: [3][tmax][d] split planes of X
  float *nrm = nullptr, *w = nullptr;  // [heads][tmax]
  unsigned long long* cnt = nullptr;   // [heads][kCountSlots][2] rows / skipped counters of the general path
  double* ldot = nullptr;              // [heads] <R_op, M> (l1 term / sqrt(dh)) of the general path
  double* dotrm_part = nullptr;        // scratch of launch_dot_rm
  std::vector<double> l_base;          // l1 offsets from rotations replaced while statistics were pending
  double* L = nullptr;         // [heads]
  unsigned long long *rows = nullptr, *skipped = nullptr;
  int* nonfinite = nullptr;
  void* Y = nullptr;           // [tmax][d] rotated activations (quantiser score)
  float *row_sse = nullptr, *row_en = nullptr;
  double* qsum = nullptr;      // [2]
  // polar workspaces
  float* PX = nullptr;                               // polar iterate, fp32 [heads][dh][dh]
  bf16_bits *PXn[2] = {nullptr, nullptr};            // iterate as bf16 split planes [3][heads][dh][dh], ping-pong
  bf16_bits *PXt[2] = {nullptr, nullptr};            // ... transposed
  bf16_bits *PW = nullptr, *PW2 = nullptr;           // polynomial factor planes [3][heads][dh][dh]
  double* resid = nullptr;                           // [kResidSlots][heads] residual history of one update
  double* resid_part = nullptr;                      // [heads][parts] per-wavefront partials of one Gram GEMM
  int resid_parts = 0;
  double *fro2 = nullptr, *inner = nullptr;          // [heads]
  double* dot_part = nullptr;                        // [heads][(dh/64)^2] per-tile partials of <R, M>
  int64_t last_T = 0;
  size_t stat_words = 0;
  // heads of width 128 with bf16 activations take the fused step kernel (head_step.hip)
  bool head_fused = false;
  float* Mpart = nullptr;                            // [head_splits][heads][128][128] partial M of the token shares
  int ksplit_max = 0;                                // > 0: one narrow rotation (general path): the accumulate GEMM may split its
                                                     // token range into up to this many shares of Mpart ([ksplit_max][dh][dh])
  int head_splits = 0;
  int parts_pending = 0;                             // > 0: M of all heads still lies in that many token shares of Mpart
                                                     // (a first batch's shares are summed when M is next needed: by the
                                                     // update, which takes ||M||_F from the same pass, or by a reader)
  bool taps = false;                                 // keep the corner signs of every step for conqur_get_last_corners
  bool last_signs_valid = false;

  int timing = 0;   // 0 off, 1 whole-call events, 2 per-stage events and GEMM clock probes as well
  unsigned long long* clk[2] = {nullptr, nullptr};   // clock probes of the step's rotate / accumulate GEMM
  int clk_wg[2] = {0, 0};                            // workgroups that wrote them in the last step (0: none)
  hipEvent_t ev[ST_COUNT][2]{};
  bool ev_valid[ST_COUNT]{};
  hipEvent_t ev_resid = nullptr;   // behind the copy of a closing residual: the host waits for this, not for the stream
  hipEvent_t ev_sq = nullptr;      // behind the copy of ||D^2||_F^2 of the closing step's D^2 product
  double* host_res = nullptr;      // pinned: [kResidSlots][heads] residual history, then the update's result block
  float* host_rows = nullptr;      // pinned: per-row errors and energies of one score call (up to kHostSumRows rows)
  std::vector<void*> allocs;
};

namespace {

conqur_status fail(conqur_ctx* c, conqur_status st, const std::string& msg) {
  if (c) c->err = msg;
  return st;
}
conqur_status hip_fail(conqur_ctx* c, hipError_t e, const char* where) {
  return fail(c, e == hipErrorOutOfMemory ? CONQUR_ENOMEM : CONQUR_EHIP, std::string(where) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(expr)                                        \
  do {                                                       \
    hipError_t e_ = (expr);                                  \
    if (e_ != hipSuccess) return hip_fail(ctx, e_, #expr);   \
  } while (0)

template <typename T>
hipError_t dev_alloc(conqur_ctx* c, T** p, size_t count) {
  void* q = nullptr;
  hipError_t e = hipMalloc(&q, count * sizeof(T) + 256);
  if (e != hipSuccess) return e;
  c->allocs.push_back(q);
  *p = reinterpret_cast<T*>(q);
  return hipMemsetAsync(q, 0, count * sizeof(T) + 256, c->stream);
}

struct StageTimer {
  conqur_ctx* c; int st; bool on;
  StageTimer(conqur_ctx* c_, int st_, int level = 2) : c(c_), st(st_), on(c_->timing >= level) {
    if (on) (void)hipEventRecord(c->ev[st][0], c->stream);
  }
  ~StageTimer() {
    if (on) { (void)hipEventRecord(c->ev[st][1], c->stream); c->ev_valid[st] = true; }
  }
};

conqur_status check_x(conqur_ctx* ctx, const void* X, uint64_t T, uint64_t stride) {
  if (!ctx) return CONQUR_EINVAL;
  if (!X) return fail(ctx, CONQUR_EINVAL, "X_dev is NULL");
  if (T < 1 || (int64_t)T > ctx->tmax) return fail(ctx, CONQUR_EINVAL, "T must be in [1, max_tokens]");
  if (stride < (uint64_t)ctx->d) return fail(ctx, CONQUR_EINVAL, "row_stride_elems < d");
  const uint64_t esz = ctx->f32 ? 4 : 2;
  if ((reinterpret_cast<uintptr_t>(X) & 15) || ((stride * esz) & 15))
    return fail(ctx, CONQUR_EINVAL, "X_dev base and row pitch must be 16-byte aligned");
  if (T * stride >= (1ull << 30)) return fail(ctx, CONQUR_EINVAL, "T * row_stride_elems must be below 2^30");
  return CONQUR_OK;
}

// Rotate GEMM: acc[i][j] = sum_k x_ik R_op[k][j] per head, as an NT product with
// B = R_op^T.  fp32 activations go through 3 + 3 bf16 planes (6 segments).
void rotate_args(conqur_ctx* c, const void* X, int64_t T, int64_t stride, GemmArgs* g) {
  std::memset(g, 0, sizeof(*g));
  const int64_t rplane = (int64_t)c->heads * c->dh * c->dh;
  g->B = c->RopT; g->ldb = c->dh; g->batchB = (int64_t)c->dh * c->dh;
  g->M = (int)T; g->N = c->dh; g->K = c->dh;
  g->batchA = c->dh;
  if (c->f32) {
    g->A = c->Xs; g->lda = c->d;
    g->nseg = kSeg6.n;
    for (int s = 0; s < kSeg6.n; ++s) { g->a_seg[s] = kSeg6.a[s] * c->tmax * c->d; g->b_seg[s] = kSeg6.b[s] * rplane; }
  } else {
    g->A = reinterpret_cast<const bf16_bits*>(X); g->lda = stride;
    g->nseg = 1;
  }
}

conqur_status refresh_operand(conqur_ctx* ctx) {
  const int64_t plane = (int64_t)ctx->heads * ctx->dh * ctx->dh;
  HIP_TRY(launch_pack(ctx->R, ctx->heads, ctx->dh, ctx->dh, ctx->np, nullptr, ctx->RopT, plane, ctx->stream));
  return CONQUR_OK;
}

}  // namespace

extern "C" {

const char* conqur_version(void) { return "conqur-gfx950 0.1"; }

const char* conqur_last_error(const conqur_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

void conqur_destroy(conqur_ctx* ctx) {
  if (!ctx) return;
  (void)hipSetDevice(ctx->cfg.device);
  (void)hipStreamSynchronize(ctx->stream);
  for (void* p : ctx->allocs) (void)hipFree(p);
  for (int s = 0; s < ST_COUNT; ++s)
    for (int k = 0; k < 2; ++k)
      if (ctx->ev[s][k]) (void)hipEventDestroy(ctx->ev[s][k]);
  if (ctx->ev_resid) (void)hipEventDestroy(ctx->ev_resid);
  if (ctx->ev_sq) (void)hipEventDestroy(ctx->ev_sq);
  if (ctx->host_res) (void)hipHostFree(ctx->host_res);
  if (ctx->host_rows) (void)hipHostFree(ctx->host_rows);
  delete ctx;
}

conqur_status conqur_init(const conqur_config* cfg, const float* R0_host, conqur_ctx** out) {
  if (!cfg || !R0_host || !out) return CONQUR_EINVAL;
  *out = nullptr;
  if (cfg->d == 0 || cfg->heads == 0 || cfg->d % cfg->heads) return CONQUR_EINVAL;
  const uint32_t dh = cfg->d / cfg->heads;
  if (dh % 16 || dh > 8192 || cfg->d > 65536) return CONQUR_EINVAL;
  if (cfg->act_dtype != CONQUR_F32 && cfg->act_dtype != CONQUR_BF16) return CONQUR_EINVAL;
  if (cfg->max_tokens == 0 || cfg->max_tokens > (1u << 22) || cfg->polar_precision > 2 || cfg->polar_verify > 1) return CONQUR_EINVAL;
  if (!(cfg->prox_lambda >= 0.0f) || !(cfg->polar_tol >= 0.0f)) return CONQUR_EINVAL;
  // the GEMM kernels address an operand's rows through 32-bit byte offsets: the transposed operands [dh][pitch]
  if ((int64_t)dh * round_up((int64_t)cfg->max_tokens, 64) >= (1ll << 30)) return CONQUR_EINVAL;
  if (cfg->act_dtype == CONQUR_F32 && (int64_t)cfg->d * cfg->max_tokens >= (1ll << 30)) return CONQUR_EINVAL;   // split planes of X
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev) return CONQUR_EHIP;
  if (hipSetDevice(cfg->device) != hipSuccess) return CONQUR_EHIP;
  {   // conqur_score_rows_static's array on this device: its address is looked up here, outside any graph capture
    float* scratch = nullptr;
    if (static_scratch_for_current_device(&scratch) != hipSuccess) return CONQUR_EHIP;
  }

  conqur_ctx* ctx = new (std::nothrow) conqur_ctx();
  if (!ctx) return CONQUR_ENOMEM;
  ctx->cfg = *cfg;
  // 9.5e-5: below the 1e-4 the update must end at, above the 8.4e-5 the orthogonality bound certifies at dh = 8192
  // (its fp32 rounding term alone is 1e-8 dh), so that the largest width does not fall back to measuring every time
  if (ctx->cfg.polar_tol == 0.0f) ctx->cfg.polar_tol = 9.5e-5f;
  if (ctx->cfg.polar_max_iters == 0) ctx->cfg.polar_max_iters = 200;
  ctx->d = (int)cfg->d; ctx->heads = (int)cfg->heads; ctx->dh = (int)dh;
  ctx->f32 = cfg->act_dtype == CONQUR_F32;
  ctx->np = ctx->f32 ? 3 : 1;
  ctx->tmax = cfg->max_tokens;
  ctx->pitch = round_up(ctx->tmax, 64);
  ctx->stream = reinterpret_cast<hipStream_t>(cfg->stream);

  const size_t blk = (size_t)ctx->heads * dh * dh;
  const size_t d = ctx->d, tmax = ctx->tmax, pitch = ctx->pitch, np = ctx->np;
  hipError_t e = hipSuccess;
  auto A = [&](hipError_t r) { if (e == hipSuccess) e = r; };
  A(dev_alloc(ctx, &ctx->R, blk));
  A(dev_alloc(ctx, &ctx->RopT, np * blk));
  A(dev_alloc(ctx, &ctx->M, blk));
  A(dev_alloc(ctx, &ctx->Xt, np * d * pitch));
  A(dev_alloc(ctx, &ctx->St, d * pitch));
  if (ctx->f32) A(dev_alloc(ctx, &ctx->Xs, 3 * tmax * d));
  A(dev_alloc(ctx, &ctx->nrm, (size_t)ctx->heads * tmax));
  A(dev_alloc(ctx, &ctx->w, (size_t)ctx->heads * tmax));
  // L, rows, skipped (fused per-head step) and the slot counters (general path) share one allocation so that one
  // fill clears the batch statistics
  ctx->stat_words = (size_t)3 * ctx->heads + (size_t)2 * kCountSlots * ctx->heads;
  A(dev_alloc(ctx, &ctx->L, ctx->stat_words));
  ctx->rows = reinterpret_cast<unsigned long long*>(ctx->L + ctx->heads);
  ctx->skipped = ctx->rows + ctx->heads;
  ctx->cnt = ctx->skipped + ctx->heads;
  // the update's scalar results share one allocation (one copy brings them to the host):
  // <R_op, M> | <R, M> | ||M||_F^2 per head, then the non-finite flag
  A(dev_alloc(ctx, &ctx->ldot, (size_t)3 * ctx->heads + 1));
  ctx->inner = ctx->ldot + ctx->heads;
  ctx->fro2 = ctx->inner + ctx->heads;
  ctx->nonfinite = reinterpret_cast<int*>(ctx->fro2 + ctx->heads);
  A(dev_alloc(ctx, &ctx->dotrm_part, (size_t)ctx->heads * dot_rm_partials((int64_t)dh * dh)));
  ctx->l_base.assign(ctx->heads, 0.0);
  ctx->h_empty.assign(ctx->heads, 1);
  ctx->h_rows.assign(ctx->heads, 0);
  A(dev_alloc(ctx, reinterpret_cast<char**>(&ctx->Y), tmax * d * (ctx->f32 ? 4 : 2)));
  A(dev_alloc(ctx, &ctx->row_sse, 2 * tmax));   // per-row SSE, then per-row energy
  ctx->row_en = ctx->row_sse + tmax;
  A(dev_alloc(ctx, &ctx->qsum, (size_t)2));
  A(dev_alloc(ctx, &ctx->PX, blk));
  for (int b = 0; b < 2; ++b) {
    A(dev_alloc(ctx, &ctx->PXn[b], 3 * blk));
    A(dev_alloc(ctx, &ctx->PXt[b], 3 * blk));
  }
  A(dev_alloc(ctx, &ctx->PW, 3 * blk));
  A(dev_alloc(ctx, &ctx->PW2, 3 * blk));
  A(dev_alloc(ctx, &ctx->resid, (size_t)kResidSlots * ctx->heads));
  ctx->resid_parts = gemm_num_partials((int)dh, (int)dh, ctx->heads, 1);   // every launch that leaves residual partials is a symmetric one
  A(dev_alloc(ctx, &ctx->resid_part, (size_t)ctx->resid_parts * ctx->heads));
  ctx->head_fused = ctx->dh == 128 && !ctx->f32;
  if (ctx->head_fused) {
    ctx->head_splits = head_step_splits(ctx->heads, ctx->tmax);
    A(dev_alloc(ctx, &ctx->Mpart, (size_t)ctx->head_splits * blk));
  }
  // One rotation of a width whose dh x dh output gives the accumulate GEMM only a few tiles (dh <= 512: at most 64 of the
  // chip's 256 compute units, each with the whole token range to itself): the token range is split into shares instead.
  if (!ctx->head_fused && ctx->heads == 1 && dh <= 512 && (blk & 1023) == 0) {
    const int tiles = gemm_num_workgroups((int)dh, (int)dh, 1);
    ctx->ksplit_max = std::max(1, std::min(16, 256 / std::max(tiles, 1)));
    if (ctx->ksplit_max > 1) A(dev_alloc(ctx, &ctx->Mpart, (size_t)ctx->ksplit_max * blk));
    else ctx->ksplit_max = 0;
  }
  A(dev_alloc(ctx, &ctx->dot_part, (size_t)ctx->heads * pack_dot_partials(ctx->dh)));
  for (int k = 0; k < 2; ++k) A(dev_alloc(ctx, &ctx->clk[k], (size_t)4 * kClkMaxWorkgroups));
  for (int s = 0; s < ST_COUNT && e == hipSuccess; ++s)
    for (int k = 0; k < 2 && e == hipSuccess; ++k) e = hipEventCreate(&ctx->ev[s][k]);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_resid, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_sq, hipEventDisableTiming);
  if (e == hipSuccess)
    e = hipHostMalloc(reinterpret_cast<void**>(&ctx->host_res), ((size_t)kResidSlots * ctx->heads + 3 * ctx->heads + 1) * sizeof(double),
                      hipHostMallocDefault);
  if (e == hipSuccess)
    e = hipHostMalloc(reinterpret_cast<void**>(&ctx->host_rows), (size_t)2 * std::min<size_t>(tmax, kHostSumRows) * sizeof(float),
                      hipHostMallocDefault);
  if (e == hipSuccess) e = hipMemcpyAsync(ctx->R, R0_host, blk * sizeof(float), hipMemcpyHostToDevice, ctx->stream);
  if (e == hipSuccess) e = launch_pack(ctx->R, ctx->heads, ctx->dh, ctx->dh, ctx->np, nullptr, ctx->RopT, (int64_t)blk, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) {
    const conqur_status st = e == hipErrorOutOfMemory ? CONQUR_ENOMEM : CONQUR_EHIP;
    conqur_destroy(ctx);
    return st;
  }
  *out = ctx;
  return CONQUR_OK;
}

conqur_status conqur_set_timing(conqur_ctx* ctx, int enable) {
  if (!ctx) return CONQUR_EINVAL;
  if (enable < 0 || enable > 2) return fail(ctx, CONQUR_EINVAL, "set_timing: level must be 0, 1 or 2");
  ctx->timing = enable;
  for (int s = 0; s < ST_COUNT; ++s) ctx->ev_valid[s] = false;
  ctx->clk_wg[0] = ctx->clk_wg[1] = 0;
  return CONQUR_OK;
}

conqur_status conqur_set_taps(conqur_ctx* ctx, int enable) {
  if (!ctx) return CONQUR_EINVAL;
  ctx->taps = enable != 0;
  return CONQUR_OK;
}

conqur_status conqur_get_timing(conqur_ctx* ctx, float* out) {
  if (!ctx || !out) return CONQUR_EINVAL;
  HIP_TRY(hipStreamSynchronize(ctx->stream));
  for (int s = 0; s < kTimingSlots; ++s) out[s] = 0.0f;
  for (int s = 0; s < ST_COUNT; ++s)
    if (ctx->ev_valid[s]) HIP_TRY(hipEventElapsedTime(&out[s], ctx->ev[s][0], ctx->ev[s][1]));
  return CONQUR_OK;
}

conqur_status conqur_get_clock_probe(conqur_ctx* ctx, float* out) {
  if (!ctx || !out) return CONQUR_EINVAL;
  HIP_TRY(hipSetDevice(ctx->cfg.device));
  HIP_TRY(hipStreamSynchronize(ctx->stream));
  for (int k = 0; k < 2; ++k) {
    float* o = out + 4 * k;
    o[0] = o[1] = o[2] = o[3] = 0.0f;
    const int n = ctx->clk_wg[k];
    if (n <= 0) continue;
    std::vector<unsigned long long> h((size_t)4 * n);
    HIP_TRY(hipMemcpy(h.data(), ctx->clk[k], h.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
    double cyc = 0, loop = 0, pro = 0, epi = 0;
    for (int i = 0; i < n; ++i) { cyc += (double)h[4 * i]; loop += (double)h[4 * i + 1]; pro += (double)h[4 * i + 2]; epi += (double)h[4 * i + 3]; }
    o[0] = loop > 0 ? (float)(100.0 * cyc / loop) : 0.0f;   // ticks are 10 ns
    o[1] = (float)(loop / n * 0.01);
    o[2] = (float)(pro / n * 0.01);
    o[3] = (float)(epi / n * 0.01);
  }
  return CONQUR_OK;
}

// Sum the pending token shares of a first batch into M (see conqur_ctx::parts_pending).
static conqur_status materialise_m(conqur_ctx* ctx) {
  if (!ctx->parts_pending) return CONQUR_OK;
  HIP_TRY(launch_head_reduce(ctx->Mpart, ctx->parts_pending, ctx->heads, ctx->M, 0, nullptr, ctx->stream));
  ctx->parts_pending = 0;
  return CONQUR_OK;
}

// The fused per-head step (heads of width 128, bf16) on the heads [head0, head0 + nheads): X holds their nheads * 128
// columns.  Every per-head buffer is addressed from head0; the token shares' partial M are packed for the range.
static conqur_status step_fused(conqur_ctx* ctx, const void* X, int64_t T, int64_t stride, int head0, int nheads) {
  hipStream_t s = ctx->stream;
  const int64_t blk = (int64_t)ctx->dh * ctx->dh;
  // as many token shares as fill the chip, within the room the partial sums were given at init
  const int room = (int)((int64_t)ctx->head_splits * ctx->heads / nheads);
  const int nsplit = std::min(room, head_step_splits(nheads, T));
  const bool full = nheads == ctx->heads;
  if (ctx->parts_pending) {   // the previous batch's shares still stand for M: sum them before Mpart is written again
    conqur_status st = materialise_m(ctx);
    if (st != CONQUR_OK) return st;
  }
  {
    StageTimer tm(ctx, ST_ROTATE);   // the fused kernel: rotate + normalise + corner + accumulate
    HIP_TRY(launch_head_step128(reinterpret_cast<const bf16_bits*>(X), T, stride, nheads, ctx->RopT + head0 * blk, ctx->Mpart, nsplit,
                                ctx->nrm + (int64_t)head0 * ctx->tmax, ctx->tmax, ctx->L + head0, ctx->rows + head0,
                                ctx->skipped + head0, ctx->nonfinite,
                                ctx->taps ? ctx->St + (int64_t)head0 * ctx->dh * ctx->pitch : nullptr, ctx->pitch, s));
  }
  // M of the range: overwritten if none of its heads holds rows, added to if all do; a mixed range is cleared where empty
  int n_empty = 0;
  for (int h = head0; h < head0 + nheads; ++h) n_empty += ctx->h_empty[h];
  if (n_empty != 0 && n_empty != nheads)
    for (int h = head0; h < head0 + nheads; ++h)
      if (ctx->h_empty[h]) HIP_TRY(launch_fill_zero(ctx->M + h * blk, blk * sizeof(float), s));
  if (full && n_empty == nheads) {
    // First batch since the update, all heads: the shares are left where they are.  Whoever needs M next sums them --
    // normally the update, in the pass that also yields ||M||_F -- so a step that is followed by its update (Alg. 1)
    // costs one launch and one round trip of M less.
    ctx->parts_pending = nsplit;
    ctx->ev_valid[ST_ACCUM] = false;
  } else {
    StageTimer tm(ctx, ST_ACCUM);    // the token shares' partial M, summed in a fixed order
    HIP_TRY(launch_head_reduce(ctx->Mpart, nsplit, nheads, ctx->M + head0 * blk, n_empty == nheads ? 0 : 1, nullptr, s));
  }
  for (int h = head0; h < head0 + nheads; ++h) { ctx->h_empty[h] = 0; ctx->h_rows[h] = 1; }
  ctx->clk_wg[0] = ctx->clk_wg[1] = 0;
  ctx->last_signs_valid = ctx->taps && full;   // the corner tap returns whole rows of width d
  ctx->m_empty = false;
  ctx->have_rows = true;
  ctx->last_T = full ? T : 0;
  return CONQUR_OK;
}

conqur_status conqur_step_batch_heads(conqur_ctx* ctx, const void* X, uint64_t T64, uint64_t stride64, uint32_t head0,
                                      uint32_t nheads) {
  if (!ctx) return CONQUR_EINVAL;
  if (nheads < 1 || (uint64_t)head0 + nheads > (uint64_t)ctx->heads) return fail(ctx, CONQUR_EINVAL, "head range outside [0, heads)");
  if (head0 == 0 && nheads == (uint32_t)ctx->heads) return conqur_step_batch(ctx, X, T64, stride64);
  if (!ctx->head_fused)
    return fail(ctx, CONQUR_EINVAL, "a partial head range needs heads of width 128 and bf16 activations");
  if (!X) return fail(ctx, CONQUR_EINVAL, "X_dev is NULL");
  if (T64 < 1 || (int64_t)T64 > ctx->tmax) return fail(ctx, CONQUR_EINVAL, "T must be in [1, max_tokens]");
  if (stride64 < (uint64_t)nheads * ctx->dh) return fail(ctx, CONQUR_EINVAL, "row_stride_elems < nheads * dh");
  if ((reinterpret_cast<uintptr_t>(X) & 15) || ((stride64 * 2) & 15))
    return fail(ctx, CONQUR_EINVAL, "X_dev base and row pitch must be 16-byte aligned");
  HIP_TRY(hipSetDevice(ctx->cfg.device));
  StageTimer whole(ctx, ST_STEP, 1);
  return step_fused(ctx, X, (int64_t)T64, (int64_t)stride64, (int)head0, (int)nheads);
}

// The statistics step of the general path (any head width, both activation dtypes).  keep_y: the rotate GEMM also
// stores the rotated rows Y = X R_op into ctx->Y (activation dtype), for a quantiser that follows in the same call.
static conqur_status step_general(conqur_ctx* ctx, const void* X, int64_t T, int64_t stride, bool keep_y) {
  const int64_t Tk = round_up(T, 64);
  hipStream_t s = ctx->stream;
  ctx->last_signs_valid = true;
  // bf16 activations: the scaled transposed operand of the accumulate GEMM is produced by the rotate GEMM's epilogue
  // (every workgroup transposes the block of X under its output block through the LDS staging of the signs), which
  // saves the transposing launch; fp32 activations (split planes) and the variant that also emits Y keep that launch.
  const bool xt_in_gemm = !ctx->f32 && !keep_y;
  {
    StageTimer tm(ctx, ST_PREP);
    HIP_TRY(launch_row_norms(X, ctx->f32, T, stride, ctx->heads, ctx->dh, ctx->nrm, ctx->w, ctx->tmax, ctx->nonfinite, s));
    if (!xt_in_gemm)
      HIP_TRY(launch_transpose_scale(X, ctx->f32, T, Tk, stride, ctx->d, ctx->dh, ctx->w, ctx->tmax, ctx->Xt, ctx->pitch,
                                     (int64_t)ctx->d * ctx->pitch, ctx->np, ctx->cnt, s));
    if (ctx->f32)
      HIP_TRY(launch_split_rows(reinterpret_cast<const float*>(X), T, stride, ctx->d, ctx->Xs, ctx->tmax * ctx->d, s));
  }
  {
    StageTimer tm(ctx, ST_ROTATE);
    GemmArgs g;
    rotate_args(ctx, X, T, stride, &g);
    g.C = ctx->St; g.ldc = ctx->pitch; g.batchC = (int64_t)ctx->dh * ctx->pitch;
    g.st_rows_valid = ctx->pitch;
    g.sign_f16 = ctx->f32 ? 0 : 1;   // the accumulate GEMM runs in fp16 for bf16 activations
    const int wg = gemm_num_workgroups(g.M, g.N, ctx->heads);
    ctx->clk_wg[0] = (ctx->timing >= 2 && wg <= kClkMaxWorkgroups) ? wg : 0;
    g.clk = ctx->clk_wg[0] ? ctx->clk[0] : nullptr;
    if (keep_y) { g.Yact = ctx->Y; g.ldy = ctx->d; g.batchY = ctx->dh; g.c_is_f32 = ctx->f32; }
    if (xt_in_gemm) {
      g.xt_w = ctx->w; g.xt_ldw = ctx->tmax; g.Xt = ctx->Xt; g.cnt = ctx->cnt; g.cnt_slots = kCountSlots;
    }
    HIP_TRY(launch_gemm_nt(g, keep_y ? EPI_SIGN_ACT : (xt_in_gemm ? EPI_SIGN_XT : EPI_SIGN), ctx->heads, s));
  }
  {
    StageTimer tm(ctx, ST_ACCUM);
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    g.A = ctx->Xt; g.lda = ctx->pitch; g.batchA = (int64_t)ctx->dh * ctx->pitch;
    g.B = ctx->St; g.ldb = ctx->pitch; g.batchB = (int64_t)ctx->dh * ctx->pitch;
    g.M = ctx->dh; g.N = ctx->dh; g.K = (int)Tk;
    const SegList& sl = ctx->f32 ? kSeg3x1 : kSeg1;
    g.nseg = sl.n;
    for (int q = 0; q < sl.n; ++q) { g.a_seg[q] = sl.a[q] * (int64_t)ctx->d * ctx->pitch; g.b_seg[q] = 0; }
    g.C = ctx->M; g.ldc = ctx->dh; g.batchC = (int64_t)ctx->dh * ctx->dh;
    g.accumulate = ctx->m_empty ? 0 : 1;
    g.out_scale = 1.0f / (kXhatScale * std::sqrt((float)ctx->dh));   // the operand carries kXhatScale x^, the corner 1/sqrt(dh)
    g.ab_f16 = ctx->f32 ? 0 : 1;
    // shares of the token range: the largest count up to ksplit_max that divides the range into whole 64-token steps
    int shares = 1;
    for (int c = ctx->ksplit_max; c > 1; --c)
      if ((Tk / 64) % c == 0) { shares = c; break; }
    if (shares > 1) {
      // every share is a batch entry: the operands advance along the tokens, the results go to the shares of Mpart
      g.K = (int)(Tk / shares);
      g.batchA = g.K; g.batchB = g.K;
      g.C = ctx->Mpart; g.accumulate = 0;
      ctx->clk_wg[1] = 0;
      HIP_TRY(launch_gemm_nt(g, EPI_F32, shares, s));
      HIP_TRY(launch_sum_shares(ctx->Mpart, shares, (int64_t)ctx->dh * ctx->dh, ctx->M, ctx->m_empty ? 0 : 1, s));
    } else {
      const int wg = gemm_num_workgroups(g.M, g.N, ctx->heads);
      ctx->clk_wg[1] = (ctx->timing >= 2 && wg <= kClkMaxWorkgroups) ? wg : 0;
      g.clk = ctx->clk_wg[1] ? ctx->clk[1] : nullptr;
      HIP_TRY(launch_gemm_nt(g, EPI_F32, ctx->heads, s));
    }
  }
  // no statistics kernel: the row counters were taken with the norms, and the l1 term of the accumulated rows is
  // sqrt(dh) <R_op, M> (k_dot_rm), evaluated when asked for and at the start of the update.
  ctx->m_empty = false;
  ctx->have_rows = true;
  ctx->last_T = T;
  return CONQUR_OK;
}

conqur_status conqur_step_batch(conqur_ctx* ctx, const void* X, uint64_t T64, uint64_t stride64) {
  conqur_status st = check_x(ctx, X, T64, stride64);
  if (st != CONQUR_OK) return st;
  HIP_TRY(hipSetDevice(ctx->cfg.device));
  StageTimer whole(ctx, ST_STEP, 1);   // ends when the function returns
  if (ctx->head_fused) return step_fused(ctx, X, (int64_t)T64, (int64_t)stride64, 0, ctx->heads);
  return step_general(ctx, X, (int64_t)T64, (int64_t)stride64, false);
}

conqur_status conqur_step_batch_quant(conqur_ctx* ctx, const void* X, uint64_t T64, uint64_t stride64, uint32_t bits,
                                      uint32_t zero_point, float clip_ratio, void* Yq, uint64_t yq_stride64) {
  conqur_status st = check_x(ctx, X, T64, stride64);
  if (st != CONQUR_OK) return st;
  if (bits < 2 || bits > 8) return fail(ctx, CONQUR_EINVAL, "bits must be in [2, 8]");
  if (zero_point > 1) return fail(ctx, CONQUR_EINVAL, "zero_point must be 0 or 1");
  if (zero_point && (!(clip_ratio > 0.0f) || clip_ratio > 1.0f)) return fail(ctx, CONQUR_EINVAL, "clip_ratio must be in (0, 1]");
  if (!Yq) return fail(ctx, CONQUR_EINVAL, "Yq_dev is NULL");
  if (yq_stride64 < (uint64_t)ctx->d || yq_stride64 >= (1ull << 40) || (reinterpret_cast<uintptr_t>(Yq) % 16) != 0 ||
      (yq_stride64 * (ctx->f32 ? 4 : 2)) % 16 != 0)
    return fail(ctx, CONQUR_EINVAL, "Yq row stride must be >= d and Yq and its rows aligned to 16 bytes");
  HIP_TRY(hipSetDevice(ctx->cfg.device));
  const int64_t T = (int64_t)T64, stride = (int64_t)stride64;
  hipStream_t s = ctx->stream;
  {
    StageTimer whole(ctx, ST_STEP, 1);
    if (ctx->head_fused) {
      // heads of width 128: the fused step kernel keeps Y on the compute unit; the rows are rotated once more for the quantiser
      st = step_fused(ctx, X, T, stride, 0, ctx->heads);
      if (st != CONQUR_OK) return st;
      GemmArgs g;
      rotate_args(ctx, X, T, stride, &g);
      g.C = ctx->Y; g.ldc = ctx->d; g.batchC = ctx->dh; g.c_is_f32 = ctx->f32;
      HIP_TRY(launch_gemm_nt(g, EPI_ACT, ctx->heads, s));
    } else {
      st = step_general(ctx, X, T, stride, true);   // one rotate GEMM: corner signs and Y
      if (st != CONQUR_OK) return st;
    }
  }
  StageTimer tm(ctx, ST_QERR);
  HIP_TRY(launch_quant_error(ctx->Y, ctx->f32, T, ctx->d, ctx->d, (int)bits, (int)zero_point, clip_ratio, ctx->row_sse,
                             ctx->row_en, nullptr, Yq, (int64_t)yq_stride64, s));
  return CONQUR_OK;
}

// Host copy of the batch statistics; for the general path the l1 term is evaluated here from M (see k_dot_rm).
static conqur_status read_stats(conqur_ctx* ctx, std::vector<double>* L, std::vector<unsigned long long>* rows,
                                std::vector<unsigned long long>* skipped) {
  const int h = ctx->heads;
  hipStream_t s = ctx->stream;
  std::vector<double> buf(ctx->stat_words);
  std::vector<double> ldot(h, 0.0);
  if (!ctx->head_fused && !ctx->m_empty) {
    HIP_TRY(launch_dot_rm(ctx->R, ctx->M, h, (int64_t)ctx->dh * ctx->dh, ctx->f32 ? 0 : 1, ctx->dotrm_part, ctx->ldot, s));
    HIP_TRY(hipMemcpyAsync(ldot.data(), ctx->ldot, h * sizeof(double), hipMemcpyDeviceToHost, s));
  }
  HIP_TRY(hipMemcpyAsync(buf.data(), ctx->L, ctx->stat_words * sizeof(double), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  const unsigned long long* u = reinterpret_cast<const unsigned long long*>(buf.data());
  L->assign(h, 0.0); rows->assign(h, 0); skipped->assign(h, 0);
  for (int i = 0; i < h; ++i) {
    (*L)[i] = ctx->head_fused ? buf[i] : ctx->l_base[i] + std::sqrt((double)ctx->dh) * ldot[i];
    (*rows)[i] = u[h + i];
    (*skipped)[i] = u[2 * h + i];
    for (int q = 0; q < kCountSlots; ++q) {
      (*rows)[i] += u[3 * h + ((size_t)i * kCountSlots + q) * 2];
      (*skipped)[i] += u[3 * h + ((size_t)i * kCountSlots + q) * 2 + 1];
    }
  }
  return CONQUR_OK;
}

conqur_status conqur_get_batch_stats(conqur_ctx* ctx, conqur_batch_stats* out) {
  if (!ctx || !out) return CONQUR_EINVAL;
  HIP_TRY(hipSetDevice(ctx->cfg.device));
  std::vector<double> L;
  std::vector<unsigned long long> rows, skipped;
  const conqur_status st = read_stats(ctx, &L, &rows, &skipped);
  if (st != CONQUR_OK) return st;
  for (int i = 0; i < ctx->heads; ++i) {
    out[i].rows = rows[i]; out[i].skipped = skipped[i]; out[i].l1 = L[i];
    out[i].objective = 2.0 * (double)rows[i] - 2.0 * L[i] / std::sqrt((double)ctx->dh);   // the l1 identity of Sec. 3.2
  }
  return CONQUR_OK;
}

// One step polynomial p(x) = a x + b x^3 for singular values in [l, u].
// Shape: f(x) = 1.5 (x/q) - 0.5 (x/q)^3, which peaks (value 1) at x = q.  The
// equal-ripple choice (f(l) = f(u), q^2 = (u^2 + u l + l^2)/3) grows small values
// fastest, but for l << u it sends the LARGEST singular values to the bottom of the
// range, where low-precision rounding then perturbs exactly the directions that
// carry the Procrustes objective.  So q is kept >= u / 1.65, which bounds
// f(u) >= 0.23: the leading directions never fall below a quarter of the current
// maximum (growth of small values 2.48 instead of 2.60 per step; with the bound at
// 1.532, f(u) >= 0.5, one more step was needed at d >= 2048 for an objective that was
// no closer to the optimum, while the unbounded choice loses a factor 2-5 in the
// objective's deficit).  Scaled so that the image of [l, u] is [1 - E, 1 + E];
// returns E.  For l = u = 1: the Newton-Schulz step.
static double step_cubic(double l, double u, double* a, double* b) {
  const double s = u * u + u * l + l * l;
  const double t = std::min(u * std::sqrt(3.0 / s), 1.65);
  const double q = u / t;
  auto f = [q](double x) { return 1.5 * (x / q) - 0.5 * (x / q) * (x / q) * (x / q); };
  const double lo = std::min(f(l), f(u));
  const double c = 2.0 / (1.0 + lo);
  *a = c * 1.5 / q;
  *b = -c * 0.5 / (q * q * q);
  return (1.0 - lo) / (1.0 + lo);
}

conqur_status conqur_update_rotation(conqur_ctx* ctx, conqur_update_stats* out) {
  if (!ctx) return CONQUR_EINVAL;
  if (!ctx->have_rows) return fail(ctx, CONQUR_ESTATE, "update_rotation: no rows accumulated since the last update");
  for (int q = 0; q < ctx->heads; ++q)
    if (ctx->head_fused && !ctx->h_rows[q])
      return fail(ctx, CONQUR_ESTATE, "update_rotation: a head range has no rows since the last update");
  HIP_TRY(hipSetDevice(ctx->cfg.device));
  hipStream_t s = ctx->stream;
  const int h = ctx->heads, dh = ctx->dh;
  const int64_t blk = (int64_t)dh * dh, plane = (int64_t)h * blk;
  const bool timed = ctx->timing || out;
  const bool trace = std::getenv("CONQUR_TRACE") != nullptr;
  if (timed) HIP_TRY(hipEventRecord(ctx->ev[ST_UPDATE][0], s));

  const int np_main = 1 + (int)ctx->cfg.polar_precision;
  // Heads of width 128 on the fused path: the launch that runs the main phase also forms the start iterate (and, below,
  // takes the closing step), so the update is the reduction of the token shares and that one launch.
  HeadPolarStart hstart;
  bool use_hstart = ctx->head_fused && dh == 128 && np_main == 1 && ctx->cfg.polar_max_iters > 0;
  if (ctx->parts_pending) {   // per-head step: M is summed from the token shares here, ||M||_F^2 from the same pass
    HIP_TRY(launch_head_reduce(ctx->Mpart, ctx->parts_pending, h, ctx->M, 0, ctx->dotrm_part, s));
    if (use_hstart) { hstart.fro2_parts = ctx->dotrm_part; hstart.nparts = kHeadReduceParts; }
    else HIP_TRY(launch_sum_partials(ctx->dotrm_part, kHeadReduceParts, h, ctx->fro2, s));
    ctx->parts_pending = 0;
  } else {
    HIP_TRY(launch_fro2(ctx->M, h, blk, ctx->dotrm_part, ctx->fro2, s));
    if (use_hstart) { hstart.fro2_parts = ctx->fro2; hstart.nparts = 1; }
  }
  if (use_hstart) {
    hstart.M = ctx->M; hstart.R = ctx->R; hstart.fro2_out = ctx->fro2; hstart.lambda = ctx->cfg.prox_lambda;
    hstart.L = ctx->L; hstart.ldot = ctx->ldot;
  }

  // Single-plane main steps run on fp16 operands (iterate and polynomial factor): the MFMA rate of bf16 with 11
  // instead of 8 significant bits, so that the rounding of a step, which the weak singular directions amplify by
  // 1/sigma, is 8 times smaller.  Every entry is at most a few units in magnitude: no range problem.  The
  // hand-over to the closing steps and the split-plane modes stay bf16 (their planes sum exactly).
  const int main_f16 = np_main == 1 ? 1 : 0;
  const SegList& seg_main = np_main == 1 ? kSeg1 : (np_main == 2 ? kSeg3 : kSeg6);
  const uint32_t cap = ctx->cfg.polar_max_iters;
  const double tol = ctx->cfg.polar_tol;
  int cur = 0;            // which ping-pong plane buffer holds the iterate
  // X0 = (M + lambda tau R) / alpha, alpha = ||M||_F (1 + lambda) >= ||X0||_2, written straight as the operand
  // planes of the first step (no fp32 copy: at least one main step runs, and the last one writes the fp32 iterate)
  // The same pass evaluates the l1 term of the rows this update consumes (general path; the fused per-head step
  // keeps it as it goes): a copy of either is taken here, before the statistics are cleared.
  if (!use_hstart) {
    HIP_TRY(launch_polar_start_pack(ctx->M, ctx->R, h, dh, ctx->cfg.prox_lambda, ctx->fro2, np_main, nullptr,
                                    ctx->PXn[cur], ctx->PXt[cur], plane, ctx->f32 ? 0 : 1,
                                    ctx->head_fused ? nullptr : ctx->dot_part, ctx->ldot, s, main_f16));
    if (ctx->head_fused) HIP_TRY(hipMemcpyAsync(ctx->ldot, ctx->L, h * sizeof(double), hipMemcpyDeviceToDevice, s));
  }
  int slot = 0;           // next residual-history slot
  uint32_t iters = 0, closing = 0;
  double mfma_flop = 0.0; // multiply-add work the products of this update issue (reported in the statistics)

  auto gram = [&](const SegList& sl, float ci, float cg, int np_w, bool want_resid, int f16 = 0) -> hipError_t {
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    g.ab_f16 = f16;
    g.A = ctx->PXt[cur]; g.B = ctx->PXt[cur]; g.lda = g.ldb = dh; g.batchA = g.batchB = blk;
    g.M = g.N = g.K = dh;
    g.nseg = sl.n;
    for (int q = 0; q < sl.n; ++q) { g.a_seg[q] = sl.a[q] * plane; g.b_seg[q] = sl.b[q] * plane; }
    g.ldc = dh; g.batchC = blk; g.Pn = ctx->PW; g.np_out = np_w; g.plane_out = plane;
    g.symmetric = 1;   // X^T X: tiles above the diagonal are computed once and stored twice
    g.resid_part = want_resid ? ctx->resid_part : nullptr; g.coef_i = ci; g.coef_g = cg;
    hipError_t e = launch_gemm_nt(g, EPI_GRAMW, h, s);
    mfma_flop += gemm_issued_flop(g, EPI_GRAMW, h);
    if (e == hipSuccess && want_resid)
      e = launch_sum_partials(ctx->resid_part, ctx->resid_parts, h, ctx->resid + (size_t)slot * h, s);
    return e;
  };
  // X' = X W (+ X): reads the planes in buffer `cur`, writes np_x planes (both layouts)
  // into the other buffer, and the fp32 iterate when asked.
  // np_t < 0: the hand-over form -- the result rounded to -np_t planes, that value in PX and in as many planes of each layout.
  auto apply = [&](const SegList& sl, const bf16_bits* W, int np_t, int np_n, bool add_x, float* out32, int f16 = 0) -> hipError_t {
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    g.ab_f16 = f16;
    g.A = ctx->PXn[cur]; g.B = W; g.lda = g.ldb = dh; g.batchA = g.batchB = blk;
    g.M = g.N = g.K = dh;
    g.nseg = sl.n;
    for (int q = 0; q < sl.n; ++q) { g.a_seg[q] = sl.a[q] * plane; g.b_seg[q] = sl.b[q] * plane; }
    g.ldc = dh; g.batchC = blk; g.plane_out = plane;
    g.Pn = ctx->PXn[cur ^ 1]; g.Pt = ctx->PXt[cur ^ 1];
    hipError_t e;
    if (np_t < 0) {
      g.C32 = ctx->PX;
      g.np_out = -np_t;
      e = launch_gemm_nt(g, EPI_XLAST, h, s);
      mfma_flop += gemm_issued_flop(g, EPI_XLAST, h);
    } else {
      g.np_out = np_t; g.np_out_n = np_n;
      g.Xadd = add_x ? ctx->PX : nullptr;
      g.C32 = out32;
      e = launch_gemm_nt(g, EPI_XOUT, h, s);
      mfma_flop += gemm_issued_flop(g, EPI_XOUT, h);
    }
    cur ^= 1;
    return e;
  };
  // W2 = D + 1.5 D^2 from the planes of D = (I - G)/2 in PW (D is symmetric, so D D^T = D^2)
  // keep_square: D^2 itself is kept as a plane and ||D^2||_F^2 goes to residual slot `slot` (copied to the host behind
  // ev_sq): both serve the orthogonality bounds of the step that applies this correction.
  int sq_slot = -1;
  auto square_correction = [&](bool keep_square) -> hipError_t {
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    g.A = ctx->PW; g.B = ctx->PW; g.lda = g.ldb = dh; g.batchA = g.batchB = blk;
    g.M = g.N = g.K = dh;
    g.nseg = 1;   // D^2 is second order small: single bf16 planes are ample
    g.ldc = dh; g.batchC = blk; g.Pn = ctx->PW2; g.np_out = 2; g.plane_out = plane;
    g.Padd = ctx->PW; g.np_add = 2; g.coef_i = 0.0f; g.coef_g = 1.5f;
    g.symmetric = 1;
    sq_slot = -1;
    mfma_flop += gemm_issued_flop(g, EPI_SQUARE, h);
    if (!keep_square) return launch_gemm_nt(g, EPI_GRAMW, h, s);
    g.Pacc = ctx->PW2 + 2 * plane;   // D^2 itself, third plane of the buffer
    g.resid_part = ctx->resid_part;
    hipError_t e = launch_gemm_nt(g, EPI_SQUARE, h, s);
    if (e == hipSuccess) e = launch_sum_partials(ctx->resid_part, ctx->resid_parts, h, ctx->resid + (size_t)slot * h, s);
    if (e == hipSuccess)
      e = hipMemcpyAsync(ctx->host_res + (size_t)slot * h, ctx->resid + (size_t)slot * h, h * sizeof(double), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipEventRecord(ctx->ev_sq, s);
    if (e == hipSuccess) sq_slot = slot++;
    return e;
  };
  // ||D^3||_F^2 (into residual slot `slot`) from the planes of D and D^2: the quintic step leaves the residual
  // I - X'^T X' = 5 D^3 + 3.75 D^4 + 4.5 D^5 (both sides polynomials in D), so this norm predicts it.
  auto cube_norm = [&]() -> hipError_t {
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    g.A = ctx->PW; g.B = ctx->PW2 + 2 * plane; g.lda = g.ldb = dh; g.batchA = g.batchB = blk;
    g.M = g.N = g.K = dh;
    g.nseg = 1;
    g.ldc = dh; g.batchC = blk; g.plane_out = plane;
    g.symmetric = 1;   // D and D^2 commute: D^3 is symmetric (up to the planes' rounding, which this estimate absorbs)
    g.resid_part = ctx->resid_part;
    hipError_t e = launch_gemm_nt(g, EPI_FRO2, h, s);
    mfma_flop += gemm_issued_flop(g, EPI_FRO2, h);
    if (e == hipSuccess) e = launch_sum_partials(ctx->resid_part, ctx->resid_parts, h, ctx->resid + (size_t)slot * h, s);
    return e;
  };
  double* const hist = ctx->host_res;   // pinned, so that the copies below are asynchronous
  // The copy of residual slot sl_idx and an event behind it; work enqueued after this does not delay the host's read.
  auto post_resid = [&](int sl_idx) -> conqur_status {
    HIP_TRY(hipMemcpyAsync(hist + (size_t)sl_idx * h, ctx->resid + (size_t)sl_idx * h, h * sizeof(double), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipEventRecord(ctx->ev_resid, s));
    return CONQUR_OK;
  };
  auto wait_resid = [&](int sl_idx, double* worst) -> conqur_status {
    HIP_TRY(hipEventSynchronize(ctx->ev_resid));
    double w = 0.0;
    for (int q = 0; q < h; ++q) w = std::max(w, std::sqrt(hist[(size_t)sl_idx * h + q]));
    *worst = w;
    return CONQUR_OK;
  };

  // ---- main phase: composed cubics X <- X (a I + b X^T X) (see step_cubic), no host round trips.
  // The singular values of X0 lie in [l, 1]; l is the value the proximal term guarantees
  // on the null space of M, halved.  (Smaller ones still grow by the factor a > 2.5 per
  // step and are finished by the closing iterations.)
  int handover_planes = 0;   // 1 / 2: the iterate in PX is exactly the sum of that many planes of buffer `cur`; 0: all three
  bool allow_fuse = true;    // (only the first main phase of an update: not the one after a nudge)
  int fused_slot = -1;       // heads of width 128: the launch of the main phase also took the closing step (per head, if
                             // its residual allowed); residual slots fused_slot (||I - G||_F^2) and fused_slot + 1 (||D^2||_F^2)
  auto main_phase = [&](double l0, bool planes_ready) -> conqur_status {
    if (!planes_ready) HIP_TRY(launch_pack(ctx->PX, h, dh, dh, np_main, ctx->PXn[cur], ctx->PXt[cur], plane, s, main_f16));
    const double e_stop = np_main == 1 ? 4e-3 : 5e-4;   // the safety margins below floor the ripple near 2e-4
    double l = l0, u = 1.0;
    if (dh == 128 && np_main == 1 && iters < cap) {
      // heads of width 128: the whole schedule in one launch, the iterate stays in LDS (head_polar.hip)
      PolarSchedule sc;
      sc.nsteps = 0;
      while (sc.nsteps < kPolarScheduleMax) {
        double a, b;
        const double E = step_cubic(l, u, &a, &b);
        sc.a[sc.nsteps] = (float)a;
        sc.b[sc.nsteps] = (float)b;
        ++sc.nsteps;
        if (E <= e_stop || iters + sc.nsteps >= cap) break;
        l = 0.98 * (1.0 - E);
        u = 1.01 * (1.0 + E);
      }
      // With the bound instead of a measurement at the end (the default) the closing step rides in the same launch:
      // every head whose residual allows the quintic form takes it and leaves R, the rotate operand and <R, M>.
      HeadPolarClose hc;
      const bool fuse = allow_fuse && !ctx->cfg.polar_verify && iters + sc.nsteps + 1 <= cap && slot + 2 < kResidSlots - 8;
      if (fuse) {
        hc.R = ctx->R; hc.RopT = ctx->RopT; hc.M = ctx->M;
        hc.res_out = ctx->resid + (size_t)slot * h; hc.sq_out = ctx->resid + (size_t)(slot + 1) * h; hc.inner_out = ctx->inner;
        hc.res_max = (float)(1e-2 * std::sqrt((double)dh));
        fused_slot = slot;
        slot += 2;
      } else {
        fused_slot = -1;
      }
      HIP_TRY(launch_head_polar128(ctx->PXn[cur], ctx->PXt[cur], h, sc, ctx->PX, ctx->PXn[cur ^ 1], ctx->PXt[cur ^ 1],
                                   fuse ? &hc : nullptr, (use_hstart && planes_ready) ? &hstart : nullptr, s));
      use_hstart = false;
      cur ^= 1;
      handover_planes = 1;
      iters += sc.nsteps;
      // per head: two 128^3 products per step, a third in the last one, and four in the closing step if it is taken
      mfma_flop += 2.0 * 128.0 * 128.0 * 128.0 * h * (2.0 * sc.nsteps + 1.0 + (fuse ? 4.0 : 0.0));
      if (trace) std::fprintf(stderr, "[conqur] polar main phase: %d steps in one launch, l0=%.3e\n", sc.nsteps, l0);
      return CONQUR_OK;
    }
    for (int k = 0; k < 64 && iters < cap && slot < kResidSlots - 8; ++k) {
      double a, b;
      const double E = step_cubic(l, u, &a, &b);
      const bool last = E <= e_stop || iters + 1 >= cap;
      HIP_TRY(gram(seg_main, (float)a, (float)b, np_main, trace, main_f16));
      ++slot;
      // The last main step hands over to the closing iterations.  Its result is rounded to the planes this phase
      // works with anyway (one: 8 bits, two: 16 bits -- a perturbation of the size every step of this phase
      // leaves), and exactly that value is held as fp32 and as planes of each layout: the closing Gram matrix
      // X^T X is then exact with 1 (4) plane products and the correction product reads an exact left operand.
      // (Three-plane main steps keep all 24 bits: their accuracy is below any such rounding.)
      if (last && np_main == 3) {
        HIP_TRY(apply(seg_main, ctx->PW, 3, 2, false, ctx->PX));
      } else {
        HIP_TRY(apply(seg_main, ctx->PW, last ? -np_main : np_main, last ? -np_main : np_main, false, nullptr, main_f16));
        if (last) handover_planes = np_main;
      }
      ++iters;
      if (trace) std::fprintf(stderr, "[conqur] polar main step %d: [l,u]=[%.3e,%.3f] a=%.4f b=%.4f ripple=%.3e planes=%d\n", k, l, u, a, b, E, np_main);
      if (last) break;
      l = 0.98 * (1.0 - E);   // safety margins against rounding
      u = 1.01 * (1.0 + E);
    }
    return CONQUR_OK;
  };
  const double lam_eff = std::max((double)ctx->cfg.prox_lambda, 9.5367431640625e-07);
  conqur_status st = main_phase(0.5 * lam_eff / ((1.0 + lam_eff) * std::sqrt((double)dh)), true);
  if (st != CONQUR_OK) return st;
  allow_fuse = false;

  // ---- closing iterations, Gram matrix in fp32-equivalent arithmetic (3 planes, 6 products).
  // With D = (I - X^T X)/2 the Newton-Schulz steps are X <- X + X D (cubic) and
  // X <- X + X (D + 1.5 D^2) (quintic, error e -> O(e^3): one step takes the bf16 floor of the
  // main phase to the fp32 floor).  The correction is small, so two planes per operand
  // suffice for the product; the fp32 iterate is added in the epilogue.
  bool converged = false, predicted = false;
  int kicks = 0;
  double res = 0.0;
  int last_slot = 0;
  const float* final_x = ctx->PX;   // where the final iterate lives (the lean closing step writes R directly)
  const bool keep_sq = !ctx->cfg.polar_verify || trace;
  bool finished = false;
  auto enqueue_finish = [&]() -> conqur_status {
    // R = final iterate (unless it is there already), <R, M>, and the rotate operand planes of R^T: one pass
    HIP_TRY(launch_polar_finish_pack(final_x, ctx->M, h, dh, ctx->np, final_x == ctx->R ? nullptr : ctx->R, ctx->RopT, plane,
                                     ctx->dot_part, ctx->inner, s));
    // statistics restart empty (Alg. 1): M is overwritten by the next accumulate
    HIP_TRY(launch_fill_zero(ctx->L, ctx->stat_words * sizeof(double), s));
    if (timed) HIP_TRY(hipEventRecord(ctx->ev[ST_UPDATE][1], s));
    return CONQUR_OK;
  };
  // Outcome of a closing step taken inside the main phase's launch (heads of width 128): accepted if every head took it
  // and the bound from ||D^2||_F (see below) is within the tolerance; otherwise the general closing steps continue from
  // the hand-over state, which that launch wrote as well.  (R of the heads that did take the step is overwritten already:
  // should the rare nudge below follow, it moves those heads towards their new rotation instead of the previous one.)
  auto fused_outcome = [&]() -> conqur_status {
    HIP_TRY(hipMemcpyAsync(hist + (size_t)fused_slot * h, ctx->resid + (size_t)fused_slot * h, 2 * h * sizeof(double),
                           hipMemcpyDeviceToHost, s));
    HIP_TRY(hipEventRecord(ctx->ev_resid, s));
    // expected to be the end: what follows the last step goes in before the host waits
    HIP_TRY(launch_fill_zero(ctx->L, ctx->stat_words * sizeof(double), s));
    if (timed) HIP_TRY(hipEventRecord(ctx->ev[ST_UPDATE][1], s));
    HIP_TRY(hipEventSynchronize(ctx->ev_resid));
    bool ok = true;
    double worst_res = 0.0, worst_pred = 0.0;
    for (int q = 0; q < h; ++q) {
      const double r2 = hist[(size_t)fused_slot * h + q], s2 = hist[(size_t)(fused_slot + 1) * h + q];
      if (!std::isfinite(r2)) return fail(ctx, CONQUR_ENONFINITE, "update_rotation: non-finite polar iterate");
      worst_res = std::max(worst_res, std::sqrt(r2));
      if (!(s2 >= 0.0)) { ok = false; continue; }
      const double b = kCubeFactor * std::pow(std::sqrt(s2), 1.5) + kOrthFloorPerDim * dh;
      worst_pred = std::max(worst_pred, b);
      if (!(std::isfinite(b) && b <= tol)) ok = false;
    }
    if (trace) std::fprintf(stderr, "[conqur] polar closing in the main phase's launch: resid_F=%.6e bound on resid_F=%.4e accepted=%d\n",
                            worst_res, worst_pred, (int)ok);
    if (!ok) { fused_slot = -1; return CONQUR_OK; }
    for (int q = 0; q < h; ++q) {
      const double b = kCubeFactor * std::pow(std::sqrt(hist[(size_t)(fused_slot + 1) * h + q]), 1.5) + kOrthFloorPerDim * dh;
      hist[(size_t)(fused_slot + 1) * h + q] = b * b;
    }
    last_slot = fused_slot + 1;
    ++iters; ++closing;
    converged = predicted = finished = true;
    final_x = ctx->R;
    return CONQUR_OK;
  };
  if (fused_slot >= 0) {
    st = fused_outcome();
    if (st != CONQUR_OK) return st;
  }
  while (!converged) {
    HIP_TRY(gram(handover_planes == 1 ? kSeg1 : (handover_planes == 2 ? kSeg4 : kSeg6), 0.5f, -0.5f, 2, true));
    const SegList& seg_corr = handover_planes == 1 ? kSeg2 : kSeg3;   // the correction product X (D + 1.5 D^2)
    handover_planes = 0;   // whatever follows (correction step, nudge) writes all three planes again
    last_slot = slot++;
    // The first check after a main phase practically always calls for the quintic step: enqueue its D^2 product
    // before the host waits for the residual, so that the device keeps working through the round trip.
    const bool spec_square = closing == 0;
    st = post_resid(last_slot);   // before the D^2 product, so that the host reads the residual while that runs
    if (st != CONQUR_OK) return st;
    if (spec_square) HIP_TRY(square_correction(keep_sq));
    st = wait_resid(last_slot, &res);
    if (st != CONQUR_OK) return st;
    if (trace) std::fprintf(stderr, "[conqur] polar closing check: resid_F=%.6e (iters %u)\n", res, iters);
    if (!std::isfinite(res)) return fail(ctx, CONQUR_ENONFINITE, "update_rotation: non-finite polar iterate");
    if (res <= tol) { converged = true; break; }
    if (iters >= cap || slot >= kResidSlots - 8) break;
    if (res > 0.7 && kicks < 2 && iters + 8 < cap && final_x == ctx->PX) {
      // Some singular values are still (near) zero: either far below the assumed bound or
      // pinned there by an exact symmetry of M (identical columns, which identical
      // corner-sign columns produce and which the iteration, rounding included,
      // preserves).  Nudge the iterate towards the previous rotation -- on those
      // directions every completion is optimal and this one is nearest to R_prev --
      // and run the main phase again from the nudge's scale.
      const double kappa = np_main == 1 ? 1.0 / 64.0 : 1.0 / 256.0;
      HIP_TRY(launch_axpy(ctx->PX, ctx->R, plane, (float)kappa, s));
      ++kicks;
      st = main_phase(0.25 * kappa / std::sqrt((double)dh), false);
      if (st != CONQUR_OK) return st;
      continue;
    }
    const bf16_bits* W = ctx->PW;
    const bool quintic = res <= 1e-2 * std::sqrt((double)dh);   // rms deviation of the singular values below 1e-2
    const bool predict = quintic && keep_sq;
    if (quintic) {
      if (!spec_square) HIP_TRY(square_correction(keep_sq));
      W = ctx->PW2;
    }
    // lean: the step is expected to be the last one -- no operand planes for a further Gram / apply, and the
    // result goes straight into R
    const bool lean = predict && !ctx->cfg.polar_verify;
    if (final_x != ctx->PX) {   // an earlier lean step was not the last after all: continue from its result
      HIP_TRY(hipMemcpyAsync(ctx->PX, ctx->R, (size_t)plane * sizeof(float), hipMemcpyDeviceToDevice, s));
      final_x = ctx->PX;
    }
    HIP_TRY(apply(seg_corr, W, lean ? 0 : 3, lean ? 0 : 2, true, lean ? ctx->R : ctx->PX));
    if (lean) final_x = ctx->R;
    ++iters; ++closing;
    if (predict) {
      // Orthogonality of the corrected iterate without another fp32-equivalent Gram matrix: the exact-arithmetic
      // residual of the quintic step, 5 ||D^3||_F (1 + 0.75 rho + 0.9 rho^2) with rho = ||D||_2 <= 0.05 here
      // (kCubeFactor = 5.5 also covers the bf16 rounding of the D^3 product),
      // plus the rounding of the correction product and of the fp32 iterate (kOrthFloor per unit of dh,
      // calibrated against the measured residual).
      // First from what the D^2 product left behind, without another GEMM: D is symmetric, so ||D||_2^2 = ||D^2||_2
      // <= ||D^2||_F and ||D^3||_F <= ||D||_2 ||D^2||_F <= ||D^2||_F^(3/2).  Looser than the norm itself by about
      // dh^(1/4), which the tolerance still accommodates up to dh of a few thousand.
      if (sq_slot >= 0 && !ctx->cfg.polar_verify) {
        HIP_TRY(hipEventSynchronize(ctx->ev_sq));
        double worst = 0.0;
        for (int q = 0; q < h; ++q) worst = std::max(worst, std::sqrt(hist[(size_t)sq_slot * h + q]));
        const double pred1 = kCubeFactor * std::pow(worst, 1.5) + kOrthFloorPerDim * dh;
        if (trace) std::fprintf(stderr, "[conqur] polar closing: ||D^2||_F=%.4e bound on resid_F=%.4e\n", worst, pred1);
        if (std::isfinite(pred1) && pred1 <= tol) {
          for (int q = 0; q < h; ++q) {
            const double b = kCubeFactor * std::pow(std::sqrt(hist[(size_t)sq_slot * h + q]), 1.5) + kOrthFloorPerDim * dh;
            hist[(size_t)sq_slot * h + q] = b * b;
          }
          last_slot = sq_slot;
          converged = true;
          predicted = true;
          break;
        }
      }
      HIP_TRY(cube_norm());
      const int cslot = slot++;
      st = post_resid(cslot);
      if (st != CONQUR_OK) return st;
      if (lean) {   // expected to be the end: the finishing kernels go in before the host waits for the norm
        st = enqueue_finish();
        if (st != CONQUR_OK) return st;
        finished = true;
      }
      double d3 = 0.0;
      st = wait_resid(cslot, &d3);
      if (st != CONQUR_OK) return st;
      const double pred = kCubeFactor * d3 + kOrthFloorPerDim * dh;
      if (trace) std::fprintf(stderr, "[conqur] polar closing: ||D^3||_F=%.4e predicted resid_F=%.4e\n", d3, pred);
      if (!ctx->cfg.polar_verify && std::isfinite(pred) && pred <= tol) {
        for (int q = 0; q < h; ++q) {
          const double d3q = std::sqrt(hist[(size_t)cslot * h + q]);
          hist[(size_t)cslot * h + q] = (kCubeFactor * d3q + kOrthFloorPerDim * dh) * (kCubeFactor * d3q + kOrthFloorPerDim * dh);
        }
        last_slot = cslot;
        converged = true;
        predicted = true;
        break;
      }
      if (lean) {   // prediction above the tolerance: measure after all, which needs the operand planes
        finished = false;
        HIP_TRY(launch_pack(ctx->R, h, dh, dh, 3, ctx->PXn[cur], ctx->PXt[cur], plane, s));
      }
    }
  }

  if (!finished) {
    st = enqueue_finish();
    if (st != CONQUR_OK) return st;
  }
  ctx->ev_valid[ST_UPDATE] = timed;
  // <R_op, M> | <R, M> | ||M||_F^2 | non-finite flag: one copy of the result block
  double* const resblk = ctx->host_res + (size_t)kResidSlots * h;
  HIP_TRY(hipMemcpyAsync(resblk, ctx->ldot, ((size_t)3 * h + 1) * sizeof(double), hipMemcpyDeviceToHost, s));
  HIP_TRY(launch_fill_zero(ctx->nonfinite, sizeof(int), s));
  HIP_TRY(hipStreamSynchronize(s));
  const double *ldot = resblk, *inner = resblk + h, *fro2 = resblk + 2 * h;
  int nonfinite = 0;
  std::memcpy(&nonfinite, resblk + 3 * h, sizeof(int));
  ctx->m_empty = true;
  ctx->have_rows = false;
  ctx->h_empty.assign(h, 1);
  ctx->h_rows.assign(h, 0);
  if (out) {
    float ms = 0.0f;
    HIP_TRY(hipEventElapsedTime(&ms, ctx->ev[ST_UPDATE][0], ctx->ev[ST_UPDATE][1]));
    for (int q = 0; q < h; ++q) {
      out[q].iters = iters; out[q].accurate = closing; out[q].orth_measured = predicted ? 0u : 1u;
      out[q].orth_err = std::sqrt(hist[(size_t)last_slot * h + q]);
      out[q].inner = inner[q]; out[q].m_fro = std::sqrt(fro2[q]); out[q].ms = ms;
      out[q].l1 = ctx->head_fused ? ldot[q] : ctx->l_base[q] + std::sqrt((double)dh) * ldot[q];
      out[q].mfma_flop = mfma_flop;
    }
  }
  ctx->l_base.assign(h, 0.0);
  if (!converged) return fail(ctx, CONQUR_ENOCONV, "update_rotation: polar iteration hit polar_max_iters");
  if (nonfinite) return fail(ctx, CONQUR_ENONFINITE, "rows with non-finite values were skipped");
  return CONQUR_OK;
}

static conqur_status quant_error_impl(conqur_ctx* ctx, const void* X, uint64_t T64, uint64_t stride64, uint32_t bits,
                                      int zero_point, float clip, double* sse, double* energy) {
  conqur_status st = check_x(ctx, X, T64, stride64);
  if (st != CONQUR_OK) return st;
  if (bits < 2 || bits > 8) return fail(ctx, CONQUR_EINVAL, "bits must be in [2, 8]");
  if (zero_point && (!(clip > 0.0f) || clip > 1.0f)) return fail(ctx, CONQUR_EINVAL, "clip_ratio must be in (0, 1]");
  if (!sse || !energy) return fail(ctx, CONQUR_EINVAL, "sse_host / energy_host is NULL");
  HIP_TRY(hipSetDevice(ctx->cfg.device));
  const int64_t T = (int64_t)T64, stride = (int64_t)stride64;
  hipStream_t s = ctx->stream;
  {
  StageTimer whole(ctx, ST_QUANT, 1);
  {
    StageTimer tm(ctx, ST_QROT);
    if (ctx->f32)
      HIP_TRY(launch_split_rows(reinterpret_cast<const float*>(X), T, stride, ctx->d, ctx->Xs, ctx->tmax * ctx->d, s));
    GemmArgs g;
    rotate_args(ctx, X, T, stride, &g);
    g.C = ctx->Y; g.ldc = ctx->d; g.batchC = ctx->dh; g.c_is_f32 = ctx->f32;
    HIP_TRY(launch_gemm_nt(g, EPI_ACT, ctx->heads, s));
  }
  {
    StageTimer tm(ctx, ST_QERR);
    // a batch's per-row results are small: the host adds them (fixed order) instead of one more kernel launch
    // (the per-row energies directly behind the per-row errors: one copy brings both)
    HIP_TRY(launch_quant_error(ctx->Y, ctx->f32, T, ctx->d, ctx->d, (int)bits, zero_point, clip, ctx->row_sse, ctx->row_sse + T,
                               T <= kHostSumRows ? nullptr : ctx->qsum, nullptr, 0, s));
  }
  }
  double host[2] = {0.0, 0.0};
  if (T <= kHostSumRows) {
    const float* rows = ctx->host_rows;   // pinned
    HIP_TRY(hipMemcpyAsync(ctx->host_rows, ctx->row_sse, (size_t)2 * T * sizeof(float), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    for (int64_t i = 0; i < T; ++i) { host[0] += (double)rows[i]; host[1] += (double)rows[T + i]; }
  } else {
    HIP_TRY(hipMemcpyAsync(host, ctx->qsum, sizeof(host), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
  }
  *sse = host[0];
  *energy = host[1];
  return CONQUR_OK;
}

conqur_status conqur_quant_error(conqur_ctx* ctx, const void* X, uint64_t T, uint64_t stride, uint32_t bits, double* sse,
                                 double* energy) {
  return quant_error_impl(ctx, X, T, stride, bits, 0, 1.0f, sse, energy);
}

conqur_status conqur_quant_error_zp(conqur_ctx* ctx, const void* X, uint64_t T, uint64_t stride, uint32_t bits,
                                    float clip_ratio, double* sse, double* energy) {
  return quant_error_impl(ctx, X, T, stride, bits, 1, clip_ratio, sse, energy);
}

conqur_status conqur_rotate(conqur_ctx* ctx, const void* X, uint64_t T64, uint64_t stride64, void* Y, uint64_t y_stride64) {
  conqur_status st = check_x(ctx, X, T64, stride64);
  if (st != CONQUR_OK) return st;
  if (!Y) return fail(ctx, CONQUR_EINVAL, "Y_dev is NULL");
  const uint64_t esz = ctx->f32 ? 4 : 2;
  if (y_stride64 < (uint64_t)ctx->d || y_stride64 >= (1ull << 21) || (reinterpret_cast<uintptr_t>(Y) % esz) != 0)
    return fail(ctx, CONQUR_EINVAL, "Y row stride must be >= d and < 2^21, and Y aligned to its element size");
  HIP_TRY(hipSetDevice(ctx->cfg.device));
  const int64_t T = (int64_t)T64, stride = (int64_t)stride64;
  hipStream_t s = ctx->stream;
  if (ctx->f32)
    HIP_TRY(launch_split_rows(reinterpret_cast<const float*>(X), T, stride, ctx->d, ctx->Xs, ctx->tmax * ctx->d, s));
  GemmArgs g;
  rotate_args(ctx, X, T, stride, &g);
  g.C = Y; g.ldc = (int64_t)y_stride64; g.batchC = ctx->dh; g.c_is_f32 = ctx->f32;
  HIP_TRY(launch_gemm_nt(g, EPI_ACT, ctx->heads, s));
  return CONQUR_OK;
}

conqur_status conqur_rotate_quant(conqur_ctx* ctx, const void* X, uint64_t T64, uint64_t stride64, uint32_t bits,
                                  uint32_t zero_point, float clip_ratio, void* Yq, uint64_t yq_stride64) {
  conqur_status st = check_x(ctx, X, T64, stride64);
  if (st != CONQUR_OK) return st;
  if (bits < 2 || bits > 8) return fail(ctx, CONQUR_EINVAL, "bits must be in [2, 8]");
  if (zero_point > 1) return fail(ctx, CONQUR_EINVAL, "zero_point must be 0 or 1");
  if (zero_point && (!(clip_ratio > 0.0f) || clip_ratio > 1.0f)) return fail(ctx, CONQUR_EINVAL, "clip_ratio must be in (0, 1]");
  if (!Yq) return fail(ctx, CONQUR_EINVAL, "Yq_dev is NULL");
  // the quantising kernel stores 16-byte chunks
  if (yq_stride64 < (uint64_t)ctx->d || yq_stride64 >= (1ull << 40) || (reinterpret_cast<uintptr_t>(Yq) % 16) != 0 ||
      (yq_stride64 * (ctx->f32 ? 4 : 2)) % 16 != 0)
    return fail(ctx, CONQUR_EINVAL, "Yq row stride must be >= d and Yq and its rows aligned to 16 bytes");
  HIP_TRY(hipSetDevice(ctx->cfg.device));
  const int64_t T = (int64_t)T64, stride = (int64_t)stride64;
  hipStream_t s = ctx->stream;
  StageTimer whole(ctx, ST_QUANT, 1);   // the stages are timed in the slots of conqur_quant_error
  {
    StageTimer tm(ctx, ST_QROT);
    if (ctx->f32)
      HIP_TRY(launch_split_rows(reinterpret_cast<const float*>(X), T, stride, ctx->d, ctx->Xs, ctx->tmax * ctx->d, s));
    GemmArgs g;
    rotate_args(ctx, X, T, stride, &g);
    g.C = ctx->Y; g.ldc = ctx->d; g.batchC = ctx->dh; g.c_is_f32 = ctx->f32;
    HIP_TRY(launch_gemm_nt(g, EPI_ACT, ctx->heads, s));
  }
  {
    StageTimer tm(ctx, ST_QERR);
    HIP_TRY(launch_quant_error(ctx->Y, ctx->f32, T, ctx->d, ctx->d, (int)bits, (int)zero_point, clip_ratio, ctx->row_sse,
                               ctx->row_en, nullptr, Yq, (int64_t)yq_stride64, s));
  }
  return CONQUR_OK;
}

conqur_status conqur_row_diagnostics(conqur_ctx* ctx, const void* X, uint64_t T64, uint64_t stride64, float* pr_host,
                                     float* rho_host) {
  conqur_status st = check_x(ctx, X, T64, stride64);
  if (st != CONQUR_OK) return st;
  HIP_TRY(hipSetDevice(ctx->cfg.device));
  const int64_t T = (int64_t)T64, stride = (int64_t)stride64;
  hipStream_t s = ctx->stream;
  if (ctx->f32)
    HIP_TRY(launch_split_rows(reinterpret_cast<const float*>(X), T, stride, ctx->d, ctx->Xs, ctx->tmax * ctx->d, s));
  GemmArgs g;
  rotate_args(ctx, X, T, stride, &g);
  g.C = ctx->Y; g.ldc = ctx->d; g.batchC = ctx->dh; g.c_is_f32 = ctx->f32;
  HIP_TRY(launch_gemm_nt(g, EPI_ACT, ctx->heads, s));
  HIP_TRY(launch_row_diag(ctx->Y, ctx->f32, T, ctx->d, ctx->d, ctx->row_sse, ctx->row_en, s));
  if (pr_host) HIP_TRY(hipMemcpyAsync(pr_host, ctx->row_sse, T * sizeof(float), hipMemcpyDeviceToHost, s));
  if (rho_host) HIP_TRY(hipMemcpyAsync(rho_host, ctx->row_en, T * sizeof(float), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  return CONQUR_OK;
}

conqur_status conqur_get_state(conqur_ctx* ctx, float* R_host, float* M_host, uint64_t* n_rows) {
  if (!ctx) return CONQUR_EINVAL;
  const size_t blk = (size_t)ctx->heads * ctx->dh * ctx->dh;
  hipStream_t s = ctx->stream;
  if (R_host) HIP_TRY(hipMemcpyAsync(R_host, ctx->R, blk * sizeof(float), hipMemcpyDeviceToHost, s));
  if (M_host && ctx->parts_pending) {
    HIP_TRY(hipSetDevice(ctx->cfg.device));
    conqur_status st = materialise_m(ctx);
    if (st != CONQUR_OK) return st;
  }
  if (M_host) {
    if (ctx->m_empty) std::memset(M_host, 0, blk * sizeof(float));
    else HIP_TRY(hipMemcpyAsync(M_host, ctx->M, blk * sizeof(float), hipMemcpyDeviceToHost, s));
  }
  std::vector<unsigned long long> rows(ctx->heads, 0ull);
  if (n_rows) {   // the fused per-head step counts in ctx->rows, the general path in the slot counters: both are added
    std::vector<unsigned long long> buf(ctx->stat_words);
    HIP_TRY(hipMemcpyAsync(buf.data(), ctx->L, ctx->stat_words * sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    const int h = ctx->heads;
    for (int i = 0; i < h; ++i) {
      rows[i] = buf[h + i];
      for (int q = 0; q < kCountSlots; ++q) rows[i] += buf[3 * h + ((size_t)i * kCountSlots + q) * 2];
    }
  }
  HIP_TRY(hipStreamSynchronize(s));
  if (M_host && !ctx->m_empty)   // heads stepped in ranges: those without rows still hold the M of before the last update
    for (int i = 0; i < ctx->heads; ++i)
      if (ctx->h_empty[i] && ctx->head_fused)
        std::memset(M_host + (size_t)i * ctx->dh * ctx->dh, 0, (size_t)ctx->dh * ctx->dh * sizeof(float));
  if (n_rows) for (int i = 0; i < ctx->heads; ++i) n_rows[i] = rows[i];
  return CONQUR_OK;
}

conqur_status conqur_set_state(conqur_ctx* ctx, const float* R_host, const float* M_host) {
  if (!ctx) return CONQUR_EINVAL;
  const size_t blk = (size_t)ctx->heads * ctx->dh * ctx->dh;
  hipStream_t s = ctx->stream;
  HIP_TRY(hipSetDevice(ctx->cfg.device));
  const int h = ctx->heads;
  const int64_t n = (int64_t)ctx->dh * ctx->dh;
  // The general path reads the l1 term of the pending rows off M through the current rotation (k_dot_rm).  Replacing
  // the rotation while rows are pending keeps it right by moving the difference into an offset.
  const bool rebase = R_host && !M_host && !ctx->head_fused && !ctx->m_empty;
  std::vector<double> d_old(h, 0.0), d_new(h, 0.0);
  if (rebase) {
    HIP_TRY(launch_dot_rm(ctx->R, ctx->M, h, n, ctx->f32 ? 0 : 1, ctx->dotrm_part, ctx->ldot, s));
    HIP_TRY(hipMemcpyAsync(d_old.data(), ctx->ldot, h * sizeof(double), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
  }
  if (R_host) {
    HIP_TRY(hipMemcpyAsync(ctx->R, R_host, blk * sizeof(float), hipMemcpyHostToDevice, s));
    conqur_status st = refresh_operand(ctx);
    if (st != CONQUR_OK) return st;
  }
  if (rebase) {
    HIP_TRY(launch_dot_rm(ctx->R, ctx->M, h, n, ctx->f32 ? 0 : 1, ctx->dotrm_part, ctx->ldot, s));
    HIP_TRY(hipMemcpyAsync(d_new.data(), ctx->ldot, h * sizeof(double), hipMemcpyDeviceToHost, s));
  }
  if (M_host) {
    HIP_TRY(hipMemcpyAsync(ctx->M, M_host, blk * sizeof(float), hipMemcpyHostToDevice, s));
    ctx->parts_pending = 0;   // whatever shares were pending are replaced with the rest of M
    ctx->m_empty = false;
    ctx->have_rows = true;
    ctx->h_empty.assign(h, 0);
    ctx->h_rows.assign(h, 1);
    ctx->l_base.assign(h, 0.0);   // the rows behind the old M are gone
  }
  HIP_TRY(hipStreamSynchronize(s));
  if (rebase)
    for (int i = 0; i < h; ++i) ctx->l_base[i] += std::sqrt((double)ctx->dh) * (d_old[i] - d_new[i]);
  return CONQUR_OK;
}

conqur_status conqur_get_last_corners(conqur_ctx* ctx, int8_t* signs, float* norms) {
  if (!ctx) return CONQUR_EINVAL;
  if (ctx->last_T == 0) return fail(ctx, CONQUR_ESTATE, "no step_batch yet");
  if (signs && !ctx->last_signs_valid)
    return fail(ctx, CONQUR_ESTATE, "the last step did not keep the corner signs: call conqur_set_taps(ctx, 1) before it");
  const int64_t T = ctx->last_T, d = ctx->d, pitch = ctx->pitch, tmax = ctx->tmax;
  hipStream_t s = ctx->stream;
  // whole buffers in one plain copy each, sliced on the host (a debug tap: simplicity over bytes moved)
  std::vector<float> nrm((size_t)ctx->heads * tmax);
  HIP_TRY(hipMemcpyAsync(nrm.data(), ctx->nrm, nrm.size() * sizeof(float), hipMemcpyDeviceToHost, s));
  std::vector<bf16_bits> st;
  if (signs) {
    st.resize((size_t)d * pitch);
    HIP_TRY(hipMemcpyAsync(st.data(), ctx->St, st.size() * sizeof(bf16_bits), hipMemcpyDeviceToHost, s));
  }
  HIP_TRY(hipStreamSynchronize(s));
  if (norms)
    for (int h = 0; h < ctx->heads; ++h) std::memcpy(norms + (size_t)h * T, nrm.data() + (size_t)h * tmax, T * sizeof(float));
  if (signs)
    for (int64_t j = 0; j < d; ++j) {
      const float* nh = nrm.data() + (j / ctx->dh) * tmax;
      for (int64_t i = 0; i < T; ++i)
        signs[i * d + j] = nh[i] > 0.0f ? ((st[j * pitch + i] & 0x8000) ? -1 : 1) : 0;
    }
  return CONQUR_OK;
}

}  // extern "C"
