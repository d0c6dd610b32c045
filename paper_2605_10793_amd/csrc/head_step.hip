// Fused statistics step for per-head rotations of width 128 with bf16 activations
// (rotate + normalise + corner + accumulate of one batch in one kernel; Sec. 3.3-3.4,
// per-head blocks as for the value / output projections of Alg. 1).
//
// At this width a head's rotation (32 KiB as bf16) and its cross-covariance (64 KiB of
// fp32 accumulators) live on one compute unit, so the step is bound by reading X once
// (256 bytes per token and head) instead of by GEMM launches: a workgroup owns one
// head and one contiguous share of the tokens, keeps R_h^T in LDS and M_h in MFMA
// accumulators, and streams 128-token tiles through 16 wavefronts (the per-tile work is a
// chain of short, latency-bound phases; wider tiles halve the number of chains):
//   1. tile -> registers (16-byte loads, prefetched one tile ahead), row norms by
//      16-lane shuffles, natural copy to LDS;
//   2. Y = X R_h (32x32x16 bf16 MFMA; A = X tile, B = R_h^T), in flight with the scaled
//      transposed copy x^ (fp16) of the tile; from the accumulators: the corner signs,
//      written transposed (+-1 as fp16) to LDS;
//   3. M_h += x^^T C (32x32x16 fp16 MFMA, contraction over the tile's 128 tokens).
// Each workgroup ends by storing its partial M_h; k_head_reduce adds the shares in a
// fixed order.  Rows that are zero or non-finite are skipped exactly as in k_row_norms.
#include "kernels.h"

namespace conqur {

namespace {

constexpr int DH = 128;        // head width
constexpr int TT = 128;        // tokens per tile
constexpr int NTHREADS = 1024; // 16 wavefronts
constexpr int XROW = 256;      // bytes per natural row (128 bf16), 16 chunks of 16 bytes, XOR swizzled
constexpr int TROW = 272;      // bytes per transposed row (128 fp16 + 8 pad): ds_read_b128 of 16 consecutive rows hits 64 banks

constexpr int kSmemBytes = DH * XROW + TT * XROW + 2 * DH * TROW;
constexpr float kOutScale = 1.0f / (kXhatScale * 11.313708498984761f);   // the operand carries kXhatScale x^, the corner 1/sqrt(128)

__device__ __forceinline__ int xoff(int row, int chunk) { return row * XROW + ((chunk ^ (row & 15)) << 4); }

template <bool STORE_SIGNS>
__global__ void __launch_bounds__(NTHREADS) k_head_step128(const bf16_bits* __restrict__ X, int64_t T, int64_t stride, int heads,
                                                      const bf16_bits* __restrict__ RopT, float* __restrict__ Mpart,
                                                      int64_t tokens_per_split, float* __restrict__ nrm, int64_t ldn,
                                                      double* __restrict__ L, unsigned long long* __restrict__ rows,
                                                      unsigned long long* __restrict__ skipped, int* __restrict__ nonfinite,
                                                      bf16_bits* __restrict__ St, int64_t pitch) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];      // kSmemBytes, above the static 64 KiB limit
  unsigned char* const sR = smem;                        // R_h^T: row n, K = input channel
  unsigned char* const sX = sR + DH * XROW;              // tile, natural: row token, K = channel
  unsigned char* const sXt = sX + TT * XROW;             // x^ transposed (fp16): row channel, K = token
  unsigned char* const sCt = sXt + DH * TROW;            // corner signs transposed (fp16): row n, K = token
  __shared__ float sW[2][TT];      // kXhatScale / ||x|| per token of the tile (0: skipped), by tile parity
  __shared__ double shd[3][16];

  const int h = blockIdx.x, sp = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int64_t t_begin = (int64_t)sp * tokens_per_split;
  const int64_t t_end = t_begin + tokens_per_split < T ? t_begin + tokens_per_split : T;
  const int ntiles = t_end > t_begin ? (int)((t_end - t_begin + TT - 1) / TT) : 0;

  // R_h^T -> LDS (row n, 16 chunks)
  {
    const bf16_bits* Rh = RopT + (int64_t)h * DH * DH;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int idx = q * NTHREADS + tid, row = idx >> 4, chunk = idx & 15;
      *reinterpret_cast<uint4*>(sR + xoff(row, chunk)) = *reinterpret_cast<const uint4*>(Rh + row * DH + chunk * 8);
    }
  }

  // Thread -> tile element map of phase 1: row (token) lrow + 64 q, chunk lchunk: the 16 lanes of a row sit in one wavefront.
  const int lrow = tid >> 4, lchunk = tid & 15;
  const bf16_bits* Xh = X + (int64_t)h * DH + lchunk * 8;
  uint4 cur[2], nxt[2];
  auto load_tile = [&](int tile, uint4* dst) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int64_t t = t_begin + (int64_t)tile * TT + lrow + 64 * q;
      dst[q] = (tile < ntiles && t < t_end) ? *reinterpret_cast<const uint4*>(Xh + t * stride) : make_uint4(0u, 0u, 0u, 0u);
    }
  };
  load_tile(0, cur);

  // 16 wavefronts (4 per SIMD, so that one's LDS and conversion work runs beside the others' MFMAs).
  const int ti = wave >> 2, nb = wave & 3;        // rotate: tokens [32 ti, +32) x columns [32 nb, +32)
  const int rm = wave >> 2, cn = wave & 3;        // accumulate: channels [32 rm, +32) x columns [32 cn, +32)
  f32x16 accM;
#pragma unroll
  for (int e = 0; e < 16; ++e) accM[e] = 0.0f;
  double l_acc = 0.0;
  unsigned n_rows = 0, n_skipped = 0;

  for (int tile = 0; tile < ntiles; ++tile) {
    const int par = tile & 1;
    // ---- phase 1: norms, natural copy
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int r = lrow + 64 * q;
      const int64_t t = t_begin + (int64_t)tile * TT + r;
      const uint4 v = cur[q];
      float ss = 0.0f;
      {
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float a = __uint_as_float(u[e] << 16), b = __uint_as_float(u[e] & 0xffff0000u);
          ss += a * a + b * b;
        }
      }
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);   // over the 16 lanes of the row
      *reinterpret_cast<uint4*>(sX + xoff(r, lchunk)) = v;
      if (lchunk == 0) {
        float n = 0.0f, w = 0.0f;
        if (t < t_end) {
          if (!isfinite(ss)) {
            atomicOr(nonfinite, 1);
            ++n_skipped;
          } else if (ss > 0.0f) {
            n = sqrtf(ss);
            w = kXhatScale / n;
            ++n_rows;
          } else {
            ++n_skipped;
          }
          nrm[(int64_t)h * ldn + t] = n;
        }
        sW[par][r] = w;
      }
    }
    load_tile(tile + 1, nxt);   // in flight during phases 2 and 3
    __syncthreads();

    // ---- phase 2a: scaled transposed copy x^ (fp16).  Thread = (token pair p, chunk g): 4-byte LDS writes whose
    // banks differ across the 64 token pairs of a wavefront.
    {
      const int p = tid & 63, g = tid >> 6;
      const float w0 = sW[par][2 * p], w1 = sW[par][2 * p + 1];
      {
        const int chunk = g;
        const uint4 a = *reinterpret_cast<const uint4*>(sX + xoff(2 * p, chunk));
        const uint4 b = *reinterpret_cast<const uint4*>(sX + xoff(2 * p + 1, chunk));
        const uint32_t ua[4] = {a.x, a.y, a.z, a.w}, ub[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t xa = (e & 1) ? (ua[e >> 1] & 0xffff0000u) : (ua[e >> 1] << 16);
          const uint32_t xb = (e & 1) ? (ub[e >> 1] & 0xffff0000u) : (ub[e >> 1] << 16);
          // a skipped row has w = 0 and possibly Inf/NaN values: select, do not multiply
          const float fa = w0 != 0.0f ? __uint_as_float(xa) * w0 : 0.0f;
          const float fb = w1 != 0.0f ? __uint_as_float(xb) * w1 : 0.0f;
          const uint32_t packed = (uint32_t)f32_to_f16(fa) | ((uint32_t)f32_to_f16(fb) << 16);
          *reinterpret_cast<uint32_t*>(sXt + (chunk * 8 + e) * TROW + 4 * p) = packed;
        }
      }
    }
    // ---- phase 2b: Y = X R_h.  Wavefront (ti, nb) owns tokens [32 ti, +32) x output columns [32 nb, +32).
    f32x16 accY;
#pragma unroll
    for (int e = 0; e < 16; ++e) accY[e] = 0.0f;
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk) {
      const bf16x8 fb = *reinterpret_cast<const bf16x8*>(sR + xoff(32 * nb + col, 2 * kk + half));
      const bf16x8 fa = *reinterpret_cast<const bf16x8*>(sX + xoff(32 * ti + col, 2 * kk + half));
      accY = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, accY, 0, 0, 0);
    }
    // accY[4 j + ii] = y[token 32 ti + 8 j + 4 half + ii][n = 32 nb + col]
    {
      // corner signs, transposed: 4 consecutive tokens of column n are 8 bytes
      const int n = 32 * nb + col;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        uint32_t sg[4];
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) sg[ii] = accY[4 * j + ii] >= 0.0f ? 0x3C00u : 0xBC00u;   // sgn(0) = +1
        uint2 pk;
        pk.x = sg[0] | (sg[1] << 16);
        pk.y = sg[2] | (sg[3] << 16);
        const int tok = 32 * ti + 8 * j + 4 * half;
        *reinterpret_cast<uint2*>(sCt + n * TROW + 2 * tok) = pk;
        if constexpr (STORE_SIGNS) {
          const int64_t t = t_begin + (int64_t)tile * TT + tok;
          if (t < t_end)   // pitch and t are multiples of 4: the 4 tokens are in range together up to the pitch
            *reinterpret_cast<uint2*>(St + ((int64_t)h * DH + n) * pitch + t) = pk;
        }
      }
    }
    __syncthreads();

    // ---- phase 3: M_h += x^^T C.  Wavefront (rm, cn) owns channels [32 rm, +32) x columns [32 cn, +32) of M_h.
#pragma unroll
    for (int kk = 0; kk < TT / 16; ++kk) {
      const f16x8 fa = *reinterpret_cast<const f16x8*>(sXt + (32 * rm + col) * TROW + (2 * kk + half) * 16);
      const f16x8 fb = *reinterpret_cast<const f16x8*>(sCt + (32 * cn + col) * TROW + (2 * kk + half) * 16);
      accM = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa, fb, accM, 0, 0, 0);
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) cur[q] = nxt[q];
    // no barrier here: the next phase 1 writes sX and the other parity of sW, which nobody reads in phase 3;
    // sXt / sCt are written again only after the next tile's first barrier.
  }

  // ---- partial M_h of this share; and this share's l1 term without a per-token reduction:
  //   sum_t ||y_t||_1 / ||x_t|| = sum_t sum_n sgn(y_tn) y_tn / ||x_t|| = sqrt(dh) <R_op, x^^T C>   (y = x R_op, C = sgn(y)/sqrt(dh))
  // i.e. the inner product of the operand rotation with the partial M just accumulated (the l1 identity of Sec. 3.2
  // read per batch).
  {
    float* Mp = Mpart + ((int64_t)sp * heads + h) * DH * DH;
    float dot = 0.0f;
    {
      const int n = 32 * cn + col;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = 32 * rm + 8 * (e >> 2) + 4 * half + (e & 3);
        const float mv = accM[e] * kOutScale;
        Mp[m * DH + n] = mv;
        const bf16_bits r = *reinterpret_cast<const bf16_bits*>(sR + xoff(n, m >> 3) + (m & 7) * 2);   // R_op[m][n]
        dot += mv * bf16_to_f32(r);
      }
    }
    l_acc = (double)dot * 11.313708498984761;   // sqrt(128)
  }
  // ---- statistics of this share: one atomic per workgroup and counter
  {
    double r = (double)n_rows, k = (double)n_skipped;
    l_acc = wave_sum_d(l_acc); r = wave_sum_d(r); k = wave_sum_d(k);
    if (lane == 0) { shd[0][wave] = l_acc; shd[1][wave] = r; shd[2][wave] = k; }
    __syncthreads();
    if (tid == 0) {
      double lt = 0.0, rt = 0.0, kt = 0.0;
      for (int i = 0; i < NTHREADS / 64; ++i) { lt += shd[0][i]; rt += shd[1][i]; kt += shd[2][i]; }
      atomicAdd(L + h, lt);
      atomicAdd(rows + h, (unsigned long long)rt);
      atomicAdd(skipped + h, (unsigned long long)kt);
    }
  }
}

// M[h] (+)= sum over shares of Mpart[share][h], fixed order.  FRO2: also the sum of squares of the block's 1024 results
// (one double per workgroup, fro2_part[blockIdx.x]; a head is DH * DH / 1024 = 16 consecutive workgroups), so that the
// update that follows needs no separate pass over M for ||M_h||_F.
template <bool FRO2>
__global__ void __launch_bounds__(256) k_head_reduce(const float* __restrict__ Mpart, int nsplit, int64_t n_total,
                                                     float* __restrict__ M, int accumulate, double* __restrict__ fro2_part) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;   // n_total is a multiple of 1024: no ragged block
  float4 acc = accumulate ? *reinterpret_cast<const float4*>(M + i) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  for (int s0 = 0; s0 < nsplit; s0 += 8) {   // eight shares' loads in flight, added in share order
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      v[u] = s0 + u < nsplit ? *reinterpret_cast<const float4*>(Mpart + (s0 + u) * n_total + i) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
    for (int u = 0; u < 8; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
  }
  *reinterpret_cast<float4*>(M + i) = acc;
  if constexpr (FRO2) {
    __shared__ double sh[4];
    double q = (double)acc.x * acc.x + (double)acc.y * acc.y + (double)acc.z * acc.z + (double)acc.w * acc.w;
    q = wave_sum_d(q);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = q;
    __syncthreads();
    if (threadIdx.x == 0) fro2_part[blockIdx.x] = sh[0] + sh[1] + sh[2] + sh[3];
  }
}

}  // namespace

int head_step_splits(int heads, int64_t T) {
  int64_t by_tiles = (T + TT - 1) / TT;
  int64_t want = 256 / heads;
  if (want < 1) want = 1;
  if (want > 16) want = 16;
  return (int)(want < by_tiles ? want : by_tiles);
}

hipError_t launch_head_step128(const bf16_bits* X, int64_t T, int64_t stride, int heads, const bf16_bits* RopT, float* Mpart,
                               int nsplit, float* nrm, int64_t ldn, double* L, unsigned long long* rows,
                               unsigned long long* skipped, int* nonfinite, bf16_bits* St, int64_t pitch, hipStream_t s) {
  if (heads < 1 || T < 1 || nsplit < 1) return hipErrorInvalidValue;
  // whole tiles per share, so that the shares' 4-token sign stores never straddle a share boundary
  const int64_t tiles = (T + TT - 1) / TT;
  const int64_t tokens_per_split = (tiles + nsplit - 1) / nsplit * TT;
  const dim3 grid(heads, nsplit);
  static PerDeviceOnce configured;
  hipError_t e = configured.run([] {
    hipError_t r = hipFuncSetAttribute(reinterpret_cast<const void*>(k_head_step128<true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kSmemBytes);
    if (r == hipSuccess)
      r = hipFuncSetAttribute(reinterpret_cast<const void*>(k_head_step128<false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                              kSmemBytes);
    return r;
  });
  if (e != hipSuccess) return e;
  if (St)
    hipLaunchKernelGGL(k_head_step128<true>, grid, dim3(NTHREADS), kSmemBytes, s, X, T, stride, heads, RopT, Mpart, tokens_per_split, nrm, ldn,
                       L, rows, skipped, nonfinite, St, pitch);
  else
    hipLaunchKernelGGL(k_head_step128<false>, grid, dim3(NTHREADS), kSmemBytes, s, X, T, stride, heads, RopT, Mpart, tokens_per_split, nrm, ldn,
                       L, rows, skipped, nonfinite, St, pitch);
  return hipGetLastError();
}

hipError_t launch_sum_shares(const float* part, int nsplit, int64_t n_total, float* M, int accumulate, hipStream_t s) {
  if (nsplit < 1 || n_total < 1024 || (n_total & 1023)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_head_reduce<false>, dim3((unsigned)(n_total / 1024)), dim3(256), 0, s, part, nsplit, n_total, M, accumulate,
                     (double*)nullptr);
  return hipGetLastError();
}

hipError_t launch_head_reduce(const float* Mpart, int nsplit, int heads, float* M, int accumulate, double* fro2_part, hipStream_t s) {
  const int64_t n_total = (int64_t)heads * DH * DH;
  const dim3 grid((unsigned)(n_total / 1024));
  if (fro2_part)
    hipLaunchKernelGGL(k_head_reduce<true>, grid, dim3(256), 0, s, Mpart, nsplit, n_total, M, accumulate, fro2_part);
  else
    hipLaunchKernelGGL(k_head_reduce<false>, grid, dim3(256), 0, s, Mpart, nsplit, n_total, M, accumulate, fro2_part);
  return hipGetLastError();
}

}  // namespace conqur
