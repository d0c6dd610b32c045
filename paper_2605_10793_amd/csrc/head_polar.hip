// Main phase of the polar iteration for heads of width 128, one launch for all steps
// (the composed cubics X <- X (a_k I + b_k X^T X) of the Procrustes update, Sec. 3.3).
//
// At this width the iterate (32 KiB as fp16, natural and transposed), and the
// polynomial factor W (32 KiB) live in the LDS of one compute unit, so a workgroup
// per head runs the whole schedule without touching HBM between steps; the general
// path needs two GEMM launches per step, which at 128 x 128 are launch latency only.
// Per step, with every product a 32x32x16 fp16 MFMA on K-contiguous operands (the iterate and the factor are held as
// fp16: 11 significant bits at the rate of bf16's 8; every entry is at most a few units in magnitude):
//   G = X^T X            A = B = X^T                     -> W = a I + b G, fp16, to LDS
//   X' = X W             A = X,  B = W (symmetric)       -> accumulators hold X'
// An accumulator lane owns 4 consecutive rows of one column, i.e. 8 contiguous bytes of the transposed matrix:
// X'^T goes to LDS as packed 8-byte writes, X' itself as four 2-byte writes per such group (64 per lane and step,
// their addresses computed once).  Computing the product in the other orientation as well (X'^T = W X^T, packed
// stores for both layouts) cost a third of the step's MFMA and LDS-read time and is kept for the last step only,
// whose results leave for HBM.
// The last step writes what the closing iterations read: the iterate rounded to bf16, as
// fp32 and as one plane of each layout.
#include "kernels.h"

namespace conqur {

namespace {

constexpr int DH = 128;
constexpr int ROWB = 256;   // bytes per LDS row (128 bf16), 16 chunks of 16 bytes, XOR swizzled
constexpr int kSmemBytes = 3 * DH * ROWB;

__device__ __forceinline__ int loff(int row, int chunk) { return row * ROWB + ((chunk ^ (row & 15)) << 4); }

__global__ void __launch_bounds__(256) k_head_polar128(const bf16_bits* __restrict__ Xn0, const bf16_bits* __restrict__ Xt0,
                                                       const PolarSchedule sched, float* __restrict__ X32,
                                                       bf16_bits* __restrict__ Pn, bf16_bits* __restrict__ Pt) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* const sXn = smem;                  // X   : row r, K = column
  unsigned char* const sXt = smem + DH * ROWB;      // X^T : row c, K = row of X
  unsigned char* const sW = smem + 2 * DH * ROWB;   // W   : symmetric
  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int wm = wave >> 1, wn = wave & 1;          // this wavefront's 64 x 64 block of every 128 x 128 product
  const int64_t hoff = (int64_t)h * DH * DH;

#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int idx = q * 256 + tid, row = idx >> 4, chunk = idx & 15;
    *reinterpret_cast<uint4*>(sXn + loff(row, chunk)) = *reinterpret_cast<const uint4*>(Xn0 + hoff + row * DH + chunk * 8);
    *reinterpret_cast<uint4*>(sXt + loff(row, chunk)) = *reinterpret_cast<const uint4*>(Xt0 + hoff + row * DH + chunk * 8);
  }
  __syncthreads();

  auto frag = [&](const unsigned char* base, int row, int kk) {
    return *reinterpret_cast<const f16x8*>(base + loff(row, 2 * kk + half));
  };
  // acc[i][j] = sum_k A[rowA + 32 i + .][k] B[rowB + 32 j + .][k]
  auto product = [&](const unsigned char* A, int rowA, const unsigned char* B, int rowB, f32x16 (&acc)[2][2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk) {
      f16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[i] = frag(A, rowA + 32 * i + col, kk);
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j] = frag(B, rowB + 32 * j + col, kk);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  };
  // Element e = 4 jj + ii of acc[i][j]: row m = rowA + 32 i + 8 jj + 4 half + ii, column n = rowB + 32 j + col.
  // Store the transposed matrix into an LDS operand: row n, K positions m .. m + 3 (8 bytes).
  auto store_transposed = [&](unsigned char* dst, int rowA, int rowB, const f32x16 (&acc)[2][2], float ci, float cg) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = rowB + 32 * j + col;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int m0 = rowA + 32 * i + 8 * jj + 4 * half;
          float v[4];
#pragma unroll
          for (int ii = 0; ii < 4; ++ii) v[ii] = cg * acc[i][j][4 * jj + ii] + ((m0 + ii == n) ? ci : 0.0f);
          uint2 pk;
          pk.x = f32x2_to_f16x2(v[0], v[1]);
          pk.y = f32x2_to_f16x2(v[2], v[3]);
          *reinterpret_cast<uint2*>(dst + loff(n, m0 >> 3) + (m0 & 7) * 2) = pk;
        }
      }
  };

  // LDS byte offsets of the natural-layout positions of this lane's accumulator elements in tile row i = 0
  // (tile row 1 lies 32 rows = 32 * ROWB bytes further on): element e = 4 jj + ii of acc[.][j].
  uint32_t nat_addr[2][4][4];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
      for (int ii = 0; ii < 4; ++ii) {
        const int m = 64 * wm + 8 * jj + 4 * half + ii, n = 64 * wn + 32 * j + col;
        nat_addr[j][jj][ii] = (uint32_t)(loff(m, n >> 3) + (n & 7) * 2);
      }
  // The iterate itself into an LDS operand: row m, K position n, one fp16 value at a time.
  auto store_natural = [&](unsigned char* dst, const f32x16 (&acc)[2][2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const uint32_t lo = f32x2_to_f16x2(acc[i][j][4 * jj], acc[i][j][4 * jj + 1]);
          const uint32_t hi = f32x2_to_f16x2(acc[i][j][4 * jj + 2], acc[i][j][4 * jj + 3]);
          unsigned char* d = dst + i * 32 * ROWB;
          *reinterpret_cast<unsigned short*>(d + nat_addr[j][jj][0]) = (unsigned short)lo;
          *reinterpret_cast<unsigned short*>(d + nat_addr[j][jj][1]) = (unsigned short)(lo >> 16);
          *reinterpret_cast<unsigned short*>(d + nat_addr[j][jj][2]) = (unsigned short)hi;
          *reinterpret_cast<unsigned short*>(d + nat_addr[j][jj][3]) = (unsigned short)(hi >> 16);
        }
  };

  f32x16 acc[2][2], accT[2][2];
  for (int k = 0; k < sched.nsteps; ++k) {
    const bool last = k + 1 == sched.nsteps;
    // G = X^T X;  W = a I + b G (G symmetric: storing the transpose stores W itself)
    product(sXt, 64 * wm, sXt, 64 * wn, acc);
    store_transposed(sW, 64 * wm, 64 * wn, acc, sched.a[k], sched.b[k]);
    __syncthreads();
    product(sXn, 64 * wm, sW, 64 * wn, acc);    // X'   [r][c]
    if (last) {
      product(sW, 64 * wm, sXn, 64 * wn, accT);   // X'^T [c][r]: the natural-layout plane below as packed stores
      break;
    }
    __syncthreads();                            // every wavefront has read the old iterate
    store_transposed(sXt, 64 * wm, 64 * wn, acc, 0.0f, 1.0f);
    store_natural(sXn, acc);
    __syncthreads();
  }

  // Hand-over to the closing iterations: the result rounded to bf16 like every step's, and exactly that value as fp32 X,
  // as one transposed plane (from X') and as one natural plane (from X'^T; the two orientations issue the same products
  // in the same order, so they hold the same numbers): the closing Gram matrix is then exact with one plane product.
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = 64 * wn + 32 * j + col;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int m0 = 64 * wm + 32 * i + 8 * jj + 4 * half;
        uint2 hi, thi;
        hi.x = f32x2_to_bf16x2(acc[i][j][4 * jj], acc[i][j][4 * jj + 1]);
        hi.y = f32x2_to_bf16x2(acc[i][j][4 * jj + 2], acc[i][j][4 * jj + 3]);
        thi.x = f32x2_to_bf16x2(accT[i][j][4 * jj], accT[i][j][4 * jj + 1]);
        thi.y = f32x2_to_bf16x2(accT[i][j][4 * jj + 2], accT[i][j][4 * jj + 3]);
        X32[hoff + (int64_t)m0 * DH + n] = __uint_as_float(hi.x << 16);
        X32[hoff + (int64_t)(m0 + 1) * DH + n] = __uint_as_float(hi.x & 0xffff0000u);
        X32[hoff + (int64_t)(m0 + 2) * DH + n] = __uint_as_float(hi.y << 16);
        X32[hoff + (int64_t)(m0 + 3) * DH + n] = __uint_as_float(hi.y & 0xffff0000u);
        *reinterpret_cast<uint2*>(Pt + hoff + (int64_t)n * DH + m0) = hi;     // X^T[c = n][r = m0 ..]
        *reinterpret_cast<uint2*>(Pn + hoff + (int64_t)n * DH + m0) = thi;    // accT: X[r = n][c = m0 ..]
      }
    }
}

}  // namespace

hipError_t launch_head_polar128(const bf16_bits* Xn0, const bf16_bits* Xt0, int heads, const PolarSchedule& sched, float* X32,
                                bf16_bits* Pn, bf16_bits* Pt, hipStream_t s) {
  if (heads < 1 || sched.nsteps < 1 || sched.nsteps > kPolarScheduleMax) return hipErrorInvalidValue;
  static PerDeviceOnce configured;
  hipError_t e = configured.run([] {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(k_head_polar128), hipFuncAttributeMaxDynamicSharedMemorySize,
                               kSmemBytes);
  });
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_head_polar128, dim3(heads), dim3(256), kSmemBytes, s, Xn0, Xt0, sched, X32, Pn, Pt);
  return hipGetLastError();
}

}  // namespace conqur
