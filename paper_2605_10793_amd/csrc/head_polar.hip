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
// fp32 and as one plane of each layout.  On request the same launch then takes the closing
// step itself (exact Gram matrix of that bf16 iterate, D, D^2, two-plane correction; bf16
// MFMAs) and leaves the rotation, the rotate operand and <R, M>: see HeadPolarClose.
#include "kernels.h"

namespace conqur {

namespace {

constexpr int DH = 128;
constexpr int ROWB = 256;   // bytes per LDS row (128 bf16), 16 chunks of 16 bytes, XOR swizzled
constexpr int kSmemBytes = 3 * DH * ROWB;
constexpr int kSmemBytesClose = 4 * DH * ROWB;   // the closing step holds two planes of its correction beside the iterate

__device__ __forceinline__ int loff(int row, int chunk) { return row * ROWB + ((chunk ^ (row & 15)) << 4); }

template <bool CLOSE>
__global__ void __launch_bounds__(256) k_head_polar128(const bf16_bits* __restrict__ Xn0, const bf16_bits* __restrict__ Xt0,
                                                       const PolarSchedule sched, float* __restrict__ X32,
                                                       bf16_bits* __restrict__ Pn, bf16_bits* __restrict__ Pt,
                                                       const HeadPolarClose cl, const HeadPolarStart st) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* const sXn = smem;                  // X   : row r, K = column
  unsigned char* const sXt = smem + DH * ROWB;      // X^T : row c, K = row of X
  unsigned char* const sW = smem + 2 * DH * ROWB;   // W   : symmetric
  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int wm = wave >> 1, wn = wave & 1;          // this wavefront's 64 x 64 block of every 128 x 128 product
  const int64_t hoff = (int64_t)h * DH * DH;

  if (!st.M) {   // the start iterate is given as planes
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int idx = q * 256 + tid, row = idx >> 4, chunk = idx & 15;
      *reinterpret_cast<uint4*>(sXn + loff(row, chunk)) = *reinterpret_cast<const uint4*>(Xn0 + hoff + row * DH + chunk * 8);
      *reinterpret_cast<uint4*>(sXt + loff(row, chunk)) = *reinterpret_cast<const uint4*>(Xt0 + hoff + row * DH + chunk * 8);
    }
    __syncthreads();
  }

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
  if (st.M) {
    // The start of the update in this launch as well (what the packing pass does on the general path):
    // X0 = (M + lambda tau R_prev) / alpha, tau = ||M||_F / sqrt(dh), alpha = ||M||_F (1 + lambda), with ||M||_F^2 summed from
    // the partial sums the reduction of the token shares left (or given whole: nparts = 1); lambda = 0 stands for the
    // limit at fp32 resolution, an empty M for R_prev itself.  Elements in the accumulators' layout, so that the two LDS
    // operands are written exactly as after a step.
    double f2 = 0.0;
    for (int p = 0; p < st.nparts; ++p) f2 += st.fro2_parts[(int64_t)h * st.nparts + p];
    if (tid == 0) {
      st.fro2_out[h] = f2;
      if (st.ldot) st.ldot[h] = st.L[h];   // the l1 term of the rows this update consumes, kept before the statistics restart
    }
    const double f = sqrt(f2);
    const bool empty = !(f > 0.0);
    const float lambda = fmaxf(st.lambda, 9.5367431640625e-07f);
    const float tau = (float)(f / sqrt((double)DH));
    const float inv_alpha = empty ? 1.0f : (float)(1.0 / (f * (1.0 + (double)lambda)));
    const float cm = empty ? 0.0f : inv_alpha, cr = empty ? 1.0f : lambda * tau * inv_alpha;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int m = 64 * wm + 32 * i + 8 * (e >> 2) + 4 * half + (e & 3), n = 64 * wn + 32 * j + col;
          const int64_t off = hoff + (int64_t)m * DH + n;
          acc[i][j][e] = cm * st.M[off] + cr * st.R[off];
        }
    store_transposed(sXt, 64 * wm, 64 * wn, acc, 0.0f, 1.0f);
    store_natural(sXn, acc);
    __syncthreads();
  }
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
        // from here on the accumulators hold the rounded values (exact as bf16)
        acc[i][j][4 * jj] = __uint_as_float(hi.x << 16); acc[i][j][4 * jj + 1] = __uint_as_float(hi.x & 0xffff0000u);
        acc[i][j][4 * jj + 2] = __uint_as_float(hi.y << 16); acc[i][j][4 * jj + 3] = __uint_as_float(hi.y & 0xffff0000u);
        accT[i][j][4 * jj] = __uint_as_float(thi.x << 16); accT[i][j][4 * jj + 1] = __uint_as_float(thi.x & 0xffff0000u);
        accT[i][j][4 * jj + 2] = __uint_as_float(thi.y << 16); accT[i][j][4 * jj + 3] = __uint_as_float(thi.y & 0xffff0000u);
        X32[hoff + (int64_t)m0 * DH + n] = acc[i][j][4 * jj];
        X32[hoff + (int64_t)(m0 + 1) * DH + n] = acc[i][j][4 * jj + 1];
        X32[hoff + (int64_t)(m0 + 2) * DH + n] = acc[i][j][4 * jj + 2];
        X32[hoff + (int64_t)(m0 + 3) * DH + n] = acc[i][j][4 * jj + 3];
        *reinterpret_cast<uint2*>(Pt + hoff + (int64_t)n * DH + m0) = hi;     // X^T[c = n][r = m0 ..]
        *reinterpret_cast<uint2*>(Pn + hoff + (int64_t)n * DH + m0) = thi;    // accT: X[r = n][c = m0 ..]
      }
    }

  if constexpr (CLOSE) {
    // ---- the closing step of the update in the same launch (Sec. 3.3; the general path's sequence of Gram matrix, D^2,
    // correction product and finishing pass, with the same operand planes): D = (I - X^T X)/2 from the exact bf16 iterate,
    // X <- X + X (D + 1.5 D^2) with the correction as two bf16 planes, then R, the rotate operand R^T and <R, M>.
    // The step is taken only if this head's residual allows the quintic form (cl.res_max); otherwise the head reports
    // its residual, marks the step as not taken (sq_out < 0) and the host continues on the general path from the
    // hand-over state written above.
    unsigned char* const sD0 = sW;                    // first plane of D, then of the correction
    unsigned char* const sD1 = smem + 3 * DH * ROWB;  // second plane
    __shared__ double red[3][4];
    // bf16 planes of a symmetric matrix given as accumulator blocks: the transposed store of block (wm, wn) is block
    // (wn, wm) of the matrix itself
    auto store_planes = [&](const f32x16 (&v)[2][2]) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int n = 64 * wn + 32 * j + col;
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const int m0 = 64 * wm + 32 * i + 8 * jj + 4 * half;
            uint2 h0, h1;
            h0.x = f32x2_to_bf16x2(v[i][j][4 * jj], v[i][j][4 * jj + 1]);
            h0.y = f32x2_to_bf16x2(v[i][j][4 * jj + 2], v[i][j][4 * jj + 3]);
            h1.x = f32x2_to_bf16x2(v[i][j][4 * jj] - __uint_as_float(h0.x << 16), v[i][j][4 * jj + 1] - __uint_as_float(h0.x & 0xffff0000u));
            h1.y = f32x2_to_bf16x2(v[i][j][4 * jj + 2] - __uint_as_float(h0.y << 16), v[i][j][4 * jj + 3] - __uint_as_float(h0.y & 0xffff0000u));
            *reinterpret_cast<uint2*>(sD0 + loff(n, m0 >> 3) + (m0 & 7) * 2) = h0;
            *reinterpret_cast<uint2*>(sD1 + loff(n, m0 >> 3) + (m0 & 7) * 2) = h1;
          }
        }
    };
    auto product_bf16 = [&](const unsigned char* A, int rowA, const unsigned char* Bm, int rowB, f32x16 (&out)[2][2]) {
#pragma unroll
      for (int kk = 0; kk < DH / 16; ++kk) {
        bf16x8 fa[2], fb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(A + loff(rowA + 32 * i + col, 2 * kk + half));
#pragma unroll
        for (int j = 0; j < 2; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(Bm + loff(rowB + 32 * j + col, 2 * kk + half));
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) out[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], out[i][j], 0, 0, 0);
      }
    };
    auto zero = [](f32x16 (&v)[2][2]) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) v[i][j][e] = 0.0f;
    };
    // sum of one double per lane over the workgroup, known to every thread afterwards
    auto block_sum = [&](double v, int slot) {
      v = wave_sum_d(v);
      if (lane == 0) red[slot][wave] = v;
      __syncthreads();
      return red[slot][0] + red[slot][1] + red[slot][2] + red[slot][3];
    };

    __syncthreads();   // every wavefront has finished the last step's reads of the old iterate and of W
    // the rounded iterate as bf16 operands: X^T from X', X from X'^T (packed 8-byte writes both)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = 64 * wn + 32 * j + col;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int m0 = 64 * wm + 32 * i + 8 * jj + 4 * half;
          uint2 a, t;
          a.x = f32x2_to_bf16x2(acc[i][j][4 * jj], acc[i][j][4 * jj + 1]);
          a.y = f32x2_to_bf16x2(acc[i][j][4 * jj + 2], acc[i][j][4 * jj + 3]);
          t.x = f32x2_to_bf16x2(accT[i][j][4 * jj], accT[i][j][4 * jj + 1]);
          t.y = f32x2_to_bf16x2(accT[i][j][4 * jj + 2], accT[i][j][4 * jj + 3]);
          *reinterpret_cast<uint2*>(sXt + loff(n, m0 >> 3) + (m0 & 7) * 2) = a;
          *reinterpret_cast<uint2*>(sXn + loff(n, m0 >> 3) + (m0 & 7) * 2) = t;
        }
      }
    __syncthreads();
    // G = X^T X (products of bf16 values are exact in fp32), D = (I - G) / 2, ||I - G||_F^2
    f32x16 dm[2][2];
    zero(dm);
    product_bf16(sXt, 64 * wm, sXt, 64 * wn, dm);
    double part = 0.0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        float p32 = 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int m = 64 * wm + 32 * i + 8 * (e >> 2) + 4 * half + (e & 3), n = 64 * wn + 32 * j + col;
          const float dlt = (m == n ? 1.0f : 0.0f) - dm[i][j][e];
          p32 += dlt * dlt;
          dm[i][j][e] = 0.5f * dlt;
        }
        part += (double)p32;
      }
    const double res2 = block_sum(part, 0);
    if (!(res2 <= (double)cl.res_max * cl.res_max)) {   // (also a non-finite residual)
      if (tid == 0) { cl.res_out[h] = res2; cl.sq_out[h] = -1.0; }
      return;
    }
    store_planes(dm);
    __syncthreads();
    // D^2 from the first plane (second-order small: one plane is ample), ||D^2||_F^2, the correction D + 1.5 D^2
    f32x16 sq[2][2];
    zero(sq);
    product_bf16(sD0, 64 * wm, sD0, 64 * wn, sq);
    part = 0.0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        float p32 = 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          p32 += sq[i][j][e] * sq[i][j][e];
          dm[i][j][e] += 1.5f * sq[i][j][e];
        }
        part += (double)p32;
      }
    const double sq2 = block_sum(part, 1);   // (its barrier: every wavefront has read the planes of D)
    store_planes(dm);
    __syncthreads();
    // X <- X + X (W0 + W1).  The small correction is summed on its own and the iterate added once at the end: with the
    // iterate as the accumulators' start every one of the 16 MFMAs would round at the iterate's magnitude, and the
    // orthogonality of the result was measured above the bound that holds for the general path's order.
    zero(sq);
    product_bf16(sXn, 64 * wm, sD0, 64 * wn, sq);
    product_bf16(sXn, 64 * wm, sD1, 64 * wn, sq);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] += sq[i][j][e];
    // R, the rotate operand R^T (bf16, [n][m]: packed rows of the transposed matrix) and <R, M>
    part = 0.0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = 64 * wn + 32 * j + col;
        float p32 = 0.0f;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int m0 = 64 * wm + 32 * i + 8 * jj + 4 * half;
          uint2 r;
          r.x = f32x2_to_bf16x2(acc[i][j][4 * jj], acc[i][j][4 * jj + 1]);
          r.y = f32x2_to_bf16x2(acc[i][j][4 * jj + 2], acc[i][j][4 * jj + 3]);
          *reinterpret_cast<uint2*>(cl.RopT + hoff + (int64_t)n * DH + m0) = r;
#pragma unroll
          for (int ii = 0; ii < 4; ++ii) {
            const int64_t off = hoff + (int64_t)(m0 + ii) * DH + n;
            cl.R[off] = acc[i][j][4 * jj + ii];
            p32 += acc[i][j][4 * jj + ii] * cl.M[off];
          }
        }
        part += (double)p32;
      }
    const double inner = block_sum(part, 2);
    if (tid == 0) { cl.res_out[h] = res2; cl.sq_out[h] = sq2; cl.inner_out[h] = inner; }
  }
}

}  // namespace

hipError_t launch_head_polar128(const bf16_bits* Xn0, const bf16_bits* Xt0, int heads, const PolarSchedule& sched, float* X32,
                                bf16_bits* Pn, bf16_bits* Pt, const HeadPolarClose* close, const HeadPolarStart* start,
                                hipStream_t s) {
  if (heads < 1 || sched.nsteps < 1 || sched.nsteps > kPolarScheduleMax) return hipErrorInvalidValue;
  if (close && (!close->R || !close->RopT || !close->M || !close->res_out || !close->sq_out || !close->inner_out)) return hipErrorInvalidValue;
  if (start && (!start->M || !start->R || !start->fro2_parts || start->nparts < 1 || !start->fro2_out || (start->ldot && !start->L)))
    return hipErrorInvalidValue;
  if (!start && (!Xn0 || !Xt0)) return hipErrorInvalidValue;
  static PerDeviceOnce configured;
  hipError_t e = configured.run([] {
    hipError_t r = hipFuncSetAttribute(reinterpret_cast<const void*>(k_head_polar128<false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kSmemBytes);
    if (r == hipSuccess)
      r = hipFuncSetAttribute(reinterpret_cast<const void*>(k_head_polar128<true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                              kSmemBytesClose);
    return r;
  });
  if (e != hipSuccess) return e;
  const HeadPolarStart st = start ? *start : HeadPolarStart{};
  if (close)
    hipLaunchKernelGGL(k_head_polar128<true>, dim3(heads), dim3(256), kSmemBytesClose, s, Xn0, Xt0, sched, X32, Pn, Pt, *close, st);
  else
    hipLaunchKernelGGL(k_head_polar128<false>, dim3(heads), dim3(256), kSmemBytes, s, Xn0, Xt0, sched, X32, Pn, Pt, HeadPolarClose{}, st);
  return hipGetLastError();
}

}  // namespace conqur
