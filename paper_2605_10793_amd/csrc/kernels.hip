// Non-GEMM kernels of the calibration path (see kernels.h).
#include "kernels.h"

#include <type_traits>

namespace conqur {

namespace {

__device__ __forceinline__ void unpack8(const uint4& v, float* f) {
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
  f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
  f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}

// bf16 split of an fp32 value: x ~= p0 + p1 + p2 (exact for 24-bit significands).
template <int NP>
__device__ __forceinline__ void split_bf16(float x, bf16_bits* p) {
  float r = x;
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    p[i] = f32_to_bf16(r);
    r -= bf16_to_f32(p[i]);
  }
}

__device__ __forceinline__ double block_sum_d(double v, double* sh) {
  v = wave_sum_d(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int i = 0; i < (int)(blockDim.x >> 6); ++i) t += sh[i];   // sh holds one entry per wavefront
  return t;
}

// ---------------------------------------------------------------- row norms
template <bool F32>
__global__ void __launch_bounds__(256) k_row_norms(const void* __restrict__ X, int64_t T, int64_t stride, int heads, int dh,
                                                   float* __restrict__ nrm, float* __restrict__ w, int64_t ldn,
                                                   int* __restrict__ nonfinite) {
  const int64_t gw = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (gw >= T * heads) return;
  const int64_t i = gw / heads;
  const int h = (int)(gw - i * heads);
  float ss = 0.0f;
  if constexpr (F32) {
    // four independent 16-byte loads per lane in flight (a row is read once, so the loop is latency bound otherwise)
    const float* x = reinterpret_cast<const float*>(X) + i * stride + (int64_t)h * dh;
    const int nc = dh / 4;
    for (int c0 = lane; c0 < nc; c0 += 256) {
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = c0 + u * 64;
        v[u] = c < nc ? *reinterpret_cast<const float4*>(x + c * 4) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) ss += v[u].x * v[u].x + v[u].y * v[u].y + v[u].z * v[u].z + v[u].w * v[u].w;
    }
  } else {
    // eight independent 16-byte loads per lane in flight: a head slice of 4096 bf16 is one round trip to memory
    const bf16_bits* x = reinterpret_cast<const bf16_bits*>(X) + i * stride + (int64_t)h * dh;
    const int nc = dh / 8;
    for (int c0 = lane; c0 < nc; c0 += 512) {
      uint4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int c = c0 + u * 64;
        v[u] = c < nc ? *reinterpret_cast<const uint4*>(x + c * 8) : make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        float f[8];
        unpack8(v[u], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
      }
    }
  }
  ss = wave_sum(ss);
  if (lane == 0) {
    float n = 0.0f, wi = 0.0f;
    if (!isfinite(ss)) {
      atomicOr(nonfinite, 1);
    } else if (ss > 0.0f) {
      n = sqrtf(ss);
      wi = kXhatScale / n;
    }
    nrm[(int64_t)h * ldn + i] = n;
    w[(int64_t)h * ldn + i] = wi;
  }
}

// ---------------------------------------------------------------- scaled transpose
template <bool F32, int NP>
__global__ void __launch_bounds__(256) k_transpose_scale(const void* __restrict__ X, int64_t T, int64_t stride, int d, int dh,
                                                         const float* __restrict__ w, int64_t ldn,
                                                         bf16_bits* __restrict__ Xt, int64_t pitch, int64_t plane,
                                                         unsigned long long* __restrict__ cnt) {
  // bf16 input: the tile holds the finished fp16 values (8.3 KiB, so that this kernel's workgroups still fit
  // beside a GEMM workgroup that owns 144 KiB of the CU's LDS); fp32 input: fp32 values, split after the transpose
  using TileT = typename std::conditional<NP == 1, bf16_bits, float>::type;
  __shared__ TileT tile[64][NP == 1 ? 66 : 65];
  const int64_t i0 = (int64_t)blockIdx.x * 64;
  const int k0 = blockIdx.y * 64;
  const int t = threadIdx.x;
  if (t < 64) {
    // The workgroup that holds a head's first column also counts that head's rows (entered M / skipped) among its 64
    // tokens: two ballots by one wavefront, added to one of kCountSlots slots per head so that a batch's atomics
    // spread over many addresses (atomics from all XCDs on one address serialise).
    for (int h = (k0 + dh - 1) / dh; h * dh < k0 + 64 && h * dh < d; ++h) {
      const int64_t i = i0 + t;
      const float wv = i < T ? w[(int64_t)h * ldn + i] : 0.0f;
      const unsigned long long in = __ballot(i < T && wv != 0.0f), out = __ballot(i < T && wv == 0.0f);
      if (t == 0) {
        unsigned long long* slot = cnt + ((int64_t)h * kCountSlots + (blockIdx.x % kCountSlots)) * 2;
        if (in) atomicAdd(slot, (unsigned long long)__popcll(in));
        if (out) atomicAdd(slot + 1, (unsigned long long)__popcll(out));
      }
    }
  }
  {
    const int c = t & 7;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int r = (t >> 3) + pass * 32;
      const int64_t i = i0 + r;
      const int k = k0 + c * 8;
      float f[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = 0.0f;
      if (i < T && k < d) {
        const float wi = w[(int64_t)(k / dh) * ldn + i];
        if constexpr (F32) {
          const float* x = reinterpret_cast<const float*>(X) + i * stride + k;
          const float4 a = *reinterpret_cast<const float4*>(x), b = *reinterpret_cast<const float4*>(x + 4);
          f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
        } else {
          unpack8(*reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_bits*>(X) + i * stride + k), f);
        }
        // a skipped row has w = 0; its values may be Inf/NaN, so select instead of multiplying
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = (wi != 0.0f) ? f[e] * wi : 0.0f;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if constexpr (NP == 1) tile[r][c * 8 + e] = f32_to_f16(f[e]);   // |x^| kXhatScale <= 64: fp16 keeps 11 significant bits
        else tile[r][c * 8 + e] = f[e];
      }
    }
  }
  __syncthreads();
  {
    const int tc = t & 7;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int kl = (t >> 3) + pass * 32;
      const int k = k0 + kl;
      if (k >= d) continue;
      bf16_bits out[NP][8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if constexpr (NP == 1) {
          out[0][e] = tile[tc * 8 + e][kl];
        } else {
          bf16_bits p[NP];
          split_bf16<NP>(tile[tc * 8 + e][kl], p);
#pragma unroll
          for (int q = 0; q < NP; ++q) out[q][e] = p[q];
        }
      }
#pragma unroll
      for (int q = 0; q < NP; ++q) {
        uint4 v;
        v.x = out[q][0] | ((uint32_t)out[q][1] << 16); v.y = out[q][2] | ((uint32_t)out[q][3] << 16);
        v.z = out[q][4] | ((uint32_t)out[q][5] << 16); v.w = out[q][6] | ((uint32_t)out[q][7] << 16);
        *reinterpret_cast<uint4*>(Xt + q * plane + (int64_t)k * pitch + i0 + tc * 8) = v;
      }
    }
  }
}

// ---------------------------------------------------------------- fp32 rows -> 3 bf16 planes
__global__ void __launch_bounds__(256) k_split_rows(const float* __restrict__ X, int64_t T, int64_t stride, int d,
                                                    bf16_bits* __restrict__ Xs, int64_t plane) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // one per 4 elements
  const int per_row = d / 4;
  if (idx >= T * per_row) return;
  const int64_t i = idx / per_row;
  const int k = (int)(idx - i * per_row) * 4;
  const float4 v = *reinterpret_cast<const float4*>(X + i * stride + k);
  const float f[4] = {v.x, v.y, v.z, v.w};
  bf16_bits p[4][3];
#pragma unroll
  for (int e = 0; e < 4; ++e) split_bf16<3>(f[e], p[e]);
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    uint2 o;
    o.x = p[0][q] | ((uint32_t)p[1][q] << 16);
    o.y = p[2][q] | ((uint32_t)p[3][q] << 16);
    *reinterpret_cast<uint2*>(Xs + q * plane + i * d + k) = o;
  }
}

// ---------------------------------------------------------------- fp32 matrix -> bf16 planes (natural / transposed)
// One 64 x 64 tile per workgroup.  Optional fused work, so that the matrix is read once:
//   START: the value packed is X0 = cm * src + cr * src2 (start of the polar iteration: src = M, src2 = R_prev,
//          cm = 1/alpha, cr = lambda tau / alpha from fro2 = ||M||_F^2 of this batch entry);
//   DOT:   also the partial sum over the tile of value * dotwith (the inner product <X, M>), one per workgroup;
//   out32: also the value itself in fp32.
struct PackFused {
  const float* src2;      // START
  const double* fro2;     // START
  float lambda;           // START
  int dh;                 // START (tau = ||M||_F / sqrt(dh))
  const float* dotwith;   // DOT
  double* dot_part;       // DOT: [batch][gridDim.y * gridDim.x]; START: same for <R_op, M>, or null
  int round_bf16;         // START: R_op is src2 rounded to bf16
  float* out32;           // may be null
  int out_f16;            // NP == 1 only: the plane holds fp16 instead of bf16
};

template <int NP, bool START, bool DOT>
__global__ void __launch_bounds__(256) k_pack(const float* __restrict__ src, int rows, int cols, bf16_bits* __restrict__ outN,
                                              bf16_bits* __restrict__ outT, int64_t plane, const PackFused fx) {
  __shared__ float tile[64][65];
  __shared__ double sh[4];
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  const int64_t boff = (int64_t)blockIdx.z * rows * cols;
  const int t = threadIdx.x;
  float cm = 1.0f, cr = 0.0f;
  if constexpr (START) {
    const double f = sqrt(fx.fro2[blockIdx.z]);
    const bool empty = !(f > 0.0);
    // lambda = 0 is taken as the limit lambda -> 0+ at fp32 resolution: the floor ties the
    // update to R_prev on the null space of M (where every completion is optimal) and
    // breaks exact degeneracies (repeated columns of M) that the iteration would preserve.
    const float lambda = fmaxf(fx.lambda, 9.5367431640625e-07f);
    const float tau = (float)(f / sqrt((double)fx.dh));
    const float inv_alpha = empty ? 1.0f : (float)(1.0 / (f * (1.0 + (double)lambda)));
    cm = empty ? 0.0f : inv_alpha;
    cr = empty ? 1.0f : lambda * tau * inv_alpha;
  }
  double dot = 0.0;
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int r = (t >> 4) + pass * 16;
    const int c = (t & 15) * 4;
    float f[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (r0 + r < rows && c0 + c < cols) {
      const int64_t off = boff + (int64_t)(r0 + r) * cols + c0 + c;
      const float4 v = *reinterpret_cast<const float4*>(src + off);
      f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
      if constexpr (START) {
        float4 w = *reinterpret_cast<const float4*>(fx.src2 + off);
        const float m4[4] = {f[0], f[1], f[2], f[3]};
        f[0] = cm * f[0] + cr * w.x; f[1] = cm * f[1] + cr * w.y; f[2] = cm * f[2] + cr * w.z; f[3] = cm * f[3] + cr * w.w;
        if (fx.dot_part) {   // <R_op, M> on the way (the l1 term of the rows this update consumes; see k_dot_rm)
          if (fx.round_bf16) {
            w.x = bf16_to_f32(f32_to_bf16(w.x)); w.y = bf16_to_f32(f32_to_bf16(w.y));
            w.z = bf16_to_f32(f32_to_bf16(w.z)); w.w = bf16_to_f32(f32_to_bf16(w.w));
          }
          dot += (double)m4[0] * w.x + (double)m4[1] * w.y + (double)m4[2] * w.z + (double)m4[3] * w.w;
        }
      }
      if constexpr (DOT) {
        const float4 m = *reinterpret_cast<const float4*>(fx.dotwith + off);
        dot += (double)f[0] * m.x + (double)f[1] * m.y + (double)f[2] * m.z + (double)f[3] * m.w;
      }
      if (fx.out32) *reinterpret_cast<float4*>(fx.out32 + off) = make_float4(f[0], f[1], f[2], f[3]);
      if (outN) {
        bf16_bits p[4][NP];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (NP == 1 && fx.out_f16) p[e][0] = f32_to_f16(f[e]);
          else split_bf16<NP>(f[e], p[e]);
        }
#pragma unroll
        for (int q = 0; q < NP; ++q) {
          uint2 o;
          o.x = p[0][q] | ((uint32_t)p[1][q] << 16);
          o.y = p[2][q] | ((uint32_t)p[3][q] << 16);
          *reinterpret_cast<uint2*>(outN + q * plane + off) = o;
        }
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) tile[r][c + e] = f[e];
  }
  if (DOT || (START && fx.dot_part)) {
    dot = block_sum_d(dot, sh);
    if (t == 0) fx.dot_part[((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x] = dot;
  }
  if (!outT) return;
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int cl = (t >> 3) + pass * 32;
    const int rc = (t & 7) * 8;
    if (c0 + cl >= cols || r0 + rc >= rows) continue;
    bf16_bits p[8][NP];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (NP == 1 && fx.out_f16) p[e][0] = f32_to_f16(tile[rc + e][cl]);
      else split_bf16<NP>(tile[rc + e][cl], p[e]);
    }
#pragma unroll
    for (int q = 0; q < NP; ++q) {
      uint4 v;
      v.x = p[0][q] | ((uint32_t)p[1][q] << 16); v.y = p[2][q] | ((uint32_t)p[3][q] << 16);
      v.z = p[4][q] | ((uint32_t)p[5][q] << 16); v.w = p[6][q] | ((uint32_t)p[7][q] << 16);
      *reinterpret_cast<uint4*>(outT + q * plane + boff + (int64_t)(c0 + cl) * rows + r0 + rc) = v;
    }
  }
}

// ---------------------------------------------------------------- statistics
// part[h][block] = sum over the block's elements of M_h * R_op,h, with R_op = R rounded to bf16 (bf16 activations) or R
// itself.  The l1 term of the accumulated rows is sqrt(dh) <R_op, M>: sum_i ||y_i||_1 / ||x_i|| = sum_i sum_n
// sgn(y_in) y_in / ||x_i|| with y_i = x_i R_op and M = sum_i (x_i/||x_i||)^T sgn(y_i)/sqrt(dh) (the l1 identity of
// Sec. 3.2 per site), as long as every row was rotated with this R_op.
__global__ void __launch_bounds__(256) k_dot_rm(const float* __restrict__ R, const float* __restrict__ M, int64_t n, int round_bf16,
                                                double* __restrict__ part) {
  __shared__ double sh[4];
  const int64_t hoff = (int64_t)blockIdx.y * n;
  double acc = 0.0;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4; i < n; i += (int64_t)gridDim.x * 1024) {
    float4 r = *reinterpret_cast<const float4*>(R + hoff + i);
    const float4 m = *reinterpret_cast<const float4*>(M + hoff + i);
    if (round_bf16) {
      r.x = bf16_to_f32(f32_to_bf16(r.x)); r.y = bf16_to_f32(f32_to_bf16(r.y));
      r.z = bf16_to_f32(f32_to_bf16(r.z)); r.w = bf16_to_f32(f32_to_bf16(r.w));
    }
    acc += (double)r.x * m.x + (double)r.y * m.y + (double)r.z * m.z + (double)r.w * m.w;
  }
  acc = block_sum_d(acc, sh);
  if (threadIdx.x == 0) part[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = acc;
}

__global__ void __launch_bounds__(256) k_fro2(const float* __restrict__ M, int64_t n, double* __restrict__ part) {
  __shared__ double sh[4];
  const float* m = M + (int64_t)blockIdx.y * n;
  double acc = 0.0;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4; i < n; i += (int64_t)gridDim.x * 1024) {
    const float4 v = *reinterpret_cast<const float4*>(m + i);
    acc += (double)v.x * v.x + (double)v.y * v.y + (double)v.z * v.z + (double)v.w * v.w;
  }
  acc = block_sum_d(acc, sh);
  if (threadIdx.x == 0) part[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = acc;   // summed in a fixed order afterwards
}

__global__ void __launch_bounds__(256) k_axpy(float* __restrict__ X, const float* __restrict__ R, int64_t n, float kappa) {
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4; i < n; i += (int64_t)gridDim.x * 1024) {
    float4 x = *reinterpret_cast<float4*>(X + i);
    const float4 r = *reinterpret_cast<const float4*>(R + i);
    x.x += kappa * r.x; x.y += kappa * r.y; x.z += kappa * r.z; x.w += kappa * r.w;
    *reinterpret_cast<float4*>(X + i) = x;
  }
}

// ---------------------------------------------------------------- fake-quantisation error
// One workgroup per token row: the row is read once from HBM with 16-byte loads and kept
// in registers (4 chunks per thread = 8192 bf16 / 4096 fp32 elements; longer rows re-read
// the tail, which then comes from cache).  Two barriers per row (maximum, sums); per-row
// results go to row_sse / row_en.
// ZP: the zero-point quantiser of App. B instead of the symmetric one: range [clip*min, clip*max] on the unsigned grid
// {0 .. qmax}, D = range / qmax, integer zero point zeta = -rint(lo / D), code = clamp(rint(y / D) + zeta, 0, qmax).
// EMIT: the quantised rows q are also written out in the activation dtype (Q, row stride ldq): what a linear layer with
// quantised input receives during quantisation-aware calibration (Sec. 3.4).
template <bool F32, bool ZP, bool EMIT>
__global__ void __launch_bounds__(256) k_quant_error(const void* __restrict__ Y, int64_t T, int64_t ld, int d, float qmax,
                                                     float clip, float* __restrict__ row_sse, float* __restrict__ row_en,
                                                     void* __restrict__ Q, int64_t ldq) {
  constexpr int EPC = F32 ? 4 : 8;  // elements per 16-byte chunk
  constexpr int NC = 4;             // chunks cached per thread
  __shared__ float shm[4], shn[4], shs[4], she[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = blockIdx.x;
  const int nch = d / EPC;
  auto expand = [](const uint4& v, float* f) {
    if constexpr (F32) {
      f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    } else {
      unpack8(v, f);
    }
  };
  const uint4* y = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(Y) + row * ld * (F32 ? 4 : 2));
  uint4 cache[NC];
  // symmetric: amax = max |y|.  ZP: amax = max y, amin = -min y (both start from the row's first element)
  float amax = 0.0f, amin = 0.0f;
  if constexpr (ZP) {
    float f[EPC];
    expand(y[0], f);
    amax = f[0];
    amin = -f[0];
  }
  auto track = [&](const uint4& v) {
    float f[EPC];
    expand(v, f);
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
      if constexpr (ZP) {
        amax = fmaxf(amax, f[e]);
        amin = fmaxf(amin, -f[e]);
      } else {
        amax = fmaxf(amax, fabsf(f[e]));
      }
    }
  };
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    const int c = threadIdx.x + 256 * q;
    cache[q] = make_uint4(0, 0, 0, 0);
    if (c < nch) {
      cache[q] = y[c];
      track(cache[q]);
    }
  }
  for (int c = threadIdx.x + 256 * NC; c < nch; c += 256) track(y[c]);
  amax = wave_max(amax);
  if constexpr (ZP) amin = wave_max(amin);
  if (lane == 0) { shm[wave] = amax; shn[wave] = amin; }
  __syncthreads();
  amax = fmaxf(fmaxf(shm[0], shm[1]), fmaxf(shm[2], shm[3]));
  if constexpr (ZP) amin = fmaxf(fmaxf(shn[0], shn[1]), fmaxf(shn[2], shn[3]));
  // D = max / qmax; the code is decided in fp32 as round-half-even(y * (1/D)) with the
  // correctly rounded reciprocal (a division per element would make this kernel
  // ALU bound instead of HBM bound); it can differ from round(y / D) only within an
  // ulp of a rounding tie, where both codes give the same squared error.
  float delta, inv_delta, zeta = 0.0f, lo = 0.0f;
  if constexpr (ZP) {
    lo = clip * -amin;
    const float hi = clip * amax;
    delta = (hi - lo) / qmax;
    inv_delta = delta > 0.0f ? 1.0f / delta : 0.0f;
    zeta = delta > 0.0f ? -rintf(lo / delta) : 0.0f;
  } else {
    delta = amax / qmax;
    inv_delta = amax > 0.0f ? 1.0f / delta : 0.0f;
  }
  float sse = 0.0f, en = 0.0f;
  uint4* const qrow = EMIT ? reinterpret_cast<uint4*>(reinterpret_cast<char*>(Q) + row * ldq * (F32 ? 4 : 2)) : nullptr;
  auto score = [&](const uint4& v, int c) {
    float f[EPC], qv[EPC];
    expand(v, f);
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
      float err;
      if constexpr (ZP) {
        const float code = fminf(fmaxf(rintf(f[e] * inv_delta) + zeta, 0.0f), qmax);
        // a constant row (delta = 0) has the single level lo
        err = delta > 0.0f ? fmaf(-delta, code - zeta, f[e]) : f[e] - lo;
        qv[e] = delta > 0.0f ? delta * (code - zeta) : lo;
      } else {
        const float code = fminf(fmaxf(rintf(f[e] * inv_delta), -qmax), qmax);
        err = fmaf(-delta, code, f[e]);
        qv[e] = delta * code;
      }
      sse = fmaf(err, err, sse);
      en = fmaf(f[e], f[e], en);
    }
    if constexpr (EMIT) {
      uint4 o;
      if constexpr (F32) {
        o = make_uint4(__float_as_uint(qv[0]), __float_as_uint(qv[1]), __float_as_uint(qv[2]), __float_as_uint(qv[3]));
      } else {
        o = make_uint4(f32x2_to_bf16x2(qv[0], qv[1]), f32x2_to_bf16x2(qv[2], qv[3]), f32x2_to_bf16x2(qv[4], qv[5]),
                       f32x2_to_bf16x2(qv[6], qv[7]));
      }
      qrow[c] = o;
    }
  };
#pragma unroll
  for (int q = 0; q < NC; ++q)
    if ((int)threadIdx.x + 256 * q < nch) score(cache[q], (int)threadIdx.x + 256 * q);
  for (int c = threadIdx.x + 256 * NC; c < nch; c += 256) score(y[c], c);
  sse = wave_sum(sse);
  en = wave_sum(en);
  if (lane == 0) { shs[wave] = sse; she[wave] = en; }
  __syncthreads();
  if (threadIdx.x == 0) {
    row_sse[row] = (float)((double)shs[0] + (double)shs[1] + (double)shs[2] + (double)shs[3]);
    row_en[row] = (float)((double)she[0] + (double)she[1] + (double)she[2] + (double)she[3]);
  }
}

// ---------------------------------------------------------------- row diagnostics
// One workgroup per row of Y, same single pass as k_quant_error (row cached in registers): pr = ||y||_2^4 / (d ||y||_4^4)
// (normalised participation ratio, Sec. 4.2) and rho = ||y||_inf^2 / ||y||_2^2 (App. B).  The sums run over u = y / max|y|,
// so that fourth powers neither overflow nor vanish; a row with zero or non-finite energy gets 0, 0.
template <bool F32>
__global__ void __launch_bounds__(256) k_row_diag(const void* __restrict__ Y, int64_t T, int64_t ld, int d,
                                                  float* __restrict__ row_pr, float* __restrict__ row_rho) {
  constexpr int EPC = F32 ? 4 : 8;
  constexpr int NC = 4;
  __shared__ float shm[4], sh2[4], sh4[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = blockIdx.x;
  const int nch = d / EPC;
  auto expand = [](const uint4& v, float* f) {
    if constexpr (F32) {
      f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    } else {
      unpack8(v, f);
    }
  };
  const uint4* y = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(Y) + row * ld * (F32 ? 4 : 2));
  uint4 cache[NC];
  float amax = 0.0f;
  auto track = [&](const uint4& v) {
    float f[EPC];
    expand(v, f);
#pragma unroll
    for (int e = 0; e < EPC; ++e) amax = fmaxf(amax, fabsf(f[e]));   // fmaxf drops NaN: caught through the sums below
  };
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    const int c = threadIdx.x + 256 * q;
    cache[q] = make_uint4(0, 0, 0, 0);
    if (c < nch) {
      cache[q] = y[c];
      track(cache[q]);
    }
  }
  for (int c = threadIdx.x + 256 * NC; c < nch; c += 256) track(y[c]);
  amax = wave_max(amax);
  if (lane == 0) shm[wave] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(shm[0], shm[1]), fmaxf(shm[2], shm[3]));
  const float inv = (amax > 0.0f && isfinite(amax)) ? 1.0f / amax : 0.0f;
  float s2 = 0.0f, s4 = 0.0f;
  auto score = [&](const uint4& v) {
    float f[EPC];
    expand(v, f);
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
      const float u = f[e] * inv, u2 = u * u;
      s2 += u2;
      s4 = fmaf(u2, u2, s4);
    }
  };
#pragma unroll
  for (int q = 0; q < NC; ++q)
    if ((int)threadIdx.x + 256 * q < nch) score(cache[q]);
  for (int c = threadIdx.x + 256 * NC; c < nch; c += 256) score(y[c]);
  s2 = wave_sum(s2);
  s4 = wave_sum(s4);
  if (lane == 0) { sh2[wave] = s2; sh4[wave] = s4; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const double t2 = (double)sh2[0] + (double)sh2[1] + (double)sh2[2] + (double)sh2[3];
    const double t4 = (double)sh4[0] + (double)sh4[1] + (double)sh4[2] + (double)sh4[3];
    const bool ok = inv > 0.0f && t2 > 0.0 && isfinite(t2) && t4 > 0.0;
    row_pr[row] = ok ? (float)(t2 * t2 / ((double)d * t4)) : 0.0f;
    row_rho[row] = ok ? (float)(1.0 / t2) : 0.0f;
  }
}

// out[0] = sum a, out[1] = sum b in a fixed order (one workgroup).  Results of many
// workgroups are combined this way rather than with atomics on one address, which the
// XCDs would serialise at the memory side.
__global__ void __launch_bounds__(1024) k_sum_rows(const float* __restrict__ a, const float* __restrict__ b, int64_t T,
                                                   double* __restrict__ out) {
  __shared__ double sh[16];
  double sa = 0.0, sb = 0.0;
  for (int64_t i = threadIdx.x; i < T; i += 1024) {
    sa += (double)a[i];
    sb += (double)b[i];
  }
  sa = block_sum_d(sa, sh);
  sb = block_sum_d(sb, sh);
  if (threadIdx.x == 0) {
    out[0] = sa;
    out[1] = sb;
  }
}

// out[h] = sum_i part[h][i], i < n (one workgroup per h).
__global__ void __launch_bounds__(256) k_sum_partials(const double* __restrict__ part, int n, double* __restrict__ out) {
  __shared__ double sh[4];
  const double* p = part + (int64_t)blockIdx.x * n;
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) s += p[i];
  s = block_sum_d(s, sh);
  if (threadIdx.x == 0) out[blockIdx.x] = s;
}

__global__ void __launch_bounds__(256) k_fill_zero(uint32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

inline int grid_for(int64_t items, int cap = 4096) {
  int64_t g = (items + 255) / 256;
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return (int)g;
}

}  // namespace

hipError_t launch_row_norms(const void* X, int x_is_f32, int64_t T, int64_t stride, int heads, int dh, float* nrm, float* w,
                            int64_t ldn, int* nonfinite, hipStream_t s) {
  const int64_t waves = T * heads;
  dim3 grid((unsigned)((waves + 3) / 4));
  if (x_is_f32)
    hipLaunchKernelGGL(k_row_norms<true>, grid, dim3(256), 0, s, X, T, stride, heads, dh, nrm, w, ldn, nonfinite);
  else
    hipLaunchKernelGGL(k_row_norms<false>, grid, dim3(256), 0, s, X, T, stride, heads, dh, nrm, w, ldn, nonfinite);
  return hipGetLastError();
}

hipError_t launch_transpose_scale(const void* X, int x_is_f32, int64_t T, int64_t Tk, int64_t stride, int d, int dh,
                                  const float* w, int64_t ldn, bf16_bits* Xt, int64_t pitch, int64_t plane, int np,
                                  unsigned long long* cnt, hipStream_t s) {
  dim3 grid((unsigned)(Tk / 64), (unsigned)((d + 63) / 64));
  if (x_is_f32 && np == 3)
    hipLaunchKernelGGL((k_transpose_scale<true, 3>), grid, dim3(256), 0, s, X, T, stride, d, dh, w, ldn, Xt, pitch, plane, cnt);
  else if (!x_is_f32 && np == 1)
    hipLaunchKernelGGL((k_transpose_scale<false, 1>), grid, dim3(256), 0, s, X, T, stride, d, dh, w, ldn, Xt, pitch, plane, cnt);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_split_rows(const float* X, int64_t T, int64_t stride, int d, bf16_bits* Xs, int64_t plane, hipStream_t s) {
  const int64_t items = T * (d / 4);
  hipLaunchKernelGGL(k_split_rows, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, s, X, T, stride, d, Xs, plane);
  return hipGetLastError();
}

template <bool START, bool DOT>
static hipError_t launch_pack_impl(const float* src, int batch, int rows, int cols, int np, bf16_bits* outN, bf16_bits* outT,
                                   int64_t plane, const PackFused& fx, hipStream_t s) {
  dim3 grid((cols + 63) / 64, (rows + 63) / 64, batch);
  switch (np) {
    case 1: hipLaunchKernelGGL((k_pack<1, START, DOT>), grid, dim3(256), 0, s, src, rows, cols, outN, outT, plane, fx); break;
    case 2: hipLaunchKernelGGL((k_pack<2, START, DOT>), grid, dim3(256), 0, s, src, rows, cols, outN, outT, plane, fx); break;
    case 3: hipLaunchKernelGGL((k_pack<3, START, DOT>), grid, dim3(256), 0, s, src, rows, cols, outN, outT, plane, fx); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_pack(const float* src, int batch, int rows, int cols, int np, bf16_bits* outN, bf16_bits* outT,
                       int64_t plane, hipStream_t s, int out_f16) {
  if (out_f16 && np != 1) return hipErrorInvalidValue;
  PackFused fx{};
  fx.out_f16 = out_f16;
  return launch_pack_impl<false, false>(src, batch, rows, cols, np, outN, outT, plane, fx, s);
}

int pack_dot_partials(int dh) { return ((dh + 63) / 64) * ((dh + 63) / 64); }

hipError_t launch_polar_start_pack(const float* M, const float* R, int heads, int dh, float lambda, const double* fro2, int np,
                                   float* X32, bf16_bits* outN, bf16_bits* outT, int64_t plane, int round_bf16,
                                   double* dot_part, double* dot_out, hipStream_t s, int out_f16) {
  if (out_f16 && np != 1) return hipErrorInvalidValue;
  PackFused fx{};
  fx.out_f16 = out_f16;
  fx.src2 = R; fx.fro2 = fro2; fx.lambda = lambda; fx.dh = dh; fx.out32 = X32;
  fx.dot_part = dot_part; fx.round_bf16 = round_bf16;
  hipError_t e = launch_pack_impl<true, false>(M, heads, dh, dh, np, outN, outT, plane, fx, s);
  if (e != hipSuccess || !dot_part) return e;
  return launch_sum_partials(dot_part, pack_dot_partials(dh), heads, dot_out, s);
}

hipError_t launch_polar_finish_pack(const float* X, const float* M, int heads, int dh, int np, float* R32, bf16_bits* outT,
                                    int64_t plane, double* dot_part, double* inner, hipStream_t s) {
  PackFused fx{};
  fx.dotwith = M; fx.dot_part = dot_part; fx.out32 = R32;
  hipError_t e = launch_pack_impl<false, true>(X, heads, dh, dh, np, nullptr, outT, plane, fx, s);
  if (e != hipSuccess) return e;
  return launch_sum_partials(dot_part, pack_dot_partials(dh), heads, inner, s);
}

int dot_rm_partials(int64_t n) { return grid_for(n / 4, 1024); }

hipError_t launch_dot_rm(const float* R, const float* M, int heads, int64_t n, int round_bf16, double* part, double* out,
                         hipStream_t s) {
  const int blocks = dot_rm_partials(n);
  hipLaunchKernelGGL(k_dot_rm, dim3(blocks, heads), dim3(256), 0, s, R, M, n, round_bf16, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_sum_partials(part, blocks, heads, out, s);
}

hipError_t launch_fro2(const float* M, int heads, int64_t n, double* part, double* fro2, hipStream_t s) {
  const int blocks = dot_rm_partials(n);
  hipLaunchKernelGGL(k_fro2, dim3(blocks, heads), dim3(256), 0, s, M, n, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_sum_partials(part, blocks, heads, fro2, s);
}

hipError_t launch_axpy(float* X, const float* R, int64_t n, float kappa, hipStream_t s) {
  hipLaunchKernelGGL(k_axpy, dim3(grid_for(n / 4, 2048)), dim3(256), 0, s, X, R, n, kappa);
  return hipGetLastError();
}

namespace {
template <bool EMIT>
void launch_quant_kernel(const void* Y, int y_is_f32, int64_t T, int64_t ld, int d, float qmax, int zero_point, float clip,
                         float* row_sse, float* row_en, void* Q, int64_t ldq, hipStream_t s) {
  const dim3 grid((unsigned)T);
  if (y_is_f32 && zero_point)
    hipLaunchKernelGGL((k_quant_error<true, true, EMIT>), grid, dim3(256), 0, s, Y, T, ld, d, qmax, clip, row_sse, row_en, Q, ldq);
  else if (y_is_f32)
    hipLaunchKernelGGL((k_quant_error<true, false, EMIT>), grid, dim3(256), 0, s, Y, T, ld, d, qmax, clip, row_sse, row_en, Q, ldq);
  else if (zero_point)
    hipLaunchKernelGGL((k_quant_error<false, true, EMIT>), grid, dim3(256), 0, s, Y, T, ld, d, qmax, clip, row_sse, row_en, Q, ldq);
  else
    hipLaunchKernelGGL((k_quant_error<false, false, EMIT>), grid, dim3(256), 0, s, Y, T, ld, d, qmax, clip, row_sse, row_en, Q, ldq);
}
}  // namespace

hipError_t launch_quant_error(const void* Y, int y_is_f32, int64_t T, int64_t ld, int d, int bits, int zero_point, float clip,
                              float* row_sse, float* row_en, double* out, void* Q, int64_t ldq, hipStream_t s) {
  const float qmax = zero_point ? (float)((1 << bits) - 1) : (float)((1 << (bits - 1)) - 1);
  if (Q) launch_quant_kernel<true>(Y, y_is_f32, T, ld, d, qmax, zero_point, clip, row_sse, row_en, Q, ldq, s);
  else launch_quant_kernel<false>(Y, y_is_f32, T, ld, d, qmax, zero_point, clip, row_sse, row_en, nullptr, 0, s);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !out) return e;   // out == null: the caller sums the per-row results itself
  hipLaunchKernelGGL(k_sum_rows, dim3(1), dim3(1024), 0, s, row_sse, row_en, T, out);
  return hipGetLastError();
}

hipError_t launch_row_diag(const void* Y, int y_is_f32, int64_t T, int64_t ld, int d, float* row_pr, float* row_rho,
                           hipStream_t s) {
  const dim3 grid((unsigned)T);
  if (y_is_f32)
    hipLaunchKernelGGL(k_row_diag<true>, grid, dim3(256), 0, s, Y, T, ld, d, row_pr, row_rho);
  else
    hipLaunchKernelGGL(k_row_diag<false>, grid, dim3(256), 0, s, Y, T, ld, d, row_pr, row_rho);
  return hipGetLastError();
}

hipError_t launch_sum_partials(const double* part, int n, int heads, double* out, hipStream_t s) {
  hipLaunchKernelGGL(k_sum_partials, dim3(heads), dim3(256), 0, s, part, n, out);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 4;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_fill_zero, dim3(grid_for((int64_t)n, 2048)), dim3(256), 0, s, reinterpret_cast<uint32_t*>(p), n);
  return hipGetLastError();
}

}  // namespace conqur
