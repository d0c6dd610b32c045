// Shared device/host helpers for the gfx950 kernels of libconqur.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace conqur {

// A kernel's dynamic-LDS limit (hipFuncSetAttribute) belongs to the device that is current when it is set: launchers
// raise it once per device and kernel.  One bit per device ordinal; ordinals beyond 63 set it on every launch.
class PerDeviceOnce {
 public:
  template <typename F>
  hipError_t run(F&& set) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = (dev >= 0 && dev < 64) ? (1ull << dev) : 0ull;
    if (bit && (done_.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = set();
    if (e == hipSuccess && bit) done_.fetch_or(bit, std::memory_order_release);
    return e;
  }

 private:
  std::atomic<uint64_t> done_{0};
};


typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short bf16_bits;  // raw bf16 storage

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// fp32 -> bf16, round to nearest even (NaN stays NaN, Inf stays Inf): the hardware conversion
// (v_cvt_pk_bf16_f32, one instruction for two values).
__device__ __forceinline__ bf16_bits f32_to_bf16(float f) {
  const __bf16 b = (__bf16)f;
  return __builtin_bit_cast(unsigned short, b);
}
// Two values at once, packed lo | hi << 16.
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
// Two values as fp16 (round to nearest even), packed lo | hi << 16.
__device__ __forceinline__ uint32_t f32x2_to_f16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}
__device__ __forceinline__ bf16_bits f32_to_f16(float f) {
  const _Float16 h = (_Float16)f;  // round to nearest even
  return __builtin_bit_cast(unsigned short, h);
}
__device__ __forceinline__ float bf16_to_f32(bf16_bits b) { return __uint_as_float(((uint32_t)b) << 16); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// The accumulate operand holds the unit rows x^ = x / ||x|| times this power of two, in fp16.  |x^| <= 1, and on
// outlier-dominated rows most entries are 1e-3 .. 1e-5: times 1/sqrt(dh) (the corner's magnitude) they would sit in
// fp16's subnormal range (below 6.1e-5) and lose bits; scaled up they keep all 11.  The factor and 1/sqrt(dh) are
// applied to the fp32 result instead (exact power of two; the sum cannot overflow: 64 * tokens * 1).
constexpr float kXhatScale = 64.0f;

}  // namespace conqur
