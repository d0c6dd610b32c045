// conqur_score_rows_static: the fake-quantisation score of rows that are already rotated, for callers that
// cannot allocate (code under HIP graph capture, tight serving loops).  The per-row results the score kernels
// exchange live in a file-scope device array instead of a context's workspace; the call allocates nothing,
// copies nothing to the host and does not wait for the stream.
#include "../../include/conqur.h"

#include <mutex>

#include "kernels.h"

using namespace conqur;

namespace {

constexpr int64_t kStaticMaxRows = 65536;   // rows per call; the array below holds two floats per row (512 KiB)
constexpr int kMaxDevices = 64;

// Per-row squared errors [0, kStaticMaxRows) and per-row energies [kStaticMaxRows, 2 kStaticMaxRows) of the call in
// flight.  Every GPU the library runs on holds its own copy at its own address until the process ends; the name
// below is only the host-side handle of the symbol, never a device address.
static __device__ __align__(256) float g_score_scratch[2 * kStaticMaxRows];

std::mutex g_mu;
float* g_scratch_ptr[kMaxDevices];   // device address of g_score_scratch on each device, once resolved

}  // namespace

namespace conqur {

// Device address of the scratch array on the current device; resolved once per device (with that device current).
hipError_t static_scratch_for_current_device(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_score_scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace conqur

extern "C" conqur_status conqur_score_rows_static(const void* Y_dev, uint32_t dtype, uint64_t T, uint64_t d,
                                                  uint64_t row_stride_elems, uint32_t bits, uint32_t zero_point,
                                                  float clip_ratio, double* out_dev, void* stream) {
  if (!Y_dev || !out_dev) return CONQUR_EINVAL;
  if (dtype != CONQUR_F32 && dtype != CONQUR_BF16) return CONQUR_EINVAL;
  const uint64_t esz = dtype == CONQUR_F32 ? 4 : 2;
  if (T < 1 || T > (uint64_t)kStaticMaxRows) return CONQUR_EINVAL;                  // beyond the static array
  if (d < 16 || d > 65536 || d % 16 != 0) return CONQUR_EINVAL;
  if (row_stride_elems < d || row_stride_elems >= (1ull << 40)) return CONQUR_EINVAL;
  if ((reinterpret_cast<uintptr_t>(Y_dev) & 15) || ((row_stride_elems * esz) & 15)) return CONQUR_EINVAL;
  if (reinterpret_cast<uintptr_t>(out_dev) & 7) return CONQUR_EINVAL;
  if (bits < 2 || bits > 8 || zero_point > 1) return CONQUR_EINVAL;
  if (zero_point && (!(clip_ratio > 0.0f) || clip_ratio > 1.0f)) return CONQUR_EINVAL;
  float* scratch = nullptr;
  if (static_scratch_for_current_device(&scratch) != hipSuccess) return CONQUR_EHIP;
  // Every row of the call is written before the sum kernel reads it, so nothing has to start at zero; what an
  // earlier (possibly larger) call left beyond row T is never read.
  const hipError_t e = launch_quant_error(Y_dev, dtype == CONQUR_F32, (int64_t)T, (int64_t)row_stride_elems, (int)d, (int)bits,
                                          (int)zero_point, zero_point ? clip_ratio : 1.0f, scratch, scratch + kStaticMaxRows,
                                          out_dev, nullptr, 0, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? CONQUR_OK : CONQUR_EHIP;
}
