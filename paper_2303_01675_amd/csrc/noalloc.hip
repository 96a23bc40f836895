// kfkb_op_colsum_accum_static: the bias-gradient column sum for callers that cannot allocate device memory (code
// under HIP graph capture, serving loops, harnesses that forbid hipMalloc).  Same kernels as kfkb_op_colsum_accum;
// the partial sums of the first pass live in a file-scope device array instead of a buffer the caller brings.
#include "common.h"
#include "../../include/kfkb.h"

namespace {

// Partial sums of the two-pass column reduction: [parts <= 64][2][width <= kMaxWidth] floats, 16 MiB.  Every GPU
// the library runs on holds its own copy of the array, at its own address, until the process ends.
constexpr int kMaxWidth = 32768;
constexpr int kMaxParts = 64;
constexpr size_t kScratchFloats = (size_t)kMaxParts * 2 * kMaxWidth;
static __device__ __align__(256) float scratch[kScratchFloats];

// In host code `scratch` is only a handle for the symbol, not a device address: the address on each device is
// asked for once, with that device current, and kept here.
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};

int scratch_for_current_device(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return kfkb::set_error(KFKB_E_HIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return kfkb::set_error(KFKB_E_ARG, "device index %d outside [0, %d)", dev, kMaxDevices);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr)
      return kfkb::set_error(KFKB_E_HIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return 0;
}

}  // namespace

extern "C" int kfkb_op_colsum_accum_static(int dtype, const void* dy, float* out, int rows, int N, void* stream) {
  if (dtype != KFKB_F32 && dtype != KFKB_BF16 && dtype != KFKB_F16) return kfkb::set_error(KFKB_E_ARG, "unknown dtype %d", dtype);
  if (rows < 0 || N < 8 || N % 8 != 0)
    return kfkb::set_error(KFKB_E_ARG, "kfkb_op_colsum_accum_static: need rows >= 0 and width %% 8 == 0 (rows=%d width=%d)", rows, N);
  if (N > kMaxWidth)
    return kfkb::set_error(KFKB_E_ARG, "kfkb_op_colsum_accum_static: width %d exceeds the built-in scratch (at most %d columns); "
                           "use kfkb_op_colsum_accum with a buffer of the caller's", N, kMaxWidth);
  if (rows == 0) return 0;
  if (kfkb::colsum_scratch_floats(rows, N) > kScratchFloats)
    return kfkb::set_error(KFKB_E_ARG, "kfkb_op_colsum_accum_static: rows=%d width=%d need more than the built-in scratch", rows, N);
  if (!dy || !out) return kfkb::set_error(KFKB_E_ARG, "kfkb_op_colsum_accum_static: null pointer");
  float* ptr = nullptr;
  const int rc = scratch_for_current_device(&ptr);
  if (rc != 0) return rc;
  // the first pass writes every partial sum the second pass reads (parts x N entries of slot 0), so nothing of
  // an earlier call's contents has to be cleared
  const hipError_t e = kfkb::launch_colsum_accum(dtype, dy, out, ptr, rows, N, (hipStream_t)stream);
  if (e != hipSuccess) return kfkb::set_error(KFKB_E_HIP, "kfkb_op_colsum_accum_static: launch failed: %s", hipGetErrorString(e));
  return 0;
}
