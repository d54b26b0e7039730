// Streaming copy of known size: the reference against which hardware traffic
// counters (bytes fetched from / written to HBM) are scaled.
#include "bppsa_internal.h"

namespace {

typedef float vec4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(256)
calibration_copy_kernel(const vec4* __restrict__ src, vec4* __restrict__ dst, int64_t n4) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    const vec4 v = __builtin_nontemporal_load(src + i);
    __builtin_nontemporal_store(v, dst + i);
  }
}

}  // namespace

extern "C" bppsa_status bppsa_calibration_copy(const float* src, float* dst, int64_t n, void* stream) {
  if (!src || !dst || n < 1) return BPPSA_EINVAL;
  if ((n & 3) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return BPPSA_ESHAPE;
  const int64_t n4 = n / 4;
  const int64_t want = (n4 + 255) / 256;
  const int grid = (int)(want < 8192 ? want : 8192);
  calibration_copy_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(
      reinterpret_cast<const vec4*>(src), reinterpret_cast<vec4*>(dst), n4);
  BPPSA_CHECK_LAUNCH();
  return BPPSA_OK;
}
