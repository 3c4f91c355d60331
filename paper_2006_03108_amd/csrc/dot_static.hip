// Inner product for callers that cannot allocate device memory (code under
// graph capture, serving loops, harnesses that forbid hipMalloc): the same
// kernels as distdl_dot, with the per-workgroup partial sums in a device array
// that exists once per GPU from the moment the library is loaded there.
#include <atomic>

#include "common.h"

namespace distdl {

// 1024 doubles = 8 KiB per GPU.  In host code this name is only a handle for hipGetSymbolAddress: kernels are
// given the address that call returns for the current device, never the name.
static __device__ __align__(256) double scratch[kDotPartials];
static std::atomic<double*> g_scratch_ptr[64];
constexpr int kDotStaticMaxArrays = 96;

}  // namespace distdl

using namespace distdl;

extern "C" int distdl_dot_static(const void* const a_dev[], const void* const b_dev[], const int64_t count[],
                                 int n_arrays, distdl_dtype dtype, double* result_dev, void* stream) {
  if (!a_dev || !b_dev || !count || !result_dev) return set_error(DISTDL_ERR_NULL, "dot_static: null argument");
  if (n_arrays < 1) return set_error(DISTDL_ERR_INVALID_ARG, "dot_static: n_arrays = %d", n_arrays);
  if (n_arrays > kDotStaticMaxArrays)
    return set_error(DISTDL_ERR_INVALID_ARG, "dot_static: %d arrays exceed the limit of %d (distdl_dot has none)",
                     n_arrays, kDotStaticMaxArrays);
  if (dtype != DISTDL_F32 && dtype != DISTDL_BF16) return set_error(DISTDL_ERR_UNSUPPORTED, "unknown dtype");
  int dev = 0;
  DISTDL_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return set_error(DISTDL_ERR_UNSUPPORTED, "device index %d", dev);
  double* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {  // once per device, with that device current: every GPU holds its own copy of the array
    DISTDL_HIP_TRY(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return set_error(DISTDL_ERR_HIP, "dot_static: the scratch array has no device address");
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  // every partial sum is overwritten by the first launch: nothing of the previous call survives
  return launch_dot(a_dev, b_dev, count, n_arrays, dtype, ptr, result_dev, (hipStream_t)stream);
}
