// Moves a freshly computed plan from the page-locked staging buffer into the fixed plan
// section of the device workspace (Sec. 3.3.1: the plan is computed on the CPU and copied
// asynchronously; App. D: pinned staging buffer).  A copy kernel on the run's stream reads the
// host-resident staging buffer through its device mapping: kernel-to-kernel ordering on one
// queue is cheaper than switching to a copy engine and back between two attention launches.
#include "kernels.h"

namespace fi355 {
namespace {
__global__ void __launch_bounds__(256) plan_upload_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ dst,
                                                          int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = __builtin_nontemporal_load(src + i);
}
}  // namespace

hipError_t launch_plan_upload(const int32_t* staging_dev_view, int32_t* plan_section, int32_t n_ints,
                              hipStream_t stream) {
  if (n_ints <= 0) return hipSuccess;
  hipLaunchKernelGGL(plan_upload_kernel, dim3((n_ints + 255) / 256), dim3(256), 0, stream, staging_dev_view,
                     plan_section, n_ints);
  return hipGetLastError();
}
}  // namespace fi355
