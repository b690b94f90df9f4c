// The kernel that draws the remaining work of every job slot for one generation (Alg. 1, Eq. 7);
// the arithmetic is in ones_sample.h.
#include "ones_sample.h"

namespace ones {
namespace {

constexpr int kSampleBlock = 256;

__global__ __launch_bounds__(kSampleBlock) void sample_remaining_kernel(Progress pr, JobTable tab, uint32_t Jn,
                                                                       uint32_t Jp, uint32_t key0, uint32_t key1,
                                                                       uint32_t t) {
  (void)Jp;                                                  // the grid covers the Jp slots exactly
  sample_remaining_slot(pr, tab, Jn, key0, key1, t, blockIdx.x * kSampleBlock + threadIdx.x);
}

}  // namespace

hipError_t launch_sample_remaining(const Progress &pr, const JobTable &tab, uint32_t Jn, uint32_t Jp,
                                   uint32_t key0, uint32_t key1, uint32_t t, hipStream_t s) {
  // Jp is a multiple of 64 and a workgroup serves kSampleBlock / kLanesPerSlot = 16 slots
  hipLaunchKernelGGL(sample_remaining_kernel, dim3(Jp * kLanesPerSlot / kSampleBlock), dim3(kSampleBlock), 0, s, pr,
                     tab, Jn, Jp, key0, key1, t);
  return hipGetLastError();
}

}  // namespace ones
