// The kernel that draws the remaining work of every job slot (Alg. 1, Eq. 7) for a run of
// generations at once; the arithmetic is in ones_sample.h.
#include "ones_sample.h"

namespace ones {
namespace {

constexpr int kSampleBlock = 256;

// Workgroup (x, y): sixteen slots of generation t + y, whose remaining work and term table go to
// place (t + y) mod kDrawRing of the ring that starts at tab.Y and tab.terms.
__global__ __launch_bounds__(kSampleBlock) void sample_remaining_kernel(Progress pr, JobTable tab, uint32_t Jn,
                                                                       uint32_t Jp, uint32_t key0, uint32_t key1,
                                                                       uint32_t t, uint32_t ring_stride) {
  const uint32_t gen = t + blockIdx.y;
  const size_t shift = static_cast<size_t>(gen % kDrawRing) * ring_stride;       // in doubles
  tab.Y += shift;
  tab.terms += shift;
  (void)Jp;                                                  // the grid's x covers the Jp slots exactly
  sample_remaining_slot(pr, tab, Jn, key0, key1, gen, blockIdx.x * kSampleBlock + threadIdx.x);
}

}  // namespace

hipError_t launch_sample_remaining(const Progress &pr, const JobTable &ring, uint32_t ring_stride, uint32_t Jn,
                                   uint32_t Jp, uint32_t key0, uint32_t key1, uint32_t t, uint32_t count,
                                   hipStream_t s) {
  if (count == 0 || count > static_cast<uint32_t>(kDrawRing)) return hipErrorInvalidValue;
  // Jp is a multiple of 64 and a workgroup serves kSampleBlock / kLanesPerSlot = 16 slots
  hipLaunchKernelGGL(sample_remaining_kernel, dim3(Jp * kLanesPerSlot / kSampleBlock, count), dim3(kSampleBlock), 0, s,
                     pr, ring, Jn, Jp, key0, key1, t, ring_stride);
  return hipGetLastError();
}

}  // namespace ones
