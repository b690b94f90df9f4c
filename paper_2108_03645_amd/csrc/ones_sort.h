// Ordering of candidates and the sorting network of the selection (arXiv 2108.03645, Section
// 3.2.2 "Selection"): ascending (score, pool slot).  A score is a non-negative fp64, so its bit
// pattern read as an unsigned 64-bit integer orders the same way; ties fall to the smaller slot.
#pragma once

#include "ones_device.h"

namespace ones {
namespace {

__device__ __forceinline__ bool key_less(uint64_t ka, uint32_t ia, uint64_t kb, uint32_t ib) {
  return ka < kb || (ka == kb && ia < ib);
}

// Bitonic sorting network over n (a power of two) keys by one workgroup, ascending
// (score bits, slot).  Works on LDS or, for oversized inputs, on global memory.
template <typename K64, typename I32>
__device__ __forceinline__ void bitonic_sort(K64 *sk, I32 *si, uint32_t n) {
  for (uint32_t k = 2; k <= n; k <<= 1) {
    for (uint32_t j = k >> 1; j > 0; j >>= 1) {
      for (uint32_t e = threadIdx.x; e < n / 2; e += blockDim.x) {
        const uint32_t lo = ((e & ~(j - 1)) << 1) | (e & (j - 1));
        const uint32_t hi = lo | j;
        const bool up = (lo & k) == 0;
        const uint64_t ka = sk[lo], kb = sk[hi];
        const uint32_t ia = si[lo], ib = si[hi];
        if (key_less(kb, ib, ka, ia) == up) {
          sk[lo] = kb; si[lo] = ib;
          sk[hi] = ka; si[hi] = ia;
        }
      }
      __threadfence_block();
      __syncthreads();
    }
  }
}

__device__ __forceinline__ uint32_t pow2_at_least(uint32_t v) {
  return v <= 1 ? 1u : 1u << (32 - __clz(static_cast<int>(v - 1)));
}

}  // namespace
}  // namespace ones
