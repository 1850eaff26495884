// Device-side copy of the next KV chunk into the idle staging buffer, run by the leading
// work-groups of an attention launch (Algorithm 2: the transfer of chunk r+1 overlaps the compute
// on chunk r).  Stream order gives the two hazards for free: the launch that reads the buffer
// starts after this one has ended, and the buffer's previous reader ended before this one began.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "usp_common.h"

namespace usp {

__device__ __forceinline__ void prefetch_copy(const AttnStep& s, int wg, int tid, int nthr) {
  const int64_t stride = (int64_t)s.copy_wgs * nthr;
  const int64_t first = (int64_t)wg * nthr + tid;
  for (int c = 0; c < s.n_copy; ++c) {
    const unsigned char* src = (const unsigned char*)s.copy[c].src;
    unsigned char* dst = (unsigned char*)s.copy[c].dst;
    const int64_t bytes = s.copy[c].bytes;
    const uintptr_t both = (uintptr_t)src | (uintptr_t)dst;
    if ((both & 15) == 0) {
      const uint4* s4 = (const uint4*)src;
      uint4* d4 = (uint4*)dst;
      const int64_t n = bytes >> 4;
      int64_t i = first;
      for (; i + 3 * stride < n; i += 4 * stride) {   // four loads in flight per lane
        const uint4 a = s4[i], b = s4[i + stride], e = s4[i + 2 * stride], f = s4[i + 3 * stride];
        d4[i] = a; d4[i + stride] = b; d4[i + 2 * stride] = e; d4[i + 3 * stride] = f;
      }
      for (; i < n; i += stride) d4[i] = s4[i];
      for (int64_t j = (n << 4) + first; j < bytes; j += stride) dst[j] = src[j];
    } else if ((both & 3) == 0) {                     // per-token scales: 4-byte aligned only
      const uint32_t* s1 = (const uint32_t*)src;
      uint32_t* d1 = (uint32_t*)dst;
      const int64_t n = bytes >> 2;
      for (int64_t i = first; i < n; i += stride) d1[i] = s1[i];
      for (int64_t j = (n << 2) + first; j < bytes; j += stride) dst[j] = src[j];
    } else {
      for (int64_t j = first; j < bytes; j += stride) dst[j] = src[j];
    }
  }
}

}  // namespace usp
