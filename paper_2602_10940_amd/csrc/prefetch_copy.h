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

// The transfers of a whole ring inside one launch: work-group wg of s.copy_wgs copies its share of
// chunk c = 1, 2, .. and then counts itself on s.arrive[c].  The stores carry device scope (they are
// written through to where every CU's loads find them; a fence would write back and invalidate the
// whole L2 under the attention work-groups), each thread waits for its own stores, the
// work-group barrier collects the threads, and one thread publishes the count.
__device__ __forceinline__ void store16_device_scope(uint4* p, const uint4& v) {
  typedef unsigned int vec4u __attribute__((ext_vector_type(4)));
  const vec4u x = {v.x, v.y, v.z, v.w};
  asm volatile("global_store_dwordx4 %0, %1, off sc1" :: "v"(p), "v"(x) : "memory");
}
__device__ __forceinline__ void stream_chunks(const AttnStep& s, int wg, int tid, int nthr) {
  const int64_t stride = (int64_t)s.copy_wgs * nthr;
  const int64_t first = (int64_t)wg * nthr + tid;
  for (int c = 1; c < s.n_multi; ++c) {
    const int64_t n = s.chunk[c].bytes >> 4;           // the host passes 16-byte multiples, 16-byte aligned
    for (int t = 0; t < 2; ++t) {
      const uint4* s4 = (const uint4*)(t ? s.chunk[c].v_src : s.chunk[c].k_src);
      uint4* d4 = (uint4*)(t ? s.chunk[c].v : s.chunk[c].k);
      int64_t i = first;
      for (; i + 3 * stride < n; i += 4 * stride) {   // four loads in flight per lane
        const uint4 a = s4[i], b = s4[i + stride], e = s4[i + 2 * stride], f = s4[i + 3 * stride];
        store16_device_scope(d4 + i, a); store16_device_scope(d4 + i + stride, b);
        store16_device_scope(d4 + i + 2 * stride, e); store16_device_scope(d4 + i + 3 * stride, f);
      }
      for (; i < n; i += stride) store16_device_scope(d4 + i, s4[i]);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this thread's stores have been acknowledged
    __syncthreads();
    if (tid == 0) __hip_atomic_fetch_add(s.arrive + c, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

}  // namespace usp
