// Device-side transfers that ride in an attention launch (Algorithm 2: the transfer of chunk r+1
// overlaps the compute on chunk r).
//  * prefetch_copy: the next chunk into the idle one of two staging buffers, run by extra work-groups
//    of a per-chunk launch.  Stream order gives the two hazards for free: the launch that reads the
//    buffer starts after this one has ended, and the buffer's previous reader ended before this one
//    began.
//  * stream_chunks / stream_chunks_fp8: every later chunk of a ring into a buffer of its own, run by
//    the first work-groups of the one launch over the ring, each chunk published through an arrival
//    counter; the FP8 form decodes the chunk on the way (Algorithm 1 line 4).
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
// written through to where every XCD's loads find them; a fence would write back and invalidate the
// whole L2 under the attention work-groups), each thread waits until its own stores have been
// acknowledged, the work-group barrier collects the threads, and one thread publishes the count.
// The readers make no acquire of their own either: nothing reads a staging buffer or its records
// before their chunk's count is complete, and the launch starts with invalid caches, so no cache on
// the reading side can hold an older copy of those lines.
__device__ __forceinline__ void publish_chunk(int* counter, int tid) {
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this thread's stores have been acknowledged
  __syncthreads();
  if (tid == 0) __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// A 16-byte store with device scope.  The instruction sits in inline asm (no builtin sets the scope
// bits of a plain store), where the compiler's hazard recogniser cannot see that it is a store: on
// gfx9 a store of more than 8 bytes reads its data registers late, and a VALU instruction that
// overwrites them within the next two wait states can change what is stored (seen as rare wrong
// words in some lanes when the next store's data was computed into the same registers).  The two
// wait states therefore ride inside the asm statement.
__device__ __forceinline__ void store16_device_scope(uint4* p, const uint4& v) {
  typedef unsigned int vec4u __attribute__((ext_vector_type(4)));
  const vec4u x = {v.x, v.y, v.z, v.w};
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" :: "v"(p), "v"(x) : "memory");
}
// Algorithm 1 line 4 for chunk c of a launch over several FP8 chunks: unit `first`, first + stride, ..
// of the chunk (16 codes of K and of V each; then 4 keys of the records).  The arithmetic is the
// dequantiser's: E4M3 code -> fp32 (exact), times the scale in fp32, RNE to bf16; K keeps scale 1
// and hands its scales to the records as per-key factors of the exponent.
template <bool kDeviceScope>
__device__ __forceinline__ void put16(uint4* p, const uint4& v) {
  if (kDeviceScope) store16_device_scope(p, v);
  else *p = v;
}
__device__ __forceinline__ uint4 decode8_bf16(uint32_t w0, uint32_t w1, float sc) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, true);
  const f32x2_t c = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, false), e = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, true);
  return make_uint4(pack_bf16x2(a.x * sc, a.y * sc), pack_bf16x2(b.x * sc, b.y * sc),
                    pack_bf16x2(c.x * sc, c.y * sc), pack_bf16x2(e.x * sc, e.y * sc));
}
template <bool kDeviceScope>
__device__ __forceinline__ void fp8_chunk_prepare(const AttnStep& s, int c, int64_t first, int64_t stride) {
  const AttnStep::Chunk& ch = s.chunk[c];
  int tile0 = 0, nt_total = 0;                          // first tile of the chunk, tiles of all chunks
  for (int i = 0; i < s.n_multi; ++i) {
    if (i < c) tile0 += s.chunk[i].Sc / 64;
    nt_total += s.chunk[i].Sc / 64;
  }
  const int64_t rows = (int64_t)s.B * s.H * ch.Sc;      // (head, token) rows of d = 128 or 64 codes
  const int ush = s.d == 64 ? 2 : 3;                    // log2 of the 16-code units per row
  const uint4* kc = (const uint4*)ch.k_src;
  const uint4* vc = (const uint4*)ch.v_src;
  uint4* kd = (uint4*)ch.k;
  uint4* vd = (uint4*)ch.v;
  auto emit = [&](int64_t u, const uint4& a, const uint4& b, float vs) {
    put16<kDeviceScope>(kd + 2 * u, decode8_bf16(a.x, a.y, 1.0f));
    put16<kDeviceScope>(kd + 2 * u + 1, decode8_bf16(a.z, a.w, 1.0f));
    put16<kDeviceScope>(vd + 2 * u, decode8_bf16(b.x, b.y, vs));
    put16<kDeviceScope>(vd + 2 * u + 1, decode8_bf16(b.z, b.w, vs));
  };
  const int64_t units = rows << ush;
  int64_t u = first;
  for (; u + 3 * stride < units; u += 4 * stride) {     // the loads of four units in flight per lane
    const uint4 a0 = kc[u], b0 = vc[u], a1 = kc[u + stride], b1 = vc[u + stride];
    const uint4 a2 = kc[u + 2 * stride], b2 = vc[u + 2 * stride], a3 = kc[u + 3 * stride], b3 = vc[u + 3 * stride];
    const float s0 = ch.v_scale_src[u >> ush], s1 = ch.v_scale_src[(u + stride) >> ush];
    const float s2 = ch.v_scale_src[(u + 2 * stride) >> ush], s3 = ch.v_scale_src[(u + 3 * stride) >> ush];
    emit(u, a0, b0, s0); emit(u + stride, a1, b1, s1); emit(u + 2 * stride, a2, b2, s2); emit(u + 3 * stride, a3, b3, s3);
  }
  for (; u < units; u += stride) emit(u, kc[u], vc[u], ch.v_scale_src[u >> ush]);
  const float scale2 = s.scale * 1.44269504088896340736f;
  const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
  for (int64_t u = first; u < rows / 4; u += stride) {  // chunk lengths are multiples of 64
    const int64_t row = 4 * u;
    const int64_t bh = row / ch.Sc;
    const int key = (int)(row - bh * ch.Sc);
    const float4 ks = ((const float4*)ch.k_scale_src)[u];
    float* rec = s.ext + ((bh * nt_total + tile0 + (key >> 6)) << 8) + (key & 63);
    if (ch.mask_src == nullptr) {                       // no dead keys: bias 0, flag 0
      put16<kDeviceScope>((uint4*)rec, make_uint4(__float_as_uint(ks.x * scale2), __float_as_uint(ks.y * scale2),
                                                 __float_as_uint(ks.z * scale2), __float_as_uint(ks.w * scale2)));
      put16<kDeviceScope>((uint4*)(rec + 64), zero);
      put16<kDeviceScope>((uint4*)(rec + 128), zero);
      put16<kDeviceScope>((uint4*)(rec + 192), zero);
      continue;
    }
    // masked chunk: a dead key gets factor 0 and bias -inf; the tile's flag says whether it has any.
    // The 16 lanes that share a tile are consecutive (units are handed out in lane order and a tile
    // is 16 units), so the wave's ballot holds the tile's 16 answers side by side.
    const uint32_t mk = *(const uint32_t*)(ch.mask_src + (bh / s.H) * ch.Sc + key);
    const bool k0 = (mk & 0xffu) != 0, k1 = (mk & 0xff00u) != 0, k2 = (mk & 0xff0000u) != 0, k3 = (mk & 0xff000000u) != 0;
    const unsigned long long dead = __builtin_amdgcn_ballot_w64(!(k0 && k1 && k2 && k3));
    const int lane16 = (int)(__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u))) & ~15;
    const uint32_t fl = ((dead >> lane16) & 0xffffull) != 0 ? 0x3f800000u : 0u;
    const uint32_t ninf = 0xff800000u;
    put16<kDeviceScope>((uint4*)rec, make_uint4(k0 ? __float_as_uint(ks.x * scale2) : 0u, k1 ? __float_as_uint(ks.y * scale2) : 0u,
                                               k2 ? __float_as_uint(ks.z * scale2) : 0u, k3 ? __float_as_uint(ks.w * scale2) : 0u));
    put16<kDeviceScope>((uint4*)(rec + 64), make_uint4(k0 ? 0u : ninf, k1 ? 0u : ninf, k2 ? 0u : ninf, k3 ? 0u : ninf));
    put16<kDeviceScope>((uint4*)(rec + 128), make_uint4(fl, fl, fl, fl));
    put16<kDeviceScope>((uint4*)(rec + 192), zero);
  }
}
// The copy work-groups of a launch over several FP8 chunks: chunk 1, 2, .. decoded and counted.
__device__ __forceinline__ void stream_chunks_fp8(const AttnStep& s, int wg, int tid, int nthr) {
  for (int c = 1; c < s.n_multi; ++c) {
    fp8_chunk_prepare<true>(s, c, (int64_t)wg * nthr + tid, (int64_t)s.copy_wgs * nthr);
    publish_chunk(s.arrive + c, tid);
  }
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
    publish_chunk(s.arrive + c, tid);
  }
}

}  // namespace usp
