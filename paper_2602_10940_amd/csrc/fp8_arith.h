// Arithmetic of the FP8 (E4M3) pack: FastUSP Algorithm 1 line 2, q = e4m3(x / s) with a true IEEE
// fp32 division, for many x and one s.  Shared by the pack kernels and by the diagnostic that checks
// the short bf16 sequence against the division exhaustively.
#pragma once
#include "usp_common.h"

namespace usp {

constexpr float kFp8Max = 448.0f;
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_raw __attribute__((ext_vector_type(4)));

// x / s for many x and one s.  The compiler's IEEE-correct fp32 division is: reciprocal estimate,
// one Newton step on the reciprocal, then two residual corrections of the quotient (plus operand
// pre-scaling that only engages for extreme exponents).  Everything that depends on s alone is
// hoisted here; quotient() is the per-element remainder of that same sequence and returns the
// correctly rounded quotient whenever the pre-scaling would have been a no-op, which `fast`
// guarantees for the divisor (|x| <= 448 s bounds the quotient).  Quotients too small to be
// normal fp32 can differ in their last bits, but they are far below 2^-10 and encode to +-0
// either way.  Rows outside the fast range use the plain division.
struct RowDiv {
  float s, rcp;
  bool fast;
};
__device__ __forceinline__ RowDiv make_rowdiv(float s) {
  RowDiv d;
  d.s = s;
  d.fast = s > 0x1p-60f && s < 0x1p+60f;
  const float r0 = __builtin_amdgcn_rcpf(s);
  const float e0 = fmaf(-s, r0, 1.0f);
  d.rcp = fmaf(e0, r0, r0);
  return d;
}
__device__ __forceinline__ float quotient(float x, const RowDiv& d) {
  const float q0 = x * d.rcp;
  const float r0 = fmaf(-d.s, q0, x);
  const float q1 = fmaf(r0, d.rcp, q0);
  const float r1 = fmaf(-d.s, q1, x);
  // s > 0, so the quotient has the sign of x; restoring it keeps -0 (the corrections turn it into +0)
  return __builtin_copysignf(fmaf(r1, d.rcp, q1), x);
}

// E4M3 codes of v[i] / s (round to nearest even, saturating).  In the fast range s is a normal
// number, |v[i]| <= 448 s up to one rounding, so the quotient never reaches the overflow threshold
// 464 and the hardware convert needs no clamp (inputs are assumed finite).  A denormal s can be
// far from absmax / 448 in relative terms; that path clamps to +-448 before converting.
template <bool kFast>
__device__ __forceinline__ uint2 encode8(const float (&v)[8], const RowDiv& d) {
  float t[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
    t[i] = kFast ? quotient(v[i], d) : __builtin_amdgcn_fmed3f(v[i] / d.s, -kFp8Max, kFp8Max);
  int lo = __builtin_amdgcn_cvt_pk_fp8_f32(t[0], t[1], 0, false);
  lo = __builtin_amdgcn_cvt_pk_fp8_f32(t[2], t[3], lo, true);
  int hi = __builtin_amdgcn_cvt_pk_fp8_f32(t[4], t[5], 0, false);
  hi = __builtin_amdgcn_cvt_pk_fp8_f32(t[6], t[7], hi, true);
  return make_uint2((uint32_t)lo, (uint32_t)hi);
}

__device__ __forceinline__ float absmax8(const float (&v)[8], float a) {
#pragma unroll
  for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf(v[i]));
  return a;
}

__device__ __forceinline__ float scale_from_absmax(float a) {
  float s = a / kFp8Max;
  return s == 0.0f ? 1.0f : s;
}


// ---- bf16 inputs: a shorter sequence with the same codes -------------------------------------------
// A bf16 x has 8 significant bits and the row's scale is absmax / 448 of a bf16 absmax with
// |x| <= absmax.  Over every such pair (2^29 of them, s in the fast range) the quotient after ONE
// residual correction, q1 = fma(fma(-s, q0, x), rcp, q0) with q0 = x * rcp, encodes to the same E4M3
// code as the IEEE quotient x / s (checked exhaustively on the device, usp_diag_check_bf16_division:
// q1 itself differs from the IEEE quotient in the last bit for 0.2 % of the pairs, never across a
// rounding boundary of the 4-bit format).  The sign of the code is the sign bit of x (also for -0 and
// for quotients that round to zero), so it is merged into the packed codes from the high bytes of the
// packed bf16 pairs instead of being restored per element.
// r: 8 consecutive bf16 as loaded (element 2k in the low half of r[k]).
__device__ __forceinline__ uint2 encode8_bf16_short(const u32x4_raw r, const RowDiv& d) {
  float t[8];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const float x0 = __uint_as_float(r[k] << 16), x1 = __uint_as_float(r[k] & 0xffff0000u);
    const float a0 = x0 * d.rcp, a1 = x1 * d.rcp;
    t[2 * k] = fmaf(fmaf(-d.s, a0, x0), d.rcp, a0);
    t[2 * k + 1] = fmaf(fmaf(-d.s, a1, x1), d.rcp, a1);
  }
  int lo = __builtin_amdgcn_cvt_pk_fp8_f32(t[0], t[1], 0, false);
  lo = __builtin_amdgcn_cvt_pk_fp8_f32(t[2], t[3], lo, true);
  int hi = __builtin_amdgcn_cvt_pk_fp8_f32(t[4], t[5], 0, false);
  hi = __builtin_amdgcn_cvt_pk_fp8_f32(t[6], t[7], hi, true);
  const uint32_t s_lo = __builtin_amdgcn_perm(r[1], r[0], 0x07050301u);   // the four high bytes: sign in bit 7 of each
  const uint32_t s_hi = __builtin_amdgcn_perm(r[3], r[2], 0x07050301u);
  return make_uint2(((uint32_t)lo & 0x7f7f7f7fu) | (s_lo & 0x80808080u), ((uint32_t)hi & 0x7f7f7f7fu) | (s_hi & 0x80808080u));
}
// |x| maximum of 8 packed bf16 as a bf16 bit pattern in each half of the result (non-negative floats
// order like their bit patterns)
__device__ __forceinline__ uint32_t absmax8_bf16_bits(const u32x4_raw r, uint32_t m) {
  typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const u16x2 a = __builtin_bit_cast(u16x2, r[k] & 0x7fff7fffu), b = __builtin_bit_cast(u16x2, m);
    m = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, b));
  }
  return m;
}

}  // namespace usp
