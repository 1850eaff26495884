// Log-sum-exp merge of two partial attention results (FastUSP section 3.4, the two
// equations under Algorithm 2):
//   lse = log(exp(lse1) + exp(lse2)),  O = exp(lse1 - lse) O1 + exp(lse2 - lse) O2
// evaluated in the overflow-safe order (subtract the larger lse first).
// One streaming pass: each lane moves 8 elements of one row; all lanes of a row sit in
// one wave, so outputs may alias inputs (every lane has read before any lane writes).
#include "usp_common.h"

namespace usp {
namespace {

struct MergeW {
  float w1, w2, lse;
};

// Base-2 hardware exponential and logarithm (1 ulp each): the sum lies in [1, 2], so lse carries an
// absolute error of about 1e-7, and a weight's relative error is that of one exponential.
__device__ __forceinline__ MergeW merge_weights(float a, float b) {
  constexpr float kLog2e = 1.44269504088896340736f, kLn2 = 0.69314718055994530942f;
  MergeW r;
  const float m = fmaxf(a, b);
  if (m == -INFINITY) {  // neither side saw a key
    r.w1 = 0.0f; r.w2 = 0.0f; r.lse = -INFINITY;
    return r;
  }
  const float sum = __builtin_amdgcn_exp2f((a - m) * kLog2e) + __builtin_amdgcn_exp2f((b - m) * kLog2e);
  r.lse = m + __builtin_amdgcn_logf(sum) * kLn2;
  r.w1 = __builtin_amdgcn_exp2f((a - r.lse) * kLog2e);
  r.w2 = __builtin_amdgcn_exp2f((b - r.lse) * kLog2e);
  return r;
}

__device__ __forceinline__ void ld8(const float* p, float (&v)[8]) {
  float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void ld8(const bf16_t* p, float (&v)[8]) {
  typedef uint32_t u32x4_m __attribute__((ext_vector_type(4)));
  const u32x4_m r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_m*>(p));   // read once: streaming
  v[0] = __uint_as_float(r[0] << 16); v[1] = __uint_as_float(r[0] & 0xffff0000u);
  v[2] = __uint_as_float(r[1] << 16); v[3] = __uint_as_float(r[1] & 0xffff0000u);
  v[4] = __uint_as_float(r[2] << 16); v[5] = __uint_as_float(r[2] & 0xffff0000u);
  v[6] = __uint_as_float(r[3] << 16); v[7] = __uint_as_float(r[3] & 0xffff0000u);
}
__device__ __forceinline__ void st8(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void st8(bf16_t* p, const float (&v)[8]) {
  *reinterpret_cast<uint4*>(p) = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                            pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
}

// LPR lanes per row (power of two >= d/8), 64/LPR rows per wave
template <typename T, int LPR>
__global__ __launch_bounds__(256) void lse_merge_kernel(const T* o1, const float* lse1,
                                                        const T* o2, const float* lse2,
                                                        T* o_out, float* lse_out, int64_t rows, int d) {
  constexpr int RPW = 64 / LPR;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = ((int64_t)blockIdx.x * 4 + wave) * RPW + lane / LPR;
  const int l = lane % LPR;
  const bool ok = row < rows;
  const bool has = ok && (l * 8 < d);
  float a[8], b[8];
  float la = 0.0f, lb = 0.0f;
  if (ok) { la = lse1[row]; lb = lse2[row]; }
  if (has) {
    ld8(o1 + row * d + l * 8, a);
    ld8(o2 + row * d + l * 8, b);
  }
  const MergeW w = merge_weights(la, lb);
  if (has) {
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = w.w1 * a[i] + w.w2 * b[i];
    st8(o_out + row * d + l * 8, a);
  }
  if (ok && l == 0) lse_out[row] = w.lse;
}

template <typename T>
usp_status merge_dispatch(int64_t rows, int d, const T* o1, const float* lse1, const T* o2,
                          const float* lse2, T* o_out, float* lse_out, hipStream_t st) {
  const int upr = d / 8;
#define USP_MERGE_LAUNCH(LPR)                                                                   \
  hipLaunchKernelGGL((lse_merge_kernel<T, LPR>),                                                \
                     dim3((unsigned)((rows + 4 * (64 / LPR) - 1) / (4 * (64 / LPR)))), dim3(256), \
                     0, st, o1, lse1, o2, lse2, o_out, lse_out, rows, d)
  if (upr <= 4) USP_MERGE_LAUNCH(4);
  else if (upr <= 8) USP_MERGE_LAUNCH(8);
  else if (upr <= 16) USP_MERGE_LAUNCH(16);
  else if (upr <= 32) USP_MERGE_LAUNCH(32);
  else USP_MERGE_LAUNCH(64);
#undef USP_MERGE_LAUNCH
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

}  // namespace

usp_status launch_lse_merge(int64_t rows, int d, int dt, const void* o1, const float* lse1,
                            const void* o2, const float* lse2, void* o_out, float* lse_out,
                            hipStream_t st) {
  if (rows == 0) return USP_OK;
  if (dt == USP_BF16)
    return merge_dispatch<bf16_t>(rows, d, (const bf16_t*)o1, lse1, (const bf16_t*)o2, lse2,
                                  (bf16_t*)o_out, lse_out, st);
  return merge_dispatch<float>(rows, d, (const float*)o1, lse1, (const float*)o2, lse2,
                               (float*)o_out, lse_out, st);
}

}  // namespace usp
