// Correctness-first attention step for shapes the MFMA kernel does not take: fp32 inputs
// (all arithmetic in fp32), any head dimension up to 256 that is a multiple of 4, FP8 K/V
// read directly (value = code * per-token scale).  One wave per query row, keys in tiles
// of 64 (one key per lane for the scores, one head-dim slot per lane for P.V), online
// softmax across tiles.  Computes, for one KV chunk (FastUSP section 2.2 and 2.2.2):
//   O_r = softmax(q K^T * scale) V,   lse_r = log sum_j exp(q.k_j * scale)
// and optionally folds the carried (O, lse) in with the merge equations of section 3.4.
#include "usp_common.h"
#include "prefetch_copy.h"

namespace usp {
namespace {

typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float ld_elem(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float ld_elem(const bf16_t* p, int64_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ float ld_elem(const uint8_t* p, int64_t i) {
  f32x2 r = __builtin_amdgcn_cvt_pk_f32_fp8((int)p[i], false);
  return r.x;
}
__device__ __forceinline__ void st_elem(float* p, int64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st_elem(bf16_t* p, int64_t i, float v) { p[i] = f32_to_bf16(v); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

constexpr int kMaxD = 256;
constexpr int kSlots = kMaxD / 64;

template <typename QT, typename KT>
__global__ __launch_bounds__(256) void attn_generic_kernel(AttnStep s) {
  __shared__ float q_sh[4][kMaxD];
  __shared__ float p_sh[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (s.copy_wgs > 0 && blockIdx.x >= gridDim.x - s.copy_wgs) {   // prefetch work-groups end the x axis
    if (blockIdx.y == 0 && blockIdx.z == 0)
      prefetch_copy(s, blockIdx.x - (gridDim.x - s.copy_wgs), threadIdx.x, 256);
    return;
  }
  const int i_raw = blockIdx.x * 4 + wave;  // query row
  const bool valid = i_raw < s.Sq;          // surplus waves recompute the last row, store nothing
  const int i = valid ? i_raw : s.Sq - 1;
  const int h = blockIdx.y, b = blockIdx.z;
  const QT* q = (const QT*)s.q + b * s.qs[0] + h * s.qs[1] + (int64_t)i * s.qs[2];
  const KT* k = (const KT*)s.k + b * s.ks[0] + h * s.ks[1];
  const KT* v = (const KT*)s.v + b * s.ks[0] + h * s.ks[1];
  const int64_t kt = s.ks[2];
  const float* ksc = s.k_scale ? s.k_scale + ((int64_t)b * s.H + h) * s.Sc : nullptr;
  const float* vsc = s.v_scale ? s.v_scale + ((int64_t)b * s.H + h) * s.Sc : nullptr;
  const uint8_t* mask = s.key_mask ? s.key_mask + (int64_t)b * s.Sc : nullptr;
  const int d = s.d;

  for (int t = lane; t < d; t += 64) q_sh[wave][t] = ld_elem(q, t);
  __syncthreads();

  float m = -INFINITY, l = 0.0f;
  float acc[kSlots];
#pragma unroll
  for (int c = 0; c < kSlots; ++c) acc[c] = 0.0f;

  for (int j0 = 0; j0 < s.Sc; j0 += 64) {
    const int j = j0 + lane;
    float sc = -INFINITY;
    if (j < s.Sc && (!mask || mask[j])) {
      float dot = 0.0f;
      const KT* kr = k + (int64_t)j * kt;
      for (int t = 0; t < d; ++t) dot = fmaf(q_sh[wave][t], ld_elem(kr, t), dot);
      if (ksc) dot *= ksc[j];
      sc = dot * s.scale;
    }
    const float m_new = fmaxf(m, wave_max(sc));
    float p = 0.0f, alpha = 1.0f;
    if (m_new != -INFINITY) {
      p = expf(sc - m_new);       // sc = -inf -> 0
      alpha = expf(m - m_new);    // m = -inf -> 0
    }
    l = l * alpha + wave_sum(p);
    m = m_new;
    if (vsc && j < s.Sc) p *= vsc[j];
    __syncthreads();  // previous tile's readers are done with p_sh
    p_sh[wave][lane] = p;
    __syncthreads();
    const int jn = min(64, s.Sc - j0);
#pragma unroll
    for (int c = 0; c < kSlots; ++c) {
      const int t = lane + 64 * c;
      if (t < d) {
        float a = acc[c] * alpha;
        for (int jj = 0; jj < jn; ++jj) a = fmaf(p_sh[wave][jj], ld_elem(v + (int64_t)(j0 + jj) * kt, t), a);
        acc[c] = a;
      }
    }
  }

  // chunk result and merge (section 3.4)
  const int64_t row = ((int64_t)b * s.H + h) * s.Sq + i;
  float lse_r = -INFINITY, c_cur = 0.0f;
  if (l > 0.0f) { lse_r = m + logf(l); c_cur = 1.0f / l; }
  float w_prev = 0.0f, lse_new = lse_r;
  if (s.mode >= 2) {
    const float lse_p = s.lse[row];
    const float mm = fmaxf(lse_p, lse_r);
    if (mm == -INFINITY) { w_prev = 0.0f; c_cur = 0.0f; lse_new = -INFINITY; }
    else {
      lse_new = mm + logf(expf(lse_p - mm) + expf(lse_r - mm));
      w_prev = expf(lse_p - lse_new);
      c_cur *= expf(lse_r - lse_new);
    }
  }
  float* accp = s.acc ? s.acc + row * d : nullptr;
  QT* outp = (QT*)s.out + b * s.os[0] + h * s.os[1] + (int64_t)i * s.os[2];
#pragma unroll
  for (int c = 0; c < kSlots; ++c) {
    const int t = lane + 64 * c;
    if (t < d) {
      float o = acc[c] * c_cur;
      if (s.mode >= 2) o = fmaf(w_prev, accp[t], o);
      if (!valid) continue;
      if (s.mode == 1 || s.mode == 2) accp[t] = o;
      else st_elem(outp, t, o);
    }
  }
  if (valid && lane == 0) s.lse[row] = lse_new;
}

}  // namespace

usp_status launch_attn_generic(const AttnStep& step, hipStream_t st) {
  AttnStep s = step;
  if (s.d > kMaxD) {
    set_error("generic attention kernel supports d <= %d (got %d)", kMaxD, s.d);
    return USP_ERR_UNSUPPORTED;
  }
  s.copy_wgs = s.n_copy > 0 ? 32 : 0;
  dim3 grid((unsigned)((s.Sq + 3) / 4 + s.copy_wgs), (unsigned)s.H, (unsigned)s.B), block(256);
  if (s.qo_dtype == USP_F32 && s.kv_dtype == USP_F32)
    hipLaunchKernelGGL((attn_generic_kernel<float, float>), grid, block, 0, st, s);
  else if (s.qo_dtype == USP_BF16 && s.kv_dtype == USP_BF16)
    hipLaunchKernelGGL((attn_generic_kernel<bf16_t, bf16_t>), grid, block, 0, st, s);
  else if (s.qo_dtype == USP_BF16 && s.kv_dtype == USP_FP8_E4M3FN)
    hipLaunchKernelGGL((attn_generic_kernel<bf16_t, uint8_t>), grid, block, 0, st, s);
  else if (s.qo_dtype == USP_F32 && s.kv_dtype == USP_FP8_E4M3FN)
    hipLaunchKernelGGL((attn_generic_kernel<float, uint8_t>), grid, block, 0, st, s);
  else {
    set_error("no attention kernel for qo_dtype=%d kv_dtype=%d", s.qo_dtype, s.kv_dtype);
    return USP_ERR_UNSUPPORTED;
  }
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

}  // namespace usp
