// bf16 MFMA attention step for gfx950 (head dimension 128): for one KV chunk,
//   O_r = softmax(Q K^T * scale) V,   lse_r = log sum_j exp(q.k_j * scale)
// (FastUSP section 2.2 and 2.2.2), with the carried (O, lse) of earlier chunks folded in
// by the merge equations of section 3.4 in the epilogue.
//
// Shape of the computation (all choices are for 64-wide wavefronts and the 32x32x16 bf16
// MFMA, whose operands hold 8 consecutive contraction-index values per lane):
//   * A work-group owns 256 queries of one (batch, head); each of its 8 waves owns 32.
//   * Scores are computed TRANSPOSED, S^T = K Q^T (keys are MFMA rows, queries columns), so
//     a lane owns one query column: the row max / row sum of the online softmax are in-lane
//     reductions plus one exchange between lane l and lane l^32.
//   * The exponentiated tile P^T, already in registers in the accumulator layout, is cast to
//     bf16 and used directly as the B operand of O^T += V^T P^T; it never touches LDS.
//   * K tiles (64 keys) sit in LDS row-major; V tiles sit in LDS transposed ([d][key], keys
//     permuted inside blocks of 16 so that the 8 keys a lane needs are one 16-byte read).
//   * exp is taken in base 2 with scale * log2(e) folded into one FMA.
#include "usp_common.h"

namespace usp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;          // head dimension
constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kQPerWave = 32;
constexpr int kQPerWG = kWaves * kQPerWave;   // 256
constexpr int kTile = 64;        // keys per LDS tile
constexpr int kKPitch = kD + 8;  // bf16 elements per K row in LDS (272 B: conflict-free 16 B reads)
constexpr int kVPitch = kTile + 8;  // bf16 elements per V^T row in LDS (144 B)

struct Smem {
  bf16_t k[2][kTile * kKPitch];
  bf16_t vt[2][kD * kVPitch];
  float bias[2][kTile];   // 0 for a live key, -inf for a masked / out-of-range key
  float kmul[2][kTile];   // per-key score multiplier: softmax scale * log2(e) [* FP8 scale of the key]
  float vmul[2][kTile];   // per-key FP8 scale of the V row (only read when K/V came from FP8 codes)
  int any_masked[2];
};

// position of key offset o (0..15) inside its block of 16 in the V^T rows: the B operand of
// the P.V MFMA holds, for lane group g, accumulator registers 8*half + j, i.e. key offsets
// 8*(j/4) + 4*g + j%4; storing offset o at 8*g + j makes those 8 keys contiguous.
__device__ __forceinline__ int vpos(int o) { return 8 * ((o >> 2) & 1) + 4 * (o >> 3) + (o & 3); }

__device__ __forceinline__ float xlane32_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xlane32_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__global__ __launch_bounds__(kThreads, 2) void attn_mfma_kernel(AttnStep s) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int h = blockIdx.y, b = blockIdx.z;
  const int q0 = blockIdx.x * kQPerWG + wave * kQPerWave;

  const bf16_t* qb = (const bf16_t*)s.q + b * s.qs[0] + h * s.qs[1];
  const bf16_t* kb = (const bf16_t*)s.k + b * s.ks[0] + h * s.ks[1];
  const bf16_t* vb = (const bf16_t*)s.v + b * s.ks[0] + h * s.ks[1];
  const uint8_t* mask = s.key_mask ? s.key_mask + (int64_t)b * s.Sc : nullptr;
  // K/V given as exact bf16 copies of FP8 codes: value = code * scale[key]; the scales are applied
  // to the fp32 scores and to P, so the MFMAs run on exactly representable numbers
  const float* ksc = s.k_scale ? s.k_scale + ((int64_t)b * s.H + h) * s.Sc : nullptr;
  const float* vsc = s.v_scale ? s.v_scale + ((int64_t)b * s.H + h) * s.Sc : nullptr;
  const bool scaled = ksc != nullptr;
  const int Sc = s.Sc;
  const int ntiles = (Sc + kTile - 1) / kTile;

  // Q^T operand: lane (n, g) holds Q[q0+n][16*ks + 8*g .. +7] for ks = 0..7
  bf16x8 qreg[8];
  {
    const int qi = min(q0 + n, s.Sq - 1);
    const bf16_t* qr = qb + (int64_t)qi * s.qs[2] + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qr + 16 * ks);
  }

  f32x16 oacc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.0f;
  float m = -INFINITY;   // running max, in log2 units (score * scale * log2 e)
  float lsum = 0.0f;     // this lane's share of the running sum (its 32 of every 64 keys)
  const float scale2 = s.scale * 1.44269504088896340736f;

  // ---- tile loader: global -> registers -> LDS ------------------------------------------
  // thread tid moves 16-byte pieces c = tid and tid + 512 of the 64 x 256-byte K and V tiles
  uint4 kst0, kst1, vst0, vst1;
  const int ld_key0 = tid >> 4, ld_key1 = (tid + kThreads) >> 4, ld_dc = tid & 15;
  auto load_tile = [&](int t) {
    const int ka = min(t * kTile + ld_key0, Sc - 1), kc = min(t * kTile + ld_key1, Sc - 1);
    kst0 = *reinterpret_cast<const uint4*>(kb + (int64_t)ka * s.ks[2] + ld_dc * 8);
    vst0 = *reinterpret_cast<const uint4*>(vb + (int64_t)ka * s.ks[2] + ld_dc * 8);
    kst1 = *reinterpret_cast<const uint4*>(kb + (int64_t)kc * s.ks[2] + ld_dc * 8);
    vst1 = *reinterpret_cast<const uint4*>(vb + (int64_t)kc * s.ks[2] + ld_dc * 8);
  };
  auto store_piece = [&](int buf, int kk, const uint4& kq, const uint4& vq) {
    *reinterpret_cast<uint4*>(&sm.k[buf][kk * kKPitch + ld_dc * 8]) = kq;
    const int col = (kk & ~15) + vpos(kk & 15);
    bf16_t* dst = &sm.vt[buf][(ld_dc * 8) * kVPitch + col];
    dst[0 * kVPitch] = (bf16_t)(vq.x); dst[1 * kVPitch] = (bf16_t)(vq.x >> 16);
    dst[2 * kVPitch] = (bf16_t)(vq.y); dst[3 * kVPitch] = (bf16_t)(vq.y >> 16);
    dst[4 * kVPitch] = (bf16_t)(vq.z); dst[5 * kVPitch] = (bf16_t)(vq.z >> 16);
    dst[6 * kVPitch] = (bf16_t)(vq.w); dst[7 * kVPitch] = (bf16_t)(vq.w >> 16);
  };
  auto store_tile = [&](int t, int buf) {
    store_piece(buf, ld_key0, kst0, vst0);
    store_piece(buf, ld_key1, kst1, vst1);
    if (wave == 0) {
      const int key = t * kTile + lane;
      const bool live = key < Sc && (!mask || mask[key] != 0);
      sm.bias[buf][lane] = live ? 0.0f : -INFINITY;
      if (scaled) {
        const int kc = min(key, Sc - 1);
        sm.kmul[buf][lane] = ksc[kc] * scale2;
        sm.vmul[buf][lane] = vsc[kc];
      }
      const unsigned long long dead = __ballot(!live);
      if (lane == 0) sm.any_masked[buf] = dead != 0ull;
    }
  };

  if (ntiles > 0) {
    load_tile(0);
    store_tile(0, 0);
  }
  __syncthreads();

  for (int t = 0; t < ntiles; ++t) {
    const int buf = t & 1;
    if (t + 1 < ntiles) load_tile(t + 1);

    // ---- S^T = K Q^T for the two 32-key halves ------------------------------------------
    f32x16 sacc[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[kt][i] = 0.0f;
      const bf16_t* kr = &sm.k[buf][(32 * kt + n) * kKPitch + 8 * g];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(kr + 16 * ks);
        sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], sacc[kt], 0, 0, 0);
      }
    }

    // ---- online softmax, base 2 ----------------------------------------------------------
    if (sm.any_masked[buf]) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const float4 bz = *reinterpret_cast<const float4*>(&sm.bias[buf][32 * kt + 8 * i4 + 4 * g]);
          sacc[kt][4 * i4 + 0] += bz.x; sacc[kt][4 * i4 + 1] += bz.y;
          sacc[kt][4 * i4 + 2] += bz.z; sacc[kt][4 * i4 + 3] += bz.w;
        }
    }
    float mul = scale2;
    if (scaled) {   // per-key multipliers: scores leave this block already in log2 units
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const float4 cz = *reinterpret_cast<const float4*>(&sm.kmul[buf][32 * kt + 8 * i4 + 4 * g]);
          sacc[kt][4 * i4 + 0] *= cz.x; sacc[kt][4 * i4 + 1] *= cz.y;
          sacc[kt][4 * i4 + 2] *= cz.z; sacc[kt][4 * i4 + 3] *= cz.w;
        }
      mul = 1.0f;
    }
    float tmax = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, sacc[kt][i]);
    tmax = xlane32_max(tmax) * mul;              // mul > 0: max commutes with the scaling
    const float m_new = fmaxf(m, tmax);
    const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m - m_use);
    m = m_new;
    float psum = 0.0f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kt][i], mul, -m_use));
        sacc[kt][i] = p;
        psum += p;
      }
    lsum = lsum * alpha + psum;
    if (scaled) {   // P.V on codes: fold the V row scale into P
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const float4 cz = *reinterpret_cast<const float4*>(&sm.vmul[buf][32 * kt + 8 * i4 + 4 * g]);
          sacc[kt][4 * i4 + 0] *= cz.x; sacc[kt][4 * i4 + 1] *= cz.y;
          sacc[kt][4 * i4 + 2] *= cz.z; sacc[kt][4 * i4 + 3] *= cz.w;
        }
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;

    // ---- O^T += V^T P^T ---------------------------------------------------------------------
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        u32x4 pu;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          pu[j] = pack_bf16x2(sacc[kt][8 * half + 2 * j], sacc[kt][8 * half + 2 * j + 1]);
        const bf16x8 pb = __builtin_bit_cast(bf16x8, pu);
        const int col = 32 * kt + 16 * half + 8 * g;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(&sm.vt[buf][(32 * dt + n) * kVPitch + col]);
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, oacc[dt], 0, 0, 0);
        }
      }

    if (t + 1 < ntiles) store_tile(t + 1, buf ^ 1);
    __syncthreads();
  }

  // ---- chunk result, merge with carried state, store ------------------------------------
  const float l = xlane32_sum(lsum);
  const int qi = q0 + n;
  const bool valid = qi < s.Sq;
  const int64_t row = ((int64_t)b * s.H + h) * s.Sq + (valid ? qi : s.Sq - 1);
  float lse_r = -INFINITY, c_cur = 0.0f;
  if (l > 0.0f) { lse_r = (m + log2f(l)) * 0.69314718055994530942f; c_cur = 1.0f / l; }
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
  if (!valid) return;
  float* accp = s.acc ? s.acc + row * kD : nullptr;
  bf16_t* outp = (bf16_t*)s.out + b * s.os[0] + h * s.os[1] + (int64_t)qi * s.os[2];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const int dcol = 32 * dt + 8 * i4 + 4 * g;
      float o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = oacc[dt][4 * i4 + e] * c_cur;
      if (s.mode >= 2) {
        const float4 p = *reinterpret_cast<const float4*>(accp + dcol);
        o[0] = fmaf(w_prev, p.x, o[0]); o[1] = fmaf(w_prev, p.y, o[1]);
        o[2] = fmaf(w_prev, p.z, o[2]); o[3] = fmaf(w_prev, p.w, o[3]);
      }
      if (s.mode == 1 || s.mode == 2)
        *reinterpret_cast<float4*>(accp + dcol) = make_float4(o[0], o[1], o[2], o[3]);
      else
        *reinterpret_cast<uint2*>(outp + dcol) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
    }
  if (g == 0) s.lse[row] = lse_new;
}

}  // namespace

bool attn_mfma_supported(const AttnStep& s) {
  return s.qo_dtype == USP_BF16 && s.kv_dtype == USP_BF16 && s.d == kD && s.Sq > 0;
}

usp_status launch_attn_mfma(const AttnStep& s, hipStream_t st) {
  dim3 grid((unsigned)((s.Sq + kQPerWG - 1) / kQPerWG), (unsigned)s.H, (unsigned)s.B), block(kThreads);
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Smem));
  USP_CHECK_HIP(attr);
  hipLaunchKernelGGL(attn_mfma_kernel, grid, block, sizeof(Smem), st, s);
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

}  // namespace usp
