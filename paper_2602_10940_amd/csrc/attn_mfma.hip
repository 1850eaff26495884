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
//   * K and V tiles (64 keys) sit in LDS row-major, XOR-swizzled instead of padded; the V^T
//     operand (8 keys of one head-dim column per lane) comes from the LDS transposing read.
//   * O and l are rescaled lazily: only when a row max has outgrown the exponent reference.
//   * exp is taken in base 2 with scale * log2(e) folded into one FMA.
#include "usp_common.h"

namespace usp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kD = 128;          // head dimension
constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kQPerWave = 32;
constexpr int kQPerWG = kWaves * kQPerWave;   // 256
constexpr int kTile = 64;        // keys per LDS tile
constexpr int kRowB = kD * 2;    // bytes per K / V row in LDS (256, unpadded)
constexpr int kTileB = kTile * kRowB;          // 16 KB
constexpr float kLazyTau = 8.0f; // the exponent reference is only moved when the max grows by > 2^8

// K and V tiles are row-major [key][128 bf16] in LDS without padding; bank conflicts are
// avoided by XOR-swizzling the sixteen 16-byte pieces of a row:
//   K: piece c of key r sits at piece c ^ (r & 15)       (16-byte MFMA operand reads of 16 rows)
//   V: piece c of key r sits at piece c ^ ((r & 3) << 2) (transposing 8-byte reads of 4 rows)
struct Smem {
  unsigned char k[2][kTileB];
  unsigned char v[2][kTileB];
  float bias[2][kTile];   // 0 for a live key, -inf for a masked / out-of-range key
  float kmul[2][kTile];   // per-key score multiplier: softmax scale * log2(e) * FP8 scale of the key
  float vmul[2][kTile];   // per-key FP8 scale of the V row (only read when K/V came from FP8 codes)
  int any_masked[2];
};

__device__ __forceinline__ float xlane32_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xlane32_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// LDS transposing read: the 16 lanes of a group each name 8 bytes; seen as a 4 x 16 matrix of
// bf16 (row i = the data of lanes 4i..4i+3), lane j of the group receives column j.
__device__ __forceinline__ u32x2 lds_read_tr(const unsigned char* p) {
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(p));
  return __builtin_bit_cast(u32x2, r);
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
  float m = -INFINITY;   // exponent reference (>= running max - tau), log2 units
  float lsum = 0.0f;     // this lane's share of the running sum (its 32 of every 64 keys)
  const float scale2 = s.scale * 1.44269504088896340736f;

  // ---- tile loader: global -> registers -> LDS ------------------------------------------
  // thread tid moves 16-byte pieces tid and tid + 512 of the 64 x 256-byte K and V tiles
  uint4 kst0, kst1, vst0, vst1;
  const int ld_key0 = tid >> 4, ld_key1 = (tid + kThreads) >> 4, ld_c = tid & 15;
  const int k_dst0 = ld_key0 * kRowB + ((ld_c ^ (ld_key0 & 15)) << 4);
  const int k_dst1 = ld_key1 * kRowB + ((ld_c ^ (ld_key1 & 15)) << 4);
  const int v_dst0 = ld_key0 * kRowB + ((ld_c ^ ((ld_key0 & 3) << 2)) << 4);
  const int v_dst1 = ld_key1 * kRowB + ((ld_c ^ ((ld_key1 & 3) << 2)) << 4);
  auto load_tile = [&](int t) {
    const int ka = min(t * kTile + ld_key0, Sc - 1), kc = min(t * kTile + ld_key1, Sc - 1);
    kst0 = *reinterpret_cast<const uint4*>(kb + (int64_t)ka * s.ks[2] + ld_c * 8);
    vst0 = *reinterpret_cast<const uint4*>(vb + (int64_t)ka * s.ks[2] + ld_c * 8);
    kst1 = *reinterpret_cast<const uint4*>(kb + (int64_t)kc * s.ks[2] + ld_c * 8);
    vst1 = *reinterpret_cast<const uint4*>(vb + (int64_t)kc * s.ks[2] + ld_c * 8);
  };
  auto store_tile = [&](int t, int buf) {
    *reinterpret_cast<uint4*>(&sm.k[buf][k_dst0]) = kst0;
    *reinterpret_cast<uint4*>(&sm.k[buf][k_dst1]) = kst1;
    *reinterpret_cast<uint4*>(&sm.v[buf][v_dst0]) = vst0;
    *reinterpret_cast<uint4*>(&sm.v[buf][v_dst1]) = vst1;
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

  // ---- per-lane LDS read offsets ------------------------------------------------------------
  // K operand (S^T = K Q^T): lane (n, g) reads key 32*kt + n, piece 2*ks + g, swizzled by n & 15
  const int k_rd_row = n * kRowB;
  const int k_rd_x = (g ^ (n & 15)) << 4;            // piece (2ks+g) ^ (n&15) = (2ks) ^ (g ^ (n&15))
  // V^T operand (O^T += V^T P^T), transposing read: lane l = 16*grp + 4*i + cc supplies the 8 bytes
  // of key (16*blk + 4*g + i [+8]), head-dim 32*dt + 16*(grp&1) + 4*cc .. +3
  const int tr_i = (lane >> 2) & 3, tr_cc = lane & 3, tr_dh = (lane >> 4) & 1;
  const int v_rd_row = (4 * g + tr_i) * kRowB + ((2 * tr_dh + (tr_cc >> 1)) << 4) + 8 * (tr_cc & 1);
  const int v_rd_x = tr_i << 6;                        // piece swizzle (key & 3) << 2, in bytes

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
      const unsigned char* kr = &sm.k[buf][32 * kt * kRowB + k_rd_row];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(kr + ((32 * ks) ^ k_rd_x));
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
    // Lazy rescaling: the reference m only moves when some query's max outgrew it by more than
    // tau (P then stays below 2^tau, harmless in fp32 / bf16); otherwise O and l are left alone.
    if (__builtin_amdgcn_ballot_w64(tmax > m + kLazyTau) != 0ull) {
      const float m_new = fmaxf(m, tmax);
      const float alpha = __builtin_amdgcn_exp2f(m - ((m_new == -INFINITY) ? 0.0f : m_new));
      m = m_new;
      lsum *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;
    }
    const float m_use = (m == -INFINITY) ? 0.0f : m;
    float psum = 0.0f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kt][i], mul, -m_use));
        sacc[kt][i] = p;
        psum += p;
      }
    lsum += psum;
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

    // ---- O^T += V^T P^T ---------------------------------------------------------------------
    // P^T block (kt, half) = accumulator registers 8*half .. 8*half+7 of sacc[kt]; for lane group g
    // register j is key 32*kt + 16*half + 8*(j/4) + 4*g + j%4, which is exactly the order the two
    // transposing reads below deliver V in (keys +0..3 then +8..11 of the 16-key block, offset 4*g).
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        u32x4 pu;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          pu[j] = pack_bf16x2(sacc[kt][8 * half + 2 * j], sacc[kt][8 * half + 2 * j + 1]);
        const bf16x8 pb = __builtin_bit_cast(bf16x8, pu);
        const unsigned char* vr = &sm.v[buf][(32 * kt + 16 * half) * kRowB + v_rd_row];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const int off = (dt << 6) ^ v_rd_x;
          const u32x2 lo = lds_read_tr(vr + off);
          const u32x2 hi = lds_read_tr(vr + 8 * kRowB + off);
          const u32x4 av = {lo[0], lo[1], hi[0], hi[1]};
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb, oacc[dt], 0, 0, 0);
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
