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
#include "prefetch_copy.h"

#ifndef LAB_STAMP
#define LAB_STAMP(slot)
#endif
#ifndef LAB_COUNT_SLOW
#define LAB_COUNT_SLOW()
#endif
#ifndef LAB_WG_START
#define LAB_WG_START()
#define LAB_WG_END()
#endif

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
constexpr int kQPerWGSplit = 4 * kQPerWave;     // 128: split kernel, two waves per 32 queries
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

// Work-group -> (batch*head, query block) with the 8 XCDs of the chip in mind: consecutive
// work-group ids go to consecutive XCDs (id % 8), each with its own L2.  The (head, query block)
// items, head-major, are cut into 8 contiguous ranges of equal length, one per XCD: the query
// blocks of a head stay on one XCD (two where a range boundary falls inside a head), so its K/V
// is fetched from HBM once or twice instead of once per XCD, and every XCD gets the same number
// of work-groups whatever the head count.  The grid holds 8 * ceil(items / 8) ids; ids past the
// last item return false.
constexpr int kXcds = 8;
constexpr int kSplitBelowWGs = 128;   // use the key-split kernel when 256-query work-groups number at most this
__device__ __forceinline__ bool wg_to_tile(int copy_wgs, int nqb, int bh_total, int& bh, int& qb) {
  const int id = blockIdx.x;                          // the copy work-groups are the last ids of the grid
  const int per_xcd = ((int)gridDim.x - copy_wgs) / kXcds;
  const int item = (id % kXcds) * per_xcd + id / kXcds;
  bh = item / nqb;
  qb = item - bh * nqb;
  return bh < bh_total;
}
static inline unsigned wg_grid_size(int nqb, int bh_total) {
  return (unsigned)(kXcds * ((bh_total * nqb + kXcds - 1) / kXcds));
}

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

// Chunk result from the running state (O~ = oacc, reference m in log2 units, this lane's part of l),
// merged with the carried (O, lse) of earlier chunks by the section 3.4 equations, and stored.
__device__ __forceinline__ void finish_and_store(const AttnStep& s, f32x16 (&oacc)[4], float m, float lsum,
                                                 int b, int h, int q0, int n, int g) {
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

__global__ __launch_bounds__(kThreads, 2) void attn_mfma_kernel(AttnStep s) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  int bh_, qb_;
  if (s.copy_wgs > 0 && blockIdx.x >= gridDim.x - s.copy_wgs) {   // prefetch work-group: copy and leave
    prefetch_copy(s, blockIdx.x - (gridDim.x - s.copy_wgs), threadIdx.x, kThreads);
    return;
  }
  if (!wg_to_tile(s.copy_wgs, (s.Sq + kQPerWG - 1) / kQPerWG, s.B * s.H, bh_, qb_)) return;   // whole work-group
  const int h = bh_ % s.H, b = bh_ / s.H;
  const int q0 = qb_ * kQPerWG + wave * kQPerWave;

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
    // pin Q in registers here: otherwise the waits for these loads sink into the key loop, where
    // they would also wait for the next tile's prefetch
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qreg[ks]));
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

  finish_and_store(s, oacc, m, lsum, b, h, q0, n, g);
}


// =============================================================================================
// Ping-pong kernel (fast path: no key mask, chunk length a multiple of 64, plain bf16 K/V).
//
// The 8 waves form two groups (waves 0-3 = A, 4-7 = B; each SIMD hosts one wave of each).  A
// wave alternates between a softmax phase SM(t) (VALU only: scores of tile t -> bf16 P) and a
// matrix phase MM(t) (MFMA only: O += P(t) V(t), then the scores of tile t+1).  Group B runs
// one phase behind group A and a work-group barrier separates the phases, so in every phase
// one wave of each SIMD feeds the matrix core while the other does the exponentials.
//   phase 2j   : A does SM(j),  B does MM(j-1)
//   phase 2j+1 : A does MM(j),  B does SM(j)
// K and V tiles are double-buffered in LDS and written by direct global->LDS loads, issued at
// the start of every odd phase for K(j+2) and V(j+1): each has two full phases to land.
// =============================================================================================
__device__ __forceinline__ void lds_dma16(const void* gbase, uint32_t lane_off, uint32_t lds_base) {
  // 64 lanes x 16 bytes from gbase (wave-uniform) + lane_off (per lane): lane i's 16 bytes land at
  // lds_base + 16*i.  Issued through inline asm so the compiler does not serialise later LDS reads
  // behind it; completion is awaited with an explicit vmcnt wait before the barrier that
  // publishes the tile.
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_base), "v"(lane_off), "s"(gbase) : "memory", "m0");
}
constexpr int kStages = 3;   // LDS tile buffers per tensor

struct SmemPP {
  unsigned char k[kStages][kTileB];
  unsigned char v[kStages][kTileB];
};

__device__ __forceinline__ u32x2 lds_read_tr3(const __attribute__((address_space(3))) unsigned char* p) {
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
  return __builtin_bit_cast(u32x2, r);
}

template <int N> struct IC { static constexpr int value = N; };
#ifndef USP_PREFETCH_READS
#define USP_PREFETCH_READS 12
#endif
constexpr int kPrefetchReads = USP_PREFETCH_READS;   // LDS reads in flight ahead of the first MFMA (8 or 12)

__global__ __launch_bounds__(kThreads, 2) void attn_mfma_pp_kernel(AttnStep s) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  SmemPP& sm = *reinterpret_cast<SmemPP*>(smem_raw);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it in an SGPR
  const int n = lane & 31, g = lane >> 5;
  int bh_, qb_;
  if (s.copy_wgs > 0 && blockIdx.x >= gridDim.x - s.copy_wgs) {   // prefetch work-group: copy and leave
    prefetch_copy(s, blockIdx.x - (gridDim.x - s.copy_wgs), threadIdx.x, kThreads);
    return;
  }
  if (!wg_to_tile(s.copy_wgs, (s.Sq + kQPerWG - 1) / kQPerWG, s.B * s.H, bh_, qb_)) return;   // whole work-group
  const int h = bh_ % s.H, b = bh_ / s.H;
  const int q0 = qb_ * kQPerWG + wave * kQPerWave;
  const bool grpA = wave < 4;
  LAB_WG_START();

  const bf16_t* qb = (const bf16_t*)s.q + b * s.qs[0] + h * s.qs[1];
  const unsigned char* kb = (const unsigned char*)((const bf16_t*)s.k + b * s.ks[0] + h * s.ks[1]);
  const unsigned char* vb = (const unsigned char*)((const bf16_t*)s.v + b * s.ks[0] + h * s.ks[1]);
  const int nt = s.Sc / kTile;          // host guarantees Sc % 64 == 0 and Sc > 0
  const float scale2 = s.scale * 1.44269504088896340736f;

  // ---- direct global->LDS tile loads: wave w moves rows 8w..8w+7 of a tile, 4 rows per instruction.
  // Per-lane byte offsets inside a tile are fixed; the tile base pointers advance as scalars.
  const int dma_r0 = 8 * wave + (lane >> 4), dma_r1 = dma_r0 + 4;
  const int dma_p = lane & 15;
  const uint32_t rowB = (uint32_t)(s.ks[2] * 2);   // bytes between keys in global memory
  const int64_t tileB = (int64_t)kTile * rowB;
  const uint32_t kg0 = dma_r0 * rowB + ((dma_p ^ (dma_r0 & 15)) << 4);
  const uint32_t kg1 = dma_r1 * rowB + ((dma_p ^ (dma_r1 & 15)) << 4);
  const uint32_t vg0 = dma_r0 * rowB + ((dma_p ^ ((dma_r0 & 3) << 2)) << 4);
  const uint32_t vg1 = dma_r1 * rowB + ((dma_p ^ ((dma_r1 & 3) << 2)) << 4);
  const uint32_t lds_k = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)&sm.k[0][0] + 8 * wave * kRowB);
  const uint32_t lds_v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)&sm.v[0][0] + 8 * wave * kRowB);
  auto issue_k_half = [&](const unsigned char* tile, int stage, int half) {
    lds_dma16(tile, half ? kg1 : kg0, lds_k + stage * kTileB + half * 4 * kRowB);
  };
  auto issue_v_half = [&](const unsigned char* tile, int stage, int half) {
    lds_dma16(tile, half ? vg1 : vg0, lds_v + stage * kTileB + half * 4 * kRowB);
  };

  // Tile loads are issued from the softmax phases (the phase whose critical resource, the VALU,
  // is not the matrix core): group A's SM(j) prefetches K(j+2) and V(j+1), group B's SM(j), one
  // phase later, K(j+3) and V(j+2).  Tiles needed before the first of those land are fetched here.
  issue_k_half(kb, 0, 0); issue_k_half(kb, 0, 1);
  issue_v_half(vb, 0, 0); issue_v_half(vb, 0, 1);
  if (nt > 1) { issue_k_half(kb + tileB, 1, 0); issue_k_half(kb + tileB, 1, 1); }
  if (!grpA) {
    if (nt > 1) { issue_v_half(vb + tileB, 1, 0); issue_v_half(vb + tileB, 1, 1); }
    if (nt > 2) { issue_k_half(kb + 2 * tileB, 2, 0); issue_k_half(kb + 2 * tileB, 2, 1); }
  }
  const unsigned char* kpre = kb + (grpA ? 2 : 3) * tileB;   // next K / V tile this wave prefetches
  const unsigned char* vpre = vb + (grpA ? 1 : 2) * tileB;

  // Q^T operand: lane (n, g) holds Q[q0+n][16*ks + 8*g .. +7] for ks = 0..7
  bf16x8 qreg[8];
  {
    const int qi = min(q0 + n, s.Sq - 1);
    const bf16_t* qr = qb + (int64_t)qi * s.qs[2] + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qr + 16 * ks);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qreg[ks]));
  }

  f32x16 oacc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.0f;
  f32x16 sacc[2];
  u32x4 pk[4];
  float m = -INFINITY, lsum = 0.0f;

  // per-lane LDS read addresses (see the layout notes at Smem): 8 for the K operand (one per 16-wide
  // slice of the head dimension), 4 for the V^T operand (one per 32-wide slice); stage, key block
  // and row offsets are compile-time immediates on top of these
  typedef const __attribute__((address_space(3))) unsigned char* lds_cptr;
  lds_cptr k_rd[8], v_rd[4];
  {
    const int k_rd_row = n * kRowB;
    const int k_rd_x = (g ^ (n & 15)) << 4;
    const int tr_i = (lane >> 2) & 3, tr_cc = lane & 3, tr_dh = (lane >> 4) & 1;
    const int v_rd_row = (4 * g + tr_i) * kRowB + ((2 * tr_dh + (tr_cc >> 1)) << 4) + 8 * (tr_cc & 1);
    const int v_rd_x = tr_i << 6;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      k_rd[ks] = (lds_cptr)(uintptr_t)((uint32_t)(uintptr_t)&sm.k[0][0] + k_rd_row + ((32 * ks) ^ k_rd_x));
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
      v_rd[dt] = (lds_cptr)(uintptr_t)((uint32_t)(uintptr_t)&sm.v[0][0] + v_rd_row + ((dt << 6) ^ v_rd_x));
  }

  // scores of the tile in LDS stage `stage`: sacc[kt] += K Q^T over head-dim slices ks_lo..ks_lo+3
  auto qk_block = [&](int stage, int kt, int ks_lo) {
#pragma unroll
    for (int ks = ks_lo; ks < ks_lo + 4; ++ks) {
      const bf16x8 a = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(
          k_rd[ks] + stage * kTileB + 32 * kt * kRowB);
      sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], sacc[kt], 0, 0, 0);
    }
  };
  // O^T += V^T P^T for the 16 keys of block blk of the tile in LDS stage `stage`
  auto pv_block = [&](int stage, int blk) {
    const bf16x8 pb = __builtin_bit_cast(bf16x8, pk[blk]);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      const u32x2 lo = lds_read_tr3(v_rd[dt] + stage * kTileB + 16 * blk * kRowB);
      const u32x2 hi = lds_read_tr3(v_rd[dt] + stage * kTileB + (16 * blk + 8) * kRowB);
      const u32x4 av = {lo[0], lo[1], hi[0], hi[1]};
      oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb, oacc[dt], 0, 0, 0);
    }
  };
  // matrix phase: O += P V (V tile in stage SV) interleaved with the scores of the next tile (K in
  // stage SK).  Only this wave feeds the SIMD's matrix core during the phase, so its LDS operand
  // reads are scheduled eight MFMAs ahead of their use (sched_group_barrier: 0x008 MFMA, 0x100 LDS read).
  auto MM_full = [&](int sv, int sk) {
    __builtin_amdgcn_s_setprio(2);
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[kt][i] = 0.0f;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      pv_block(sv, blk);
      qk_block(sk, blk >> 1, 4 * (blk & 1));
    }
    __builtin_amdgcn_sched_group_barrier(0x100, kPrefetchReads, 0);
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {   // P.V group
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, kPrefetchReads == 12 ? 2 : 1, 0);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {   // score group
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, kPrefetchReads == 12 ? 1 : 2, 0);
      }
    }
    __builtin_amdgcn_s_setprio(0);
  };
  auto MM_last = [&](int sv) {   // last tile: no further scores
    __builtin_amdgcn_s_setprio(2);
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) pv_block(sv, blk);
    __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
    __builtin_amdgcn_s_setprio(0);
  };
  // softmax phase: sacc (scores of one tile) -> pk (bf16 P), running reference m and sum l.
  // Fast path: exponentials are taken against the current reference m without first looking for
  // the tile's maximum; the row sum then certifies the result: if this lane's sum of P is at most
  // 2^16, no P exceeded 2^16, which fp32 accumulators and bf16 operands hold comfortably.  Only
  // when some lane fails that test (always on the first tile, where m = -inf makes every P inf)
  // does the wave find the true maximum, move m, rescale O and l, and redo the exponentials.
  // While it runs, the wave also issues its four tile loads (K into stage sk if do_k, V into stage
  // sv if do_v), spread between the exponential blocks so that the eight waves do not hit the
  // load path at once.
  auto exp_block = [&](int kt, int half, float& psum) {
    float p[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      p[j] = __builtin_amdgcn_exp2f(fmaf(sacc[kt][8 * half + j], scale2, -m));
      psum += p[j];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) pk[2 * kt + half][j] = pack_bf16x2(p[2 * j], p[2 * j + 1]);
    // anchor the block here, between the tile loads that surround it in program order
    asm volatile("" : "+v"(pk[2 * kt + half]));
  };
  auto SM = [&](int sk, int sv, bool do_k, bool do_v) {
    float psum = 0.0f;
    // sched_barrier: keep each load between two blocks of arithmetic (the scheduler would
    // otherwise hoist all four to the top, where they queue behind one another)
    if (do_k) issue_k_half(kpre, sk, 0);
    exp_block(0, 0, psum);
    __builtin_amdgcn_sched_barrier(0);
    if (do_k) issue_k_half(kpre, sk, 1);
    exp_block(0, 1, psum);
    __builtin_amdgcn_sched_barrier(0);
    if (do_v) issue_v_half(vpre, sv, 0);
    exp_block(1, 0, psum);
    __builtin_amdgcn_sched_barrier(0);
    if (do_v) issue_v_half(vpre, sv, 1);
    exp_block(1, 1, psum);
    __builtin_amdgcn_sched_barrier(0);
    kpre += tileB;
    vpre += tileB;
    if (__builtin_amdgcn_ballot_w64(!(psum <= 65536.0f)) != 0ull) {
      LAB_COUNT_SLOW();
      float tmax = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, sacc[kt][i]);
      const float m_new = fmaxf(m, xlane32_max(tmax) * scale2);
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);   // m = -inf (first tile) gives 0
      m = m_new;
      lsum *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;
      psum = 0.0f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int half = 0; half < 2; ++half) exp_block(kt, half, psum);
    }
    lsum += psum;
    // pin the results here: without a use in this phase the optimiser sinks the exponentials past
    // the barrier, next to their first use in the matrix phase
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) asm volatile("" : "+v"(pk[blk]));
    asm volatile("" : "+v"(lsum));
  };

  // prologue: the first tiles have landed -> scores of tile 0 in both groups
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[kt][i] = 0.0f;
    qk_block(0, kt, 0);
    qk_block(0, kt, 4);
  }

  // Both groups execute the same barrier sequence (two per tile index j = 0..nt); the steady-state
  // bodies are straight-line code so the accumulators stay in place.
  // sched_barrier(0): nothing may be moved across a phase boundary (the compiler would otherwise
  // sink the softmax arithmetic below the barrier, into the matrix phase of the same wave).
  // A wave waits for its own tile loads at the end of its softmax phases: the batch issued one
  // softmax phase earlier must have landed, the batch just issued (4 loads if full) may be in flight.
  auto phase_barrier = [&](int wait_mode) {   // 0: no wait, 1: vmcnt(4), 2: vmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
    if (wait_mode == 1) __builtin_amdgcn_s_waitcnt(0x0F74);
    else if (wait_mode == 2) __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };
  auto nxt = [](int x) { return x == 2 ? 0 : x + 1; };
  int st = 0;                            // LDS stage of tile j, j % 3
  if (grpA) {
    // tile j: phase 2j = SM(j), prefetching K(j+2) -> stage st+2, V(j+1) -> stage st+1;
    //         phase 2j+1 = MM(j) with V(j) in stage st, K(j+1) in stage st+1
    for (int j = 0; j < nt - 1; ++j) {
      const int s1 = nxt(st), s2 = nxt(s1);
      LAB_STAMP(6 * j);
      SM(s2, s1, j + 2 < nt, true);
      LAB_STAMP(6 * j + 1);
      phase_barrier(j + 2 < nt ? 1 : 2);
      LAB_STAMP(6 * j + 3);
      MM_full(st, s1);
      LAB_STAMP(6 * j + 5);
      phase_barrier(0);
      st = s1;
    }
    SM(0, 0, false, false);
    phase_barrier(2);
    MM_last(st);
    phase_barrier(0);
    phase_barrier(0);
    phase_barrier(0);
  } else {
    // tile j: phase 2j = MM(j-1) with V(j-1) in stage st-1, K(j) in stage st;
    //         phase 2j+1 = SM(j), prefetching K(j+3) -> stage st, V(j+2) -> stage st+2
    phase_barrier(0);                                 // phase 0: nothing to do yet
    SM(0, 2, 3 < nt, 2 < nt);                         // phase 1 (tile 0)
    phase_barrier(3 < nt ? 1 : 2);
    for (int j = 1; j < nt; ++j) {
      const int sp = st;                              // stage of tile j-1
      st = nxt(st);
      LAB_STAMP(6 * j);
      MM_full(sp, st);
      LAB_STAMP(6 * j + 1);
      phase_barrier(0);
      LAB_STAMP(6 * j + 3);
      SM(st, sp, j + 3 < nt, j + 2 < nt);             // st+2 == sp (mod 3)
      LAB_STAMP(6 * j + 5);
      phase_barrier(j + 3 < nt ? 1 : 2);
    }
    MM_last(st);
    phase_barrier(0);
    phase_barrier(0);
  }
  LAB_WG_END();

  finish_and_store(s, oacc, m, lsum, b, h, q0, n, g);
}

__global__ __launch_bounds__(kThreads, 2) void attn_mfma_pp_split_kernel(AttnStep s) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  SmemPP& sm = *reinterpret_cast<SmemPP*>(smem_raw);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it in an SGPR
  const int n = lane & 31, g = lane >> 5;
  int bh_, qb_;
  if (s.copy_wgs > 0 && blockIdx.x >= gridDim.x - s.copy_wgs) {   // prefetch work-group: copy and leave
    prefetch_copy(s, blockIdx.x - (gridDim.x - s.copy_wgs), threadIdx.x, kThreads);
    return;
  }
  if (!wg_to_tile(s.copy_wgs, (s.Sq + kQPerWGSplit - 1) / kQPerWGSplit, s.B * s.H, bh_, qb_)) return;   // whole work-group
  const int h = bh_ % s.H, b = bh_ / s.H;
  const int q0 = qb_ * kQPerWGSplit + (wave & 3) * kQPerWave;   // waves w and w+4 share their 32 queries
  const bool grpA = wave < 4;
  LAB_WG_START();

  const bf16_t* qb = (const bf16_t*)s.q + b * s.qs[0] + h * s.qs[1];
  const unsigned char* kb = (const unsigned char*)((const bf16_t*)s.k + b * s.ks[0] + h * s.ks[1]);
  const unsigned char* vb = (const unsigned char*)((const bf16_t*)s.v + b * s.ks[0] + h * s.ks[1]);
  const int nt = s.Sc / kTile;          // host guarantees Sc % 64 == 0 and Sc > 0
  const float scale2 = s.scale * 1.44269504088896340736f;

  // ---- direct global->LDS tile loads: wave w moves rows 8w..8w+7 of a tile, 4 rows per instruction.
  // Per-lane byte offsets inside a tile are fixed; the tile base pointers advance as scalars.
  const int dma_r0 = 8 * wave + (lane >> 4), dma_r1 = dma_r0 + 4;
  const int dma_p = lane & 15;
  const uint32_t rowB = (uint32_t)(s.ks[2] * 2);   // bytes between keys in global memory
  const int64_t tileB = (int64_t)kTile * rowB;
  const uint32_t kg0 = dma_r0 * rowB + ((dma_p ^ (dma_r0 & 15)) << 4);
  const uint32_t kg1 = dma_r1 * rowB + ((dma_p ^ (dma_r1 & 15)) << 4);
  const uint32_t vg0 = dma_r0 * rowB + ((dma_p ^ ((dma_r0 & 3) << 2)) << 4);
  const uint32_t vg1 = dma_r1 * rowB + ((dma_p ^ ((dma_r1 & 3) << 2)) << 4);
  const uint32_t lds_k = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)&sm.k[0][0] + 8 * wave * kRowB);
  const uint32_t lds_v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)&sm.v[0][0] + 8 * wave * kRowB);
  auto issue_k_half = [&](const unsigned char* tile, int stage, int half) {
    lds_dma16(tile, half ? kg1 : kg0, lds_k + stage * kTileB + half * 4 * kRowB);
  };
  auto issue_v_half = [&](const unsigned char* tile, int stage, int half) {
    lds_dma16(tile, half ? vg1 : vg0, lds_v + stage * kTileB + half * 4 * kRowB);
  };
  // the same rows of the partner wave (w ^ 4): 32 rows away, same swizzle (32 is a multiple of 16)
  const int64_t pair_g = (grpA ? 32 : -32) * (int64_t)rowB;
  const int pair_l = (grpA ? 32 : -32) * kRowB;
  auto issue_k_pair = [&](const unsigned char* tile, int stage, int half) {
    lds_dma16(tile + pair_g, half ? kg1 : kg0, lds_k + pair_l + stage * kTileB + half * 4 * kRowB);
  };
  auto issue_v_pair = [&](const unsigned char* tile, int stage, int half) {
    lds_dma16(tile + pair_g, half ? vg1 : vg0, lds_v + pair_l + stage * kTileB + half * 4 * kRowB);
  };

  // The group in its softmax phase p issues the whole batch of that phase, K(p+3) and V(p+1), both
  // first read in phase p+2: each wave its own rows and those of its partner in the other group,
  // whose matrix phase is not to be held up by load issue.  Tiles needed before the first batches
  // land are fetched here.
  issue_k_half(kb, 0, 0); issue_k_half(kb, 0, 1);
  issue_v_half(vb, 0, 0); issue_v_half(vb, 0, 1);
  if (nt > 1) { issue_k_half(kb + tileB, 1, 0); issue_k_half(kb + tileB, 1, 1); }
  if (nt > 2) { issue_k_half(kb + 2 * tileB, 2, 0); issue_k_half(kb + 2 * tileB, 2, 1); }
  const unsigned char* kpre = kb + (grpA ? 3 : 4) * tileB;   // K(p+3) / V(p+1) of this group's first
  const unsigned char* vpre = vb + (grpA ? 1 : 2) * tileB;   // softmax phase, p = 0 (A) or 1 (B)

  // Q^T operand: lane (n, g) holds Q[q0+n][16*ks + 8*g .. +7] for ks = 0..7
  bf16x8 qreg[8];
  {
    const int qi = min(q0 + n, s.Sq - 1);
    const bf16_t* qr = qb + (int64_t)qi * s.qs[2] + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qr + 16 * ks);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qreg[ks]));
  }

  f32x16 oacc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.0f;
  f32x16 sacc[2];
  u32x4 pk[4];
  float m = -INFINITY, lsum = 0.0f;

  // per-lane LDS read addresses (see the layout notes at Smem): 8 for the K operand (one per 16-wide
  // slice of the head dimension), 4 for the V^T operand (one per 32-wide slice); stage, key block
  // and row offsets are compile-time immediates on top of these
  typedef const __attribute__((address_space(3))) unsigned char* lds_cptr;
  lds_cptr k_rd[8], v_rd[4];
  {
    const int k_rd_row = n * kRowB;
    const int k_rd_x = (g ^ (n & 15)) << 4;
    const int tr_i = (lane >> 2) & 3, tr_cc = lane & 3, tr_dh = (lane >> 4) & 1;
    const int v_rd_row = (4 * g + tr_i) * kRowB + ((2 * tr_dh + (tr_cc >> 1)) << 4) + 8 * (tr_cc & 1);
    const int v_rd_x = tr_i << 6;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      k_rd[ks] = (lds_cptr)(uintptr_t)((uint32_t)(uintptr_t)&sm.k[0][0] + k_rd_row + ((32 * ks) ^ k_rd_x));
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
      v_rd[dt] = (lds_cptr)(uintptr_t)((uint32_t)(uintptr_t)&sm.v[0][0] + v_rd_row + ((dt << 6) ^ v_rd_x));
  }

  // scores of the tile in LDS stage `stage`: sacc[kt] += K Q^T over head-dim slices ks_lo..ks_lo+3
  auto qk_block = [&](int stage, int kt, int ks_lo) {
#pragma unroll
    for (int ks = ks_lo; ks < ks_lo + 4; ++ks) {
      const bf16x8 a = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(
          k_rd[ks] + stage * kTileB + 32 * kt * kRowB);
      sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], sacc[kt], 0, 0, 0);
    }
  };
  // O^T += V^T P^T for the 16 keys of block blk of the tile in LDS stage `stage`
  auto pv_block = [&](int stage, int blk) {
    const bf16x8 pb = __builtin_bit_cast(bf16x8, pk[blk]);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      const u32x2 lo = lds_read_tr3(v_rd[dt] + stage * kTileB + 16 * blk * kRowB);
      const u32x2 hi = lds_read_tr3(v_rd[dt] + stage * kTileB + (16 * blk + 8) * kRowB);
      const u32x4 av = {lo[0], lo[1], hi[0], hi[1]};
      oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb, oacc[dt], 0, 0, 0);
    }
  };
  // matrix phase: O += P V (V tile in stage SV) interleaved with the scores of the next tile (K in
  // stage SK).  Only this wave feeds the SIMD's matrix core during the phase, so its LDS operand
  // reads are scheduled eight MFMAs ahead of their use (sched_group_barrier: 0x008 MFMA, 0x100 LDS read).
  auto MM_full = [&](int sv, int sk) {
    __builtin_amdgcn_s_setprio(2);
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[kt][i] = 0.0f;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      pv_block(sv, blk);
      qk_block(sk, blk >> 1, 4 * (blk & 1));
    }
    __builtin_amdgcn_sched_group_barrier(0x100, kPrefetchReads, 0);
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {   // P.V group
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, kPrefetchReads == 12 ? 2 : 1, 0);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {   // score group
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, kPrefetchReads == 12 ? 1 : 2, 0);
      }
    }
    __builtin_amdgcn_s_setprio(0);
  };
  auto MM_last = [&](int sv) {   // last tile: no further scores
    __builtin_amdgcn_s_setprio(2);
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) pv_block(sv, blk);
    __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
    __builtin_amdgcn_s_setprio(0);
  };
  // softmax phase: sacc (scores of one tile) -> pk (bf16 P), running reference m and sum l.
  // Fast path: exponentials are taken against the current reference m without first looking for
  // the tile's maximum; the row sum then certifies the result: if this lane's sum of P is at most
  // 2^16, no P exceeded 2^16, which fp32 accumulators and bf16 operands hold comfortably.  Only
  // when some lane fails that test (always on the first tile, where m = -inf makes every P inf)
  // does the wave find the true maximum, move m, rescale O and l, and redo the exponentials.
  // While it runs, the wave also issues its four tile loads (K into stage sk if do_k, V into stage
  // sv if do_v), spread between the exponential blocks so that the eight waves do not hit the
  // load path at once.
  auto exp_block = [&](int kt, int half, float& psum) {
    float p[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      p[j] = __builtin_amdgcn_exp2f(fmaf(sacc[kt][8 * half + j], scale2, -m));
      psum += p[j];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) pk[2 * kt + half][j] = pack_bf16x2(p[2 * j], p[2 * j + 1]);
    // anchor the block here, between the tile loads that surround it in program order
    asm volatile("" : "+v"(pk[2 * kt + half]));
  };
  auto SM = [&](int sk, int sv, bool do_k, bool do_v) {
    float psum = 0.0f;
    // sched_barrier: keep each load between two blocks of arithmetic (the scheduler would
    // otherwise hoist all four to the top, where they queue behind one another)
    if (do_v) { issue_v_half(vpre, sv, 0); issue_v_pair(vpre, sv, 0); }
    exp_block(0, 0, psum);
    __builtin_amdgcn_sched_barrier(0);
    if (do_v) { issue_v_half(vpre, sv, 1); issue_v_pair(vpre, sv, 1); }
    exp_block(0, 1, psum);
    __builtin_amdgcn_sched_barrier(0);
    if (do_k) { issue_k_half(kpre, sk, 0); issue_k_pair(kpre, sk, 0); }
    exp_block(1, 0, psum);
    __builtin_amdgcn_sched_barrier(0);
    if (do_k) { issue_k_half(kpre, sk, 1); issue_k_pair(kpre, sk, 1); }
    exp_block(1, 1, psum);
    __builtin_amdgcn_sched_barrier(0);
    kpre += 2 * tileB;
    vpre += 2 * tileB;
    if (__builtin_amdgcn_ballot_w64(!(psum <= 65536.0f)) != 0ull) {
      LAB_COUNT_SLOW();
      float tmax = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, sacc[kt][i]);
      const float m_new = fmaxf(m, xlane32_max(tmax) * scale2);
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);   // m = -inf (first tile) gives 0
      m = m_new;
      lsum *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;
      psum = 0.0f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int half = 0; half < 2; ++half) exp_block(kt, half, psum);
    }
    lsum += psum;
    // pin the results here: without a use in this phase the optimiser sinks the exponentials past
    // the barrier, next to their first use in the matrix phase
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) asm volatile("" : "+v"(pk[blk]));
    asm volatile("" : "+v"(lsum));
  };

  // prologue: the first tiles have landed -> scores of tile 0 (group A) / tile 1 (group B)
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  __builtin_amdgcn_s_barrier();
  if (grpA || nt > 1) {
    const int st0 = grpA ? 0 : 1;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[kt][i] = 0.0f;
      qk_block(st0, kt, 0);
      qk_block(st0, kt, 4);
    }
  }

  // Phases p = 0..nt, one work-group barrier each.  Group A owns the even tiles, group B the odd
  // ones: in phase p the owner of tile p runs SM(p) while the other group runs MM(p-1), i.e.
  // O += P(p-1) V(p-1) and the scores of its next tile p+1.  Both groups execute nt + 1 barriers.
  //   reads in phase p : V(p-1) from stage (p-1)%3, K(p+1) from stage (p+1)%3
  //   batch of phase p : K(p+3) -> stage p%3 (last read, as K(p), in phase p-1),
  //                      V(p+1) -> stage (p+1)%3 (last read, as V(p-2), in phase p-1)
  //   end of phase p   : the batch of phase p-1 must have landed (first read in phase p+1); its
  //                      issuers are the group now ending a matrix phase, which waits for all of
  //                      its loads; the other group has only this phase's batch in flight
  auto end_phase = [&](bool wait_loads) {
    __builtin_amdgcn_sched_barrier(0);
    if (wait_loads) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };
  auto nxt = [](int x) { return x == 2 ? 0 : x + 1; };
  int t = grpA ? 0 : 1;                  // this group's current tile; SM(t) runs in phase t
  int st = t;                            // t % 3
  if (!grpA) end_phase(false);           // phase 0: group B has no scores yet
  while (t + 2 < nt) {
    LAB_STAMP(6 * t);
    SM(st, nxt(st), t + 3 < nt, true);                   // phase t (t + 1 < nt holds here)
    LAB_STAMP(6 * t + 1);
    end_phase(false);
    LAB_STAMP(6 * t + 2);
    const int s2 = nxt(nxt(st));                         // (t + 2) % 3
    MM_full(st, s2);                                     // phase t + 1
    LAB_STAMP(6 * t + 3);
    LAB_STAMP(6 * t + 4);
    end_phase(true);
    LAB_STAMP(6 * t + 5);
    t += 2;
    st = s2;
  }
  if (t < nt) {                                          // this group's last tile
    SM(st, nxt(st), false, t + 1 < nt);
    end_phase(false);
    MM_last(st);
    end_phase(true);
    t += 2;
  }
  // the group whose last matrix phase was phase nt-1 sits out phase nt
  if ((grpA && (nt % 2 == 0)) || (!grpA && (nt % 2 == 1))) end_phase(false);

  // ---- fold group B's partial state into group A's (same queries, disjoint keys) ----------------
  // all tile reads are behind the last barrier, so the tile buffers are reused for the exchange:
  // float slot i of wave w, lane l sits at x[(w * 66 + i) * 64 + l]
  float* xch = reinterpret_cast<float*>(smem_raw);
  if (!grpA) {
    float* dst = xch + ((wave - 4) * 66) * 64 + lane;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) dst[(16 * dt + i) * 64] = oacc[dt][i];
    dst[64 * 64] = m;
    dst[65 * 64] = lsum;
  }
  __syncthreads();
  if (!grpA) return;
  {
    const float* src = xch + (wave * 66) * 64 + lane;
    const float mB = src[64 * 64], lB = src[65 * 64];
    const float mm = fmaxf(m, mB);
    const float wa = (mm == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(m - mm);
    const float wb = (mm == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mB - mm);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[dt][i] = wa * oacc[dt][i] + wb * src[(16 * dt + i) * 64];
    lsum = wa * lsum + wb * lB;
    m = mm;
  }
  LAB_WG_END();

  finish_and_store(s, oacc, m, lsum, b, h, q0, n, g);
}


}  // namespace

bool attn_mfma_supported(const AttnStep& s) {
  return s.qo_dtype == USP_BF16 && s.kv_dtype == USP_BF16 && s.d == kD && s.Sq > 0;
}

usp_status launch_attn_mfma(const AttnStep& step, hipStream_t st) {
  AttnStep s = step;
  dim3 block(kThreads);
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Smem));
  USP_CHECK_HIP(attr);
  static const hipError_t attr_pp = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_pp_kernel),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(SmemPP));
  USP_CHECK_HIP(attr_pp);
  static const hipError_t attr_sp = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_pp_split_kernel),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(SmemPP));
  USP_CHECK_HIP(attr_sp);
  const bool fast = s.Sc > 0 && s.Sc % kTile == 0 && !s.key_mask && !s.k_scale;
  // Few query blocks (a small Q shard of a ring step): 256-query work-groups would leave CUs idle;
  // 128-query work-groups whose two wave groups split the keys fill twice as many.
  const unsigned wgs256 = wg_grid_size((s.Sq + kQPerWG - 1) / kQPerWG, s.B * s.H);
  const bool split = s.variant == 2 || (s.variant == 0 && (int)wgs256 <= kSplitBelowWGs);
  if (fast && split) {
    const unsigned wgs = wg_grid_size((s.Sq + kQPerWGSplit - 1) / kQPerWGSplit, s.B * s.H);
    s.copy_wgs = prefetch_wg_count(s, (int)wgs, 1);
    hipLaunchKernelGGL(attn_mfma_pp_split_kernel, dim3(wgs + s.copy_wgs), block, sizeof(SmemPP), st, s);
  } else {
    s.copy_wgs = prefetch_wg_count(s, (int)wgs256, 2);
    if (fast) hipLaunchKernelGGL(attn_mfma_pp_kernel, dim3(wgs256 + s.copy_wgs), block, sizeof(SmemPP), st, s);
    else hipLaunchKernelGGL(attn_mfma_kernel, dim3(wgs256 + s.copy_wgs), block, sizeof(Smem), st, s);
  }
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

}  // namespace usp
