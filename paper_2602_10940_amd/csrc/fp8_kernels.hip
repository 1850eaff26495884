// FP8 (E4M3, OCP "fn": max 448, no infinities) pack / unpack of the All-to-All and ring
// payloads: FastUSP Algorithm 1 lines 1-2 (quantise) and line 4 (dequantise), with one
// scale per row of the [rows, cols] view.
//
// Both kernels are single streaming passes: the quantiser keeps a row in registers
// between the absmax reduction and the cast, so every input byte is read from HBM
// once.  All HBM accesses are 16-byte (or 8-byte) vectors, consecutive lanes touching
// consecutive addresses.
#include <type_traits>

#include "usp_common.h"
#include "fp8_arith.h"

namespace usp {
namespace {

// Launches whose output is smaller than these are written with streaming stores (see store8_nt):
// the dequantiser's 2- or 4-byte outputs up to 64 MB (measured crossover between 57 and 85 MB), the
// quantiser's codes, a third of its traffic, up to 256 MB (faster at every size measured, to 114 MB)
constexpr int64_t kStreamDequantBelowBytes = 64ll << 20;
constexpr int64_t kStreamQuantBelowBytes = 256ll << 20;


// ---- loads of 8 consecutive elements as fp32 --------------------------------------------
// kStream: streaming load, for single-pass kernels on launches small next to the L2s (9.5 instead of
// 10.0 us on the 28 MB FLUX payload; slower on a 226 MB one)
template <bool kStream = false>
__device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
  typedef uint32_t u32x4_l __attribute__((ext_vector_type(4)));
  const u32x4_l r = kStream ? __builtin_nontemporal_load(reinterpret_cast<const u32x4_l*>(p))
                            : *reinterpret_cast<const u32x4_l*>(p);
  v[0] = __uint_as_float(r[0] << 16); v[1] = __uint_as_float(r[0] & 0xffff0000u);
  v[2] = __uint_as_float(r[1] << 16); v[3] = __uint_as_float(r[1] & 0xffff0000u);
  v[4] = __uint_as_float(r[2] << 16); v[5] = __uint_as_float(r[2] & 0xffff0000u);
  v[6] = __uint_as_float(r[3] << 16); v[7] = __uint_as_float(r[3] & 0xffff0000u);
}
template <bool kStream = false>
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  float4 a = *reinterpret_cast<const float4*>(p);
  float4 b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// Eight codes to memory; streaming (non-temporal) when the launch is small: see the note at store8_nt.
template <bool kNT>
__device__ __forceinline__ void put_codes(uint8_t* p, uint2 w) {
  typedef uint32_t u32x2_v __attribute__((ext_vector_type(2)));
  if (kNT) {
    const u32x2_v v = {w.x, w.y};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x2_v*>(p));
  } else {
    *reinterpret_cast<uint2*>(p) = w;
  }
}

// ---- rows that fit one wave: LPR lanes per row, up to NV 8-element units per lane ---------
// Mapped variants (kMapped): the row id is split into (i0..i3) and the row is read from / written to
// sum_k i_k * stride[k]; everything else is the same code.
__device__ __forceinline__ void map_row(const RowMap& m, int64_t row, int64_t& src, int64_t& dst) {
  const int64_t a = row / m.n3, i3 = row - a * m.n3;
  const int64_t b = a / m.n2, i2 = a - b * m.n2;
  const int64_t i0 = b / m.n1, i1 = b - i0 * m.n1;
  src = i0 * m.src[0] + i1 * m.src[1] + i2 * m.src[2] + i3 * m.src[3];
  dst = i0 * m.dst[0] + i1 * m.dst[1] + i2 * m.dst[2] + i3 * m.dst[3];
}

template <typename T, int LPR, int NV, bool kMapped = false, bool kNT = false, bool kStreamIn = false>
__global__ __launch_bounds__(256) void fp8_quant_rows_kernel(const T* __restrict__ x,
                                                             uint8_t* __restrict__ q,
                                                             float* __restrict__ scales,
                                                             int64_t rows, int units, RowMap map) {
  constexpr int RPW = 64 / LPR;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int64_t row = ((int64_t)blockIdx.x * 4 + wave) * RPW + lane / LPR;
  const int l = lane % LPR;
  const bool row_ok = row < rows;
  int64_t base = row * (int64_t)units * 8;   // first element of the row in x
  int64_t orow = row;                         // row of q / scales
  if (kMapped) {
    map_row(map, row_ok ? row : 0, base, orow);
  }
  const int64_t obase = orow * (int64_t)units * 8;

  float v[NV][8];
  float a = 0.0f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int u = l + i * LPR;
    if (row_ok && u < units) {
      load8<kStreamIn>(x + base + (int64_t)u * 8, v[i]);
      a = absmax8(v[i], a);
    }
  }
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) a = fmaxf(a, __shfl_xor(a, off, 64));
  const float s = scale_from_absmax(a);
  if (row_ok && l == 0) scales[orow] = s;
  const RowDiv d = make_rowdiv(s);
  if (__builtin_amdgcn_ballot_w64(!d.fast) == 0ull) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int u = l + i * LPR;
      if (row_ok && u < units) put_codes<kNT>(q + obase + (int64_t)u * 8, encode8<true>(v[i], d));
    }
  } else {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int u = l + i * LPR;
      if (row_ok && u < units) put_codes<kNT>(q + obase + (int64_t)u * 8, encode8<false>(v[i], d));
    }
  }
}

// The same for bf16 input, which is the payload type of the method: a row stays in registers as the
// packed pairs it was loaded as (4 registers per 8 elements instead of 8), its |x| maximum is taken on
// the bit patterns two elements at a time, and rows in the fast range are cast with the short
// sequence of fp8_arith.h (5 instead of 8.5 VALU operations per element; the arithmetic, not the
// memory system, was what the waves of a row spent most of their time on).
// kFull: every row has exactly LPR * NV units (the FLUX payload: 384 = 64 * 6; K/V rows of one head:
// 16 = 16 * 1), so no access needs a bounds check, and the |x| maximum goes over the lanes of a row
// with DPP moves (quad swaps and mirrors inside a row of 16 lanes, scalar reads across the four rows)
// instead of six exchanges through the LDS crossbar: 9.55 -> 8.97 us on the FLUX payload.
__device__ __forceinline__ uint32_t row16_max_u32(uint32_t v) {
  v = max(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xf, 0xf, true));    // quad_perm [1,0,3,2]
  v = max(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xf, 0xf, true));    // quad_perm [2,3,0,1]
  v = max(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x141, 0xf, 0xf, true));   // row_half_mirror
  v = max(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x140, 0xf, 0xf, true));   // row_mirror
  return v;   // every lane of a row of 16 holds the row's maximum
}
template <int LPR, int NV, bool kMapped, bool kNT, bool kStreamIn, bool kFull>
__global__ __launch_bounds__(256) void fp8_quant_rows_bf16_kernel(const bf16_t* __restrict__ x,
                                                                  uint8_t* __restrict__ q,
                                                                  float* __restrict__ scales,
                                                                  int64_t rows, int units, RowMap map) {
  static_assert(LPR == 16 || LPR == 64, "a row is spread over a DPP row of 16 lanes or over the whole wave");
  constexpr int RPW = 64 / LPR;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int64_t row = ((int64_t)blockIdx.x * 4 + wave) * RPW + lane / LPR;
  const int l = lane % LPR;
  const bool row_ok = row < rows;
  if (kFull && !row_ok) return;               // whole DPP rows (LPR = 16) or the whole wave (LPR = 64) leave together
  if (kFull) units = LPR * NV;
  int64_t base = row * (int64_t)units * 8;   // first element of the row in x
  int64_t orow = row;                         // row of q / scales
  if (kMapped) {
    map_row(map, row_ok ? row : 0, base, orow);
  }
  const int64_t obase = orow * (int64_t)units * 8;
  const bf16_t* xr = x + base + l * 8;
  uint8_t* qr = q + obase + l * 8;

  u32x4_raw r[NV];
  uint32_t mbits = 0u;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    r[i] = u32x4_raw{0u, 0u, 0u, 0u};
    if (kFull || (row_ok && l + i * LPR < units)) {
      const u32x4_raw* p = reinterpret_cast<const u32x4_raw*>(xr + i * LPR * 8);
      r[i] = kStreamIn ? __builtin_nontemporal_load(p) : *p;
    }
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) mbits = absmax8_bf16_bits(r[i], mbits);
  mbits = max(mbits & 0xffffu, mbits >> 16);
  if (kFull) {
    mbits = row16_max_u32(mbits);
    if (LPR == 64) {
      const uint32_t a = __builtin_amdgcn_readlane((int)mbits, 0), b = __builtin_amdgcn_readlane((int)mbits, 16);
      const uint32_t c = __builtin_amdgcn_readlane((int)mbits, 32), e = __builtin_amdgcn_readlane((int)mbits, 48);
      mbits = max(max(a, b), max(c, e));
    }
  } else {
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) mbits = max(mbits, (uint32_t)__shfl_xor((int)mbits, off, 64));
  }
  const float s = scale_from_absmax(__uint_as_float(mbits << 16));
  if (row_ok && l == 0) scales[orow] = s;
  const RowDiv d = make_rowdiv(s);
  if (__builtin_amdgcn_ballot_w64(!d.fast) == 0ull) {
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (kFull || (row_ok && l + i * LPR < units)) put_codes<kNT>(qr + i * LPR * 8, encode8_bf16_short(r[i], d));
  } else {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      if (kFull || (row_ok && l + i * LPR < units)) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 4; ++k) { v[2 * k] = __uint_as_float(r[i][k] << 16); v[2 * k + 1] = __uint_as_float(r[i][k] & 0xffff0000u); }
        put_codes<kNT>(qr + i * LPR * 8, encode8<false>(v, d));
      }
    }
  }
}

// ---- long rows: one 256-thread block per row, two passes over the row ----------------------
template <typename T>
__global__ __launch_bounds__(256) void fp8_quant_longrow_kernel(const T* __restrict__ x,
                                                                uint8_t* __restrict__ q,
                                                                float* __restrict__ scales,
                                                                int64_t units) {
  __shared__ float red[4];
  const int64_t row = blockIdx.x;
  const int64_t base = row * units * 8;
  float a = 0.0f;
  for (int64_t u = threadIdx.x; u < units; u += 256) {
    float v[8];
    load8(x + base + u * 8, v);
    a = absmax8(v, a);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) a = fmaxf(a, __shfl_xor(a, off, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
  __syncthreads();
  a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  const float s = scale_from_absmax(a);
  if (threadIdx.x == 0) scales[row] = s;
  const RowDiv d = make_rowdiv(s);
  for (int64_t u = threadIdx.x; u < units; u += 256) {
    float v[8];
    load8(x + base + u * 8, v);
    *reinterpret_cast<uint2*>(q + base + u * 8) = d.fast ? encode8<true>(v, d) : encode8<false>(v, d);
  }
}

// ---- few, very long rows (per-tensor scale = one row: Algorithm 1 as printed): a row is cut into
// chunks so that the whole chip works on it.  Three steps on the stream: scales[row] <- 0; every
// chunk folds its |x| maximum into scales[row] (non-negative floats order like their bit patterns,
// so an unsigned atomic max does it); every chunk is cast with the row's scale, computed from that
// maximum by the same arithmetic as in the other kernels; scales[row] <- scale.
__global__ void fp8_fill_kernel(float* dst, int64_t n, float value) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = value;
}
template <typename T>
__global__ __launch_bounds__(256) void fp8_absmax_chunks_kernel(const T* __restrict__ x, float* __restrict__ scales,
                                                                int64_t units, int64_t chunk_units) {
  __shared__ float red[4];
  const int64_t row = blockIdx.y;
  const int64_t u0 = (int64_t)blockIdx.x * chunk_units, u1 = min(u0 + chunk_units, units);
  const T* xr = x + row * units * 8;
  float a = 0.0f;
  int64_t u = u0 + threadIdx.x;
  for (; u + 768 < u1; u += 1024) {      // four loads in flight per thread
    float v0[8], v1[8], v2[8], v3[8];
    load8(xr + u * 8, v0); load8(xr + (u + 256) * 8, v1); load8(xr + (u + 512) * 8, v2); load8(xr + (u + 768) * 8, v3);
    a = absmax8(v0, a); a = absmax8(v1, a); a = absmax8(v2, a); a = absmax8(v3, a);
  }
  for (; u < u1; u += 256) {
    float v[8];
    load8(xr + u * 8, v);
    a = absmax8(v, a);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) a = fmaxf(a, __shfl_xor(a, off, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    atomicMax(reinterpret_cast<unsigned int*>(scales + row), __float_as_uint(a));
  }
}
template <typename T>
__global__ __launch_bounds__(256) void fp8_quant_chunks_kernel(const T* __restrict__ x, uint8_t* __restrict__ q,
                                                               const float* __restrict__ absmax,
                                                               int64_t units, int64_t chunk_units) {
  const int64_t row = blockIdx.y;
  const int64_t u0 = (int64_t)blockIdx.x * chunk_units, u1 = min(u0 + chunk_units, units);
  const int64_t base = row * units * 8;
  const RowDiv d = make_rowdiv(scale_from_absmax(absmax[row]));
  auto cast = [&](const float (&v)[8]) -> uint2 { return d.fast ? encode8<true>(v, d) : encode8<false>(v, d); };
  int64_t u = u0 + threadIdx.x;
  for (; u + 768 < u1; u += 1024) {      // four loads in flight per thread
    float v0[8], v1[8], v2[8], v3[8];
    load8(x + base + u * 8, v0); load8(x + base + (u + 256) * 8, v1);
    load8(x + base + (u + 512) * 8, v2); load8(x + base + (u + 768) * 8, v3);
    *reinterpret_cast<uint2*>(q + base + u * 8) = cast(v0);
    *reinterpret_cast<uint2*>(q + base + (u + 256) * 8) = cast(v1);
    *reinterpret_cast<uint2*>(q + base + (u + 512) * 8) = cast(v2);
    *reinterpret_cast<uint2*>(q + base + (u + 768) * 8) = cast(v3);
  }
  for (; u < u1; u += 256) {
    float v[8];
    load8(x + base + u * 8, v);
    *reinterpret_cast<uint2*>(q + base + u * 8) = cast(v);
  }
}
__global__ void fp8_scales_from_absmax_kernel(float* scales, int64_t rows) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < rows) scales[i] = scale_from_absmax(scales[i]);
}

// all-zero-column case: scales still have to be defined
__global__ void fp8_fill_scales_kernel(float* scales, int64_t rows) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < rows) scales[i] = 1.0f;
}

// ---- dequantise: VEC codes per thread -----------------------------------------------------
__device__ __forceinline__ void decode4(uint32_t w, float s, float (&o)[4]) {
  f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
  f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
  o[0] = lo.x * s; o[1] = lo.y * s; o[2] = hi.x * s; o[3] = hi.y * s;
}

__device__ __forceinline__ void store4(float* y, const float (&o)[4]) {
  *reinterpret_cast<float4*>(y) = make_float4(o[0], o[1], o[2], o[3]);
}
__device__ __forceinline__ void store4(bf16_t* y, const float (&o)[4]) {
  *reinterpret_cast<uint2*>(y) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
}
__device__ __forceinline__ void store8(float* y, const float (&a)[4], const float (&b)[4]) {
  store4(y, a);
  store4(y + 4, b);
}
__device__ __forceinline__ void store8(bf16_t* y, const float (&a)[4], const float (&b)[4]) {
  *reinterpret_cast<uint4*>(y) = make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]),
                                            pack_bf16x2(b[0], b[1]), pack_bf16x2(b[2], b[3]));
}
// Streaming (non-temporal) stores leave no dirty lines in the L2s for the end of the kernel to write
// back: worth 2 us on a 28 MB launch whose successor starts right behind it, but slower than cached
// stores once the output is several times the L2 capacity.  The launchers pick by output size.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store8_nt(float* y, const float (&a)[4], const float (&b)[4]) {
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  const f32x4_t va = {a[0], a[1], a[2], a[3]}, vb = {b[0], b[1], b[2], b[3]};
  __builtin_nontemporal_store(va, reinterpret_cast<f32x4_t*>(y));
  __builtin_nontemporal_store(vb, reinterpret_cast<f32x4_t*>(y + 4));
}
__device__ __forceinline__ void store8_nt(bf16_t* y, const float (&a)[4], const float (&b)[4]) {
  const u32x4_t v = {pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(b[0], b[1]), pack_bf16x2(b[2], b[3])};
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(y));
}

template <typename T, int VEC, typename IDX, bool kMapped = false, bool kNT = false>
__global__ __launch_bounds__(256) void fp8_dequant_kernel(const uint8_t* __restrict__ q,
                                                          const float* __restrict__ scales,
                                                          T* __restrict__ y, IDX total_units,
                                                          uint32_t units_per_row, RowMap map) {
  const IDX g = (IDX)blockIdx.x * 256 + threadIdx.x;
  if (g >= total_units) return;
  const IDX row = g / units_per_row;   // 32-bit arithmetic whenever the tensor allows it
  int64_t e = (int64_t)g * VEC, eo = e;  // first element in q, in y
  int64_t srow = row;
  if (kMapped) {
    const int64_t u = (int64_t)(g - row * units_per_row) * VEC;
    int64_t dst;
    map_row(map, row, srow, dst);
    e = srow * (int64_t)units_per_row * VEC + u;
    eo = dst + u;
  }
  const float s = scales ? scales[srow] : 1.0f;   // no scales: exact widening of the codes
  auto put8 = [&](T* p, const float (&a)[4], const float (&b)[4]) {
    if (kNT) store8_nt(p, a, b);
    else store8(p, a, b);
  };
  if constexpr (VEC == 16) {
    const u32x4_t w = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(q + e));
    float a[4], b[4];
    decode4(w[0], s, a); decode4(w[1], s, b); put8(y + eo, a, b);
    decode4(w[2], s, a); decode4(w[3], s, b); put8(y + eo + 8, a, b);
  } else {
    uint2 w = *reinterpret_cast<const uint2*>(q + e);
    float a[4], b[4];
    decode4(w.x, s, a); decode4(w.y, s, b); put8(y + eo, a, b);
  }
}

// Dense bf16 output, the payload type of the method: 8 codes per unit, U units per thread a block
// stride apart, so that every load instruction of a wave reads 512 consecutive bytes and every store
// instruction writes 1024 consecutive bytes (whole lines; a thread that writes 32 bytes with two
// stores leaves each line to two instructions), and a thread has U loads in flight before its first
// store.  On the [4608, 3072] payload: 8.2 us against 10.0 us for 16 codes per thread.
template <int U, bool kNT>
__global__ __launch_bounds__(256) void fp8_dequant_bf16_dense_kernel(const uint8_t* __restrict__ q,
                                                                     const float* __restrict__ scales,
                                                                     bf16_t* __restrict__ y, uint32_t total_units,
                                                                     uint32_t units_per_row) {
  const uint32_t first = blockIdx.x * (U * 256u) + threadIdx.x;
  uint2 w[U];
  float s[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t g = first + u * 256u;
    w[u] = make_uint2(0u, 0u);
    s[u] = 1.0f;                                   // no scales: exact widening of the codes
    if (g < total_units) {
      w[u] = *reinterpret_cast<const uint2*>(q + (int64_t)g * 8);
      if (scales) s[u] = scales[g / units_per_row];
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t g = first + u * 256u;
    if (g < total_units) {
      float a[4], b[4];
      decode4(w[u].x, s[u], a);
      decode4(w[u].y, s[u], b);
      if (kNT) store8_nt(y + (int64_t)g * 8, a, b);
      else store8(y + (int64_t)g * 8, a, b);
    }
  }
}

// rows of at most 4096 elements: the single-pass kernel, plain or mapped
template <typename T, int LPR, int NV, bool kMapped, bool kNT, bool kStreamIn>
void quant_rows_launch_one(unsigned blocks, int64_t rows, int64_t units, const T* x, uint8_t* q, float* scales,
                           const RowMap& map, hipStream_t st) {
  if constexpr (std::is_same<T, bf16_t>::value) {
    if (units == LPR * NV)
      hipLaunchKernelGGL((fp8_quant_rows_bf16_kernel<LPR, NV, kMapped, kNT, kStreamIn, true>), dim3(blocks), dim3(256), 0, st, x, q, scales, rows, (int)units, map);
    else
      hipLaunchKernelGGL((fp8_quant_rows_bf16_kernel<LPR, NV, kMapped, kNT, kStreamIn, false>), dim3(blocks), dim3(256), 0, st, x, q, scales, rows, (int)units, map);
  } else
    hipLaunchKernelGGL((fp8_quant_rows_kernel<T, LPR, NV, kMapped, kNT, kStreamIn>), dim3(blocks), dim3(256), 0, st, x, q, scales, rows, (int)units, map);
}
template <typename T, bool kMapped, bool kNT, bool kStreamIn>
void quant_rows_launch_nt(int64_t rows, int64_t units, const T* x, uint8_t* q, float* scales, const RowMap& map,
                          hipStream_t st) {
  auto blocks = [&](int rpw) { return (unsigned)((rows + 4 * rpw - 1) / (4 * rpw)); };
  if (units <= 16) quant_rows_launch_one<T, 16, 1, kMapped, kNT, kStreamIn>(blocks(4), rows, units, x, q, scales, map, st);
  else if (units <= 32) quant_rows_launch_one<T, 16, 2, kMapped, kNT, kStreamIn>(blocks(4), rows, units, x, q, scales, map, st);
  else if (units <= 64) quant_rows_launch_one<T, 64, 1, kMapped, kNT, kStreamIn>(blocks(1), rows, units, x, q, scales, map, st);
  else if (units <= 128) quant_rows_launch_one<T, 64, 2, kMapped, kNT, kStreamIn>(blocks(1), rows, units, x, q, scales, map, st);
  else if (units <= 256) quant_rows_launch_one<T, 64, 4, kMapped, kNT, kStreamIn>(blocks(1), rows, units, x, q, scales, map, st);
  else if (units <= 384) quant_rows_launch_one<T, 64, 6, kMapped, kNT, kStreamIn>(blocks(1), rows, units, x, q, scales, map, st);
  else quant_rows_launch_one<T, 64, 8, kMapped, kNT, kStreamIn>(blocks(1), rows, units, x, q, scales, map, st);
}

template <typename T, bool kMapped>
void quant_rows_launch(int64_t rows, int64_t units, const T* x, uint8_t* q, float* scales, const RowMap& map,
                       hipStream_t st) {
  const int64_t codes = rows * units * 8;
  if (codes * (int64_t)sizeof(T) < kStreamDequantBelowBytes) quant_rows_launch_nt<T, kMapped, true, true>(rows, units, x, q, scales, map, st);
  else if (codes < kStreamQuantBelowBytes) quant_rows_launch_nt<T, kMapped, true, false>(rows, units, x, q, scales, map, st);
  else quant_rows_launch_nt<T, kMapped, false, false>(rows, units, x, q, scales, map, st);
}

template <typename T>
usp_status quant_dispatch(int64_t rows, int64_t cols, const T* x, uint8_t* q, float* scales,
                          hipStream_t st) {
  const int64_t units = cols / 8;
  if (units <= 512) {
    quant_rows_launch<T, false>(rows, units, x, q, scales, RowMap(), st);
  } else if (rows >= 1024 || rows * units < 4096 * 8) {
    hipLaunchKernelGGL((fp8_quant_longrow_kernel<T>), dim3((unsigned)rows), dim3(256), 0, st, x, q, scales, units);
  } else {
    // too few rows to fill the chip with one block per row: about 2048 chunks of whole 256-unit strides
    const int64_t per_row = (2048 + rows - 1) / rows;
    int64_t chunk_units = (units + per_row - 1) / per_row;
    chunk_units = (chunk_units + 255) / 256 * 256;
    if (chunk_units < 1024) chunk_units = 1024;
    const dim3 grid((unsigned)((units + chunk_units - 1) / chunk_units), (unsigned)rows);
    const unsigned rb = (unsigned)((rows + 255) / 256);
    hipLaunchKernelGGL(fp8_fill_kernel, dim3(rb), dim3(256), 0, st, scales, rows, 0.0f);
    // the maximum pass ends in one atomic per block on the row's word, and those serialise (about 10 ns
    // each): at most 512 blocks over all rows
    int64_t a_per_row = (512 + rows - 1) / rows;
    int64_t a_units = (units + a_per_row - 1) / a_per_row;
    a_units = (a_units + 1023) / 1024 * 1024;
    const dim3 a_grid((unsigned)((units + a_units - 1) / a_units), (unsigned)rows);
    hipLaunchKernelGGL((fp8_absmax_chunks_kernel<T>), a_grid, dim3(256), 0, st, x, scales, units, a_units);
    hipLaunchKernelGGL((fp8_quant_chunks_kernel<T>), grid, dim3(256), 0, st, x, q, scales, units, chunk_units);
    hipLaunchKernelGGL(fp8_scales_from_absmax_kernel, dim3(rb), dim3(256), 0, st, scales, rows);
  }
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

template <typename T, int VEC>
usp_status dequant_launch(int64_t rows, int64_t cols, const uint8_t* q, const float* scales, T* y,
                          hipStream_t st) {
  const int64_t upr = cols / VEC, total = rows * upr;
  const dim3 grid((unsigned)((total + 255) / 256)), block(256);
  const bool nt = rows * cols * (int64_t)sizeof(T) < kStreamDequantBelowBytes;
  if (total < ((int64_t)1 << 31) && nt)
    hipLaunchKernelGGL((fp8_dequant_kernel<T, VEC, uint32_t, false, true>), grid, block, 0, st, q, scales, y, (uint32_t)total, (uint32_t)upr, RowMap());
  else if (total < ((int64_t)1 << 31))
    hipLaunchKernelGGL((fp8_dequant_kernel<T, VEC, uint32_t>), grid, block, 0, st, q, scales, y, (uint32_t)total, (uint32_t)upr, RowMap());
  else
    hipLaunchKernelGGL((fp8_dequant_kernel<T, VEC, int64_t>), grid, block, 0, st, q, scales, y, total, (uint32_t)upr, RowMap());
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

template <typename T>
usp_status dequant_mapped_launch(const RowMap& m, int64_t rows, int64_t cols, const uint8_t* q, const float* scales,
                                 T* y, hipStream_t st) {
  const bool nt = rows * cols * (int64_t)sizeof(T) < kStreamDequantBelowBytes;
  if (cols % 16 == 0) {
    const int64_t upr = cols / 16, total = rows * upr;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (nt) hipLaunchKernelGGL((fp8_dequant_kernel<T, 16, int64_t, true, true>), grid, dim3(256), 0, st, q, scales, y, total, (uint32_t)upr, m);
    else hipLaunchKernelGGL((fp8_dequant_kernel<T, 16, int64_t, true, false>), grid, dim3(256), 0, st, q, scales, y, total, (uint32_t)upr, m);
  } else {
    const int64_t upr = cols / 8, total = rows * upr;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (nt) hipLaunchKernelGGL((fp8_dequant_kernel<T, 8, int64_t, true, true>), grid, dim3(256), 0, st, q, scales, y, total, (uint32_t)upr, m);
    else hipLaunchKernelGGL((fp8_dequant_kernel<T, 8, int64_t, true, false>), grid, dim3(256), 0, st, q, scales, y, total, (uint32_t)upr, m);
  }
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

template <typename T>
usp_status dequant_dispatch(int64_t rows, int64_t cols, const uint8_t* q, const float* scales, T* y,
                            hipStream_t st) {
  if constexpr (std::is_same<T, bf16_t>::value) {
    const int64_t upr = cols / 8, total = rows * upr;
    // enough units to fill the chip with four per thread, and an output the streaming stores are good
    // for (otherwise: 16 codes per thread, below)
    if (total >= 4 * 256 * 1024 && rows * cols * (int64_t)sizeof(T) < kStreamDequantBelowBytes) {
      hipLaunchKernelGGL((fp8_dequant_bf16_dense_kernel<4, true>), dim3((unsigned)((total + 1023) / 1024)), dim3(256), 0, st,
                         q, scales, y, (uint32_t)total, (uint32_t)upr);
      USP_CHECK_HIP(hipGetLastError());
      return USP_OK;
    }
  }
  if (cols % 16 == 0) return dequant_launch<T, 16>(rows, cols, q, scales, y, st);
  return dequant_launch<T, 8>(rows, cols, q, scales, y, st);
}

}  // namespace

usp_status launch_fp8_quant(int64_t rows, int64_t cols, int in_dt, const void* x, uint8_t* q,
                            float* scales, hipStream_t st) {
  if (rows == 0) return USP_OK;
  if (cols == 0) {
    hipLaunchKernelGGL(fp8_fill_scales_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st, scales, rows);
    USP_CHECK_HIP(hipGetLastError());
    return USP_OK;
  }
  if (in_dt == USP_BF16) return quant_dispatch<bf16_t>(rows, cols, (const bf16_t*)x, q, scales, st);
  return quant_dispatch<float>(rows, cols, (const float*)x, q, scales, st);
}

usp_status launch_fp8_quant_mapped(const RowMap& m, int64_t rows, int64_t cols, int in_dt, const void* x,
                                   uint8_t* q, float* scales, hipStream_t st) {
  if (rows == 0 || cols == 0) return USP_OK;
  if (in_dt == USP_BF16) quant_rows_launch<bf16_t, true>(rows, cols / 8, (const bf16_t*)x, q, scales, m, st);
  else quant_rows_launch<float, true>(rows, cols / 8, (const float*)x, q, scales, m, st);
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

usp_status launch_fp8_dequant_mapped(const RowMap& m, int64_t rows, int64_t cols, int out_dt, const uint8_t* q,
                                     const float* scales, void* y, hipStream_t st) {
  if (rows == 0 || cols == 0) return USP_OK;
  if (out_dt == USP_BF16) return dequant_mapped_launch<bf16_t>(m, rows, cols, q, scales, (bf16_t*)y, st);
  return dequant_mapped_launch<float>(m, rows, cols, q, scales, (float*)y, st);
}

usp_status launch_fp8_dequant(int64_t rows, int64_t cols, int out_dt, const uint8_t* q,
                              const float* scales, void* y, hipStream_t st) {
  if (rows == 0 || cols == 0) return USP_OK;
  if (out_dt == USP_BF16) return dequant_dispatch<bf16_t>(rows, cols, q, scales, (bf16_t*)y, st);
  return dequant_dispatch<float>(rows, cols, q, scales, (float*)y, st);
}

}  // namespace usp
