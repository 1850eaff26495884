// libusp_diag.so: diagnostics that are not part of the library's ABI (usp_diag.h).  Built beside
// libusp.so and linked against it; only the benchmark and the tests load it.
//   * usp_diag_mfma_rate: the dense bf16 MFMA rate the chip sustains when nothing else is issued.  Not
//     a step of the method; it gives the measured ceiling that the attention kernel's rate is read
//     against (the clock the chip holds under a full matrix-core load depends on the operand data).
//   * usp_diag_check_bf16_division: the short division sequence of the bf16 pack against the IEEE division,
//     over every (row absmax, element) pair of bf16 values.
//   * usp_diag_payload_floor: an empty launch, a read-only and a write-only pass over a pack payload, which
//     show what bounds a single pack / unpack launch.
//   * usp_diag_ring_attn_fwd_wait: usp_ring_attn_fwd with the knobs of the bounded arrival wait of the
//     one-launch ring, so that a test can drive its give-up path from the host.
#include "usp_common.h"
#include "fp8_arith.h"
#include "usp_diag.h"

namespace usp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeThreads = 512;       // 8 waves, two per SIMD, as in the attention kernels
constexpr int kProbeMfmaPerIter = 32;

// Every wave runs iters * 32 * 32768 flop of MFMAs on four A and four B operands held in registers
// (32x32x16: 32 instructions per iteration on four accumulators; 16x16x32: 64 on eight); consecutive
// instructions take different operands.  Work-group 0 records the shader cycles and the 100 MHz ticks
// of its loop.
typedef float f32x4 __attribute__((ext_vector_type(4)));
template <int kShape>
__global__ __launch_bounds__(kProbeThreads) void mfma_rate_kernel(int iters, int random_data, float* out,
                                                                 unsigned long long* clocks) {
  bf16x8 a[4], b[4];
  unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  for (int u = 0; u < 4; ++u)
    for (int i = 0; i < 8; ++i) {   // uniform in [-1, 1], or constants
      h = h * 1664525u + 1013904223u;
      a[u][i] = (__bf16)(random_data ? ((int)(h >> 16) % 2001 - 1000) * 0.001f : 1.0f);
      h = h * 1664525u + 1013904223u;
      b[u][i] = (__bf16)(random_data ? ((int)(h >> 16) % 2001 - 1000) * 0.001f : 0.5f);
    }
  float sum = 0.0f;
  const unsigned long long t0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  if (kShape == 0) {
    f32x16 c[4];
    for (int j = 0; j < 4; ++j)
      for (int i = 0; i < 16; ++i) c[j][i] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int u = 0; u < kProbeMfmaPerIter / 4; ++u)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + j) & 3], b[j], c[j], 0, 0, 0);
    }
    for (int j = 0; j < 4; ++j)
      for (int i = 0; i < 16; ++i) sum += c[j][i];
  } else {
    f32x4 c[8];
    for (int j = 0; j < 8; ++j)
      for (int i = 0; i < 4; ++i) c[j][i] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int u = 0; u < kProbeMfmaPerIter / 4; ++u)
#pragma unroll
        for (int j = 0; j < 8; ++j)
          c[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[(u + j) & 3], b[j & 3], c[j], 0, 0, 0);
    }
    for (int j = 0; j < 8; ++j)
      for (int i = 0; i < 4; ++i) sum += c[j][i];
  }
  const unsigned long long t1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  out[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = sum;   // keeps the work alive
  if (blockIdx.x == 0 && threadIdx.x == 0) { clocks[0] = t1 - t0; clocks[1] = r1 - r0; }
}


// One block per positive finite bf16 a (the row's |x| maximum): s = a / 448 as the pack computes it;
// for every bf16 x with |x| <= a, both signs, the E4M3 code of the short sequence against the code of
// the IEEE quotient x / s.  counts: [0] pairs checked, [1] codes that differ, [2] quotients that differ
// in some bit (allowed), [3] values of a whose scale is outside the fast range (they take the division).
__device__ __forceinline__ uint32_t code_of(float t) { return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(t, t, 0, false) & 0xffu; }
__global__ __launch_bounds__(256) void check_bf16_division_kernel(unsigned long long* counts) {
  const uint32_t abits = blockIdx.x + 1;            // 0x0001 .. 0x7f7f
  const float a = __uint_as_float(abits << 16);
  const float s = scale_from_absmax(a);
  const RowDiv d = make_rowdiv(s);
  if (!d.fast) {
    if (threadIdx.x == 0) atomicAdd(&counts[3], 1ull);
    return;
  }
  unsigned long long n = 0, bad_code = 0, bad_quot = 0;
  for (uint32_t xb = threadIdx.x; xb <= abits; xb += 256) {
    // encode8_bf16_short takes packed pairs: +x in the low half, -x in the high half of every word
    const uint32_t pair = xb | ((xb | 0x8000u) << 16);
    const uint2 c = encode8_bf16_short(u32x4_raw{pair, pair, pair, pair}, d);
    for (int sg = 0; sg < 2; ++sg) {
      const float x = __uint_as_float((xb | (sg ? 0x8000u : 0u)) << 16);
      const float qt = x / s;                         // IEEE division
      const uint32_t want = code_of(qt);
      const float q0 = x * d.rcp;
      const float q1 = fmaf(fmaf(-d.s, q0, x), d.rcp, q0);
      ++n;
      if (((c.x >> (8 * sg)) & 0xffu) != want || ((c.y >> (8 * sg + 16)) & 0xffu) != want) ++bad_code;
      if (__float_as_uint(q1) != __float_as_uint(qt)) ++bad_quot;
    }
  }
  atomicAdd(&counts[0], n); atomicAdd(&counts[1], bad_code); atomicAdd(&counts[2], bad_quot);
}

// What a pack launch over a [rows, 3072] bf16 payload costs before any arithmetic: the same grid
// (one wave per row, 4 rows per block) doing nothing, only reading the rows (their |x| maximum goes to
// scales), or only writing codes.
typedef uint32_t u32x2_raw __attribute__((ext_vector_type(2)));
__global__ __launch_bounds__(256) void floor_kernel(int kind, const bf16_t* __restrict__ x, uint8_t* __restrict__ q,
                                                    float* __restrict__ scales, int rows) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * 4 + wave;
  if (kind == 0 || row >= rows) return;
  if (kind == 1) {
    uint32_t m = 0u;
#pragma unroll
    for (int i = 0; i < 6; ++i)
      m = absmax8_bf16_bits(__builtin_nontemporal_load(reinterpret_cast<const u32x4_raw*>(x + (int64_t)row * 3072 + (lane + 64 * i) * 8)), m);
    m = max(m & 0xffffu, m >> 16);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off, 64));
    if (lane == 0) scales[row] = __uint_as_float(m << 16);
  } else {
#pragma unroll
    for (int i = 0; i < 6; ++i) {
      const u32x2_raw w = {(uint32_t)row, (uint32_t)lane};
      __builtin_nontemporal_store(w, reinterpret_cast<u32x2_raw*>(q + (int64_t)row * 3072 + (lane + 64 * i) * 8));
    }
  }
}

}  // namespace

}  // namespace usp

using namespace usp;

extern "C" {

usp_status usp_diag_mfma_rate(int32_t wgs, int32_t iters, int32_t random_data, int32_t shape, float* out,
                              uint64_t* clocks, void* stream) {
  clear_error();
  USP_CHECK_ARG(wgs >= 1 && wgs <= 65536, "wgs=%d out of range [1, 65536]", wgs);
  USP_CHECK_ARG(iters >= 1 && iters <= 1000000, "iters=%d out of range [1, 1000000]", iters);
  USP_CHECK_ARG(out != nullptr && clocks != nullptr, "out or clocks is NULL");
  USP_CHECK_ARG(shape == 0 || shape == 1, "shape=%d must be 0 (32x32x16) or 1 (16x16x32)", shape);
  if (shape == 0)
    hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3((unsigned)wgs), dim3(kProbeThreads), 0, (hipStream_t)stream, iters,
                       random_data, out, reinterpret_cast<unsigned long long*>(clocks));
  else
    hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3((unsigned)wgs), dim3(kProbeThreads), 0, (hipStream_t)stream, iters,
                       random_data, out, reinterpret_cast<unsigned long long*>(clocks));
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

usp_status usp_diag_check_bf16_division(uint64_t* counts, void* stream) {
  clear_error();
  USP_CHECK_ARG(counts != nullptr, "counts is NULL");
  hipLaunchKernelGGL(check_bf16_division_kernel, dim3(0x7f7f), dim3(256), 0, (hipStream_t)stream,
                     reinterpret_cast<unsigned long long*>(counts));
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

usp_status usp_diag_payload_floor(int32_t kind, int32_t rows, const void* x, uint8_t* q, float* scales, void* stream) {
  clear_error();
  USP_CHECK_ARG(kind >= 0 && kind <= 2, "kind=%d must be 0 (empty), 1 (read only) or 2 (write only)", kind);
  USP_CHECK_ARG(rows >= 1 && rows <= (1 << 24), "rows=%d out of range", rows);
  USP_CHECK_ARG(kind == 0 || (x != nullptr && q != nullptr && scales != nullptr), "x, q or scales is NULL");
  USP_CHECK_ARG(aligned16(x) && aligned16(q), "x and q must be 16-byte aligned");
  hipLaunchKernelGGL(floor_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, (hipStream_t)stream, kind,
                     (const bf16_t*)x, q, scales, rows);
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

usp_status usp_diag_repeat_payload_calls(int32_t kind, int32_t reps, int32_t n_sets, int64_t rows, int64_t cols,
                                         const void* const* x, uint8_t* const* q, float* const* scales,
                                         void* const* y, void* stream) {
  clear_error();
  USP_CHECK_ARG(kind >= 0 && kind <= 4, "kind=%d out of range [0, 4]", kind);
  USP_CHECK_ARG(reps >= 1 && reps <= (1 << 20) && n_sets >= 1, "reps or n_sets out of range");
  USP_CHECK_ARG(x && q && scales && y, "a buffer array is NULL");
  for (int i = 0; i < reps; ++i) {
    const int j = i % n_sets;
    usp_status st;
    if (kind == 0) st = usp_fp8_quant(rows, cols, USP_BF16, x[j], q[j], scales[j], stream);
    else if (kind == 1) st = usp_fp8_dequant(rows, cols, USP_BF16, q[j], scales[j], y[j], stream);
    else {
      USP_CHECK_ARG(cols == 3072 && rows <= (1 << 24), "the floor kernels take [rows, 3072] payloads");
      st = usp_diag_payload_floor(kind - 2, (int32_t)rows, x[j], q[j], scales[j], stream);
    }
    if (st != USP_OK) return st;
  }
  return USP_OK;
}

usp_status usp_diag_repeat_merge_calls(int32_t reps, int32_t n_sets, int64_t rows, int32_t d, const void* const* o1,
                                       const float* const* lse1, const void* const* o2, const float* const* lse2,
                                       void* const* o_out, float* const* lse_out, void* stream) {
  clear_error();
  USP_CHECK_ARG(reps >= 1 && reps <= (1 << 20) && n_sets >= 1, "reps or n_sets out of range");
  USP_CHECK_ARG(o1 && lse1 && o2 && lse2 && o_out && lse_out, "a buffer array is NULL");
  for (int i = 0; i < reps; ++i) {
    const int j = i % n_sets;
    const usp_status st = usp_lse_merge(rows, d, USP_BF16, o1[j], lse1[j], o2[j], lse2[j], o_out[j], lse_out[j], stream);
    if (st != USP_OK) return st;
  }
  return USP_OK;
}

usp_status usp_diag_ring_attn_fwd_wait(const usp_attn_desc* desc, const void* q, const void* const* k_chunks,
                                       const void* const* v_chunks, const float* const* k_scales,
                                       const float* const* v_scales, const uint8_t* const* key_mask, void* out,
                                       float* lse, void* workspace, size_t workspace_bytes, void* compute_stream,
                                       int32_t arrive_need_extra, int32_t arrive_polls) {
  clear_error();
  USP_CHECK_ARG(arrive_need_extra >= 0 && arrive_need_extra <= 1024, "arrive_need_extra=%d out of range [0, 1024]", arrive_need_extra);
  USP_CHECK_ARG(arrive_polls >= 0, "arrive_polls=%d is negative", arrive_polls);
  CallOptions opt;
  opt.arrive_need_extra = arrive_need_extra;
  opt.arrive_polls = arrive_polls;
  return ring_attn_fwd_impl(desc, q, k_chunks, v_chunks, k_scales, v_scales, key_mask, out, lse, workspace,
                            workspace_bytes, compute_stream, nullptr, opt);
}

}  // extern "C"
