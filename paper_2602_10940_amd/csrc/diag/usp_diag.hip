// libusp_diag.so: diagnostics that are not part of the library's ABI (usp_diag.h).  Built beside
// libusp.so and linked against it; only the benchmark and the tests load it.
//   * usp_diag_mfma_rate: the dense bf16 MFMA rate the chip sustains when nothing else is issued.  Not
//     a step of the method; it gives the measured ceiling that the attention kernel's rate is read
//     against (the clock the chip holds under a full matrix-core load depends on the operand data).
//   * usp_diag_ring_attn_fwd_wait: usp_ring_attn_fwd with the knobs of the bounded arrival wait of the
//     one-launch ring, so that a test can drive its give-up path from the host.
#include "usp_common.h"
#include "usp_diag.h"

namespace usp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeThreads = 512;       // 8 waves, two per SIMD, as in the attention kernels
constexpr int kProbeMfmaPerIter = 32;

// Every wave runs iters * 32 MFMAs (32x32x16, fp32 accumulate) on four A and four B operands held
// in registers; consecutive instructions take different operands, and four accumulators are in
// flight per wave.  Work-group 0 records the shader cycles and the 100 MHz ticks of its loop.
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
  f32x16 c[4];
  for (int j = 0; j < 4; ++j)
    for (int i = 0; i < 16; ++i) c[j][i] = 0.0f;
  const unsigned long long t0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < kProbeMfmaPerIter / 4; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + j) & 3], b[j], c[j], 0, 0, 0);
  }
  const unsigned long long t1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  float sum = 0.0f;
  for (int j = 0; j < 4; ++j)
    for (int i = 0; i < 16; ++i) sum += c[j][i];
  out[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = sum;   // keeps the work alive
  if (blockIdx.x == 0 && threadIdx.x == 0) { clocks[0] = t1 - t0; clocks[1] = r1 - r0; }
}

}  // namespace

}  // namespace usp

using namespace usp;

extern "C" {

usp_status usp_diag_mfma_rate(int32_t wgs, int32_t iters, int32_t random_data, float* out, uint64_t* clocks,
                              void* stream) {
  clear_error();
  USP_CHECK_ARG(wgs >= 1 && wgs <= 65536, "wgs=%d out of range [1, 65536]", wgs);
  USP_CHECK_ARG(iters >= 1 && iters <= 1000000, "iters=%d out of range [1, 1000000]", iters);
  USP_CHECK_ARG(out != nullptr && clocks != nullptr, "out or clocks is NULL");
  hipLaunchKernelGGL(mfma_rate_kernel, dim3((unsigned)wgs), dim3(kProbeThreads), 0, (hipStream_t)stream, iters,
                     random_data, out, reinterpret_cast<unsigned long long*>(clocks));
  USP_CHECK_HIP(hipGetLastError());
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
