// Head-dimension padding for the bf16 d = 64 case: the matrix-core attention kernels are written
// for d = 128, and softmax(Q K^T) V is unchanged when Q and K get 64 extra zero columns (the scores
// of section 2.2 gain only zero terms) and V gets 64 extra zero columns (they come out as zero columns
// of O, which are dropped).  pad: strided [B,H,S,64] bf16 (or E4M3 codes, whose zero code is 0.0) ->
// dense [B,H,S,128]; unpad: the reverse for a bf16 O.  One thread moves 16 bytes; both kernels are bandwidth-bound and tiny next to the attention.
#include <hip/hip_runtime.h>
#include "usp_common.h"

namespace usp {
namespace {

// kUnits: 16-byte units of a source row (8 for bf16, 4 for one-byte codes); the padded row has twice as many
// blockIdx.y picks the tensor: K (0) or V (1) of a chunk, padded by one launch
template <int kUnits>
__global__ __launch_bounds__(256) void pad64_kernel(const unsigned char* __restrict__ src0, unsigned char* __restrict__ dst0,
                                                    const unsigned char* __restrict__ src1, unsigned char* __restrict__ dst1,
                                                    int H, int S, int64_t s0, int64_t s1, int64_t s2, int64_t rows) {
  const unsigned char* src = blockIdx.y ? src1 : src0;
  unsigned char* dst = blockIdx.y ? dst1 : dst0;
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = g / (2 * kUnits);
  if (row >= rows) return;
  const int part = (int)(g - row * (2 * kUnits));
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (part < kUnits) {
    const int64_t t = row % S, bh = row / S, h = bh % H, b = bh / H;
    v = *reinterpret_cast<const uint4*>(src + (b * s0 + h * s1 + t * s2) * (kUnits * 16 / 64) + part * 16);
  }
  *reinterpret_cast<uint4*>(dst + (row * 2 * kUnits + part) * 16) = v;
}

__global__ __launch_bounds__(256) void unpad64_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int H, int S,
                                                      int64_t s0, int64_t s1, int64_t s2, int64_t rows) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;   // 8 units of 16 bytes per output row
  const int64_t row = g >> 3;
  if (row >= rows) return;
  const int part = (int)(g & 7);
  const int64_t t = row % S, bh = row / S, h = bh % H, b = bh / H;
  *reinterpret_cast<uint4*>(dst + b * s0 + h * s1 + t * s2 + part * 8) =
      *reinterpret_cast<const uint4*>(src + row * 128 + part * 8);
}

}  // namespace

usp_status launch_pad64(const void* k_src, void* k_dst, const void* v_src, void* v_dst, int B, int H, int S,
                        const int64_t stride[3], int elt_bytes, hipStream_t st) {
  const int64_t rows = (int64_t)B * H * S;
  if (rows == 0) return USP_OK;
  if (elt_bytes == 2)
    hipLaunchKernelGGL(pad64_kernel<8>, dim3((unsigned)((rows * 16 + 255) / 256), 2), dim3(256), 0, st, (const unsigned char*)k_src,
                       (unsigned char*)k_dst, (const unsigned char*)v_src, (unsigned char*)v_dst, H, S, stride[0], stride[1], stride[2], rows);
  else
    hipLaunchKernelGGL(pad64_kernel<4>, dim3((unsigned)((rows * 8 + 255) / 256), 2), dim3(256), 0, st, (const unsigned char*)k_src,
                       (unsigned char*)k_dst, (const unsigned char*)v_src, (unsigned char*)v_dst, H, S, stride[0], stride[1], stride[2], rows);
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

usp_status launch_unpad64(const void* src, void* dst, int B, int H, int S, const int64_t stride[3], hipStream_t st) {
  const int64_t rows = (int64_t)B * H * S;
  if (rows == 0) return USP_OK;
  hipLaunchKernelGGL(unpad64_kernel, dim3((unsigned)((rows * 8 + 255) / 256)), dim3(256), 0, st, (const bf16_t*)src,
                     (bf16_t*)dst, H, S, stride[0], stride[1], stride[2], rows);
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

}  // namespace usp
