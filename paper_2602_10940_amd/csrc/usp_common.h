// Internal helpers shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>
#include "usp.h"

namespace usp {

// thread-local message behind usp_last_error()
void set_error(const char* fmt, ...);
void clear_error();

#define USP_CHECK_ARG(cond, ...)                       \
  do {                                                 \
    if (!(cond)) {                                     \
      ::usp::set_error(__VA_ARGS__);                   \
      return USP_ERR_INVALID_ARG;                      \
    }                                                  \
  } while (0)

#define USP_CHECK_HIP(expr)                                                    \
  do {                                                                         \
    hipError_t e_ = (expr);                                                    \
    if (e_ != hipSuccess) {                                                    \
      ::usp::set_error("%s failed: %s", #expr, hipGetErrorString(e_));         \
      return USP_ERR_HIP;                                                      \
    }                                                                          \
  } while (0)

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- device-side scalar type helpers ---------------------------------------------------
typedef uint16_t bf16_t;  // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round to nearest even (finite inputs; NaN stays NaN via the quiet bit)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// two fp32 -> packed bf16x2 (low half = a), hardware RNE convert
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __bf16 bf16x2_v __attribute__((ext_vector_type(2)));
  typedef float f32x2_v __attribute__((ext_vector_type(2)));
  f32x2_v f = {a, b};
  bf16x2_v r = __builtin_convertvector(f, bf16x2_v);
  return *reinterpret_cast<uint32_t*>(&r);
}

// ---- kernel launchers implemented in the .hip files ------------------------------------
// Row visiting order of the mapped FP8 kernels: row id -> (i0..i3), i3 fastest -> two offsets.
struct RowMap {
  uint32_t n1, n2, n3;       // extents of i1..i3 (i0 is what is left)
  int64_t src[4], dst[4];
};
usp_status launch_fp8_quant_mapped(const RowMap& m, int64_t rows, int64_t cols, int in_dt, const void* x,
                                   uint8_t* q, float* scales, hipStream_t st);
usp_status launch_fp8_dequant_mapped(const RowMap& m, int64_t rows, int64_t cols, int out_dt, const uint8_t* q,
                                     const float* scales, void* y, hipStream_t st);
usp_status launch_fp8_quant(int64_t rows, int64_t cols, int in_dt, const void* x, uint8_t* q,
                            float* scales, hipStream_t st);
usp_status launch_fp8_dequant(int64_t rows, int64_t cols, int out_dt, const uint8_t* q,
                              const float* scales, void* y, hipStream_t st);
usp_status launch_lse_merge(int64_t rows, int d, int dt, const void* o1, const float* lse1,
                            const void* o2, const float* lse2, void* o_out, float* lse_out,
                            hipStream_t st);

// One attention step over one KV chunk.
struct AttnStep {
  int B, H, d, Sq, Sc;
  int qo_dtype;              // USP_F32 / USP_BF16
  int kv_dtype;              // USP_F32 / USP_BF16 / USP_FP8_E4M3FN
  const void* q;
  const void* k;
  const void* v;
  const float* k_scale;      // FP8 only: [B,H,Sc]
  const float* v_scale;
  const uint8_t* key_mask;   // [B,Sc] or null
  int64_t qs[3], ks[3], os[3];
  float scale;
  // merge-in-epilogue: mode 0 = write (O_r, lse_r) to out/lse in qo_dtype (single chunk or unfused)
  //                    mode 1 = first of several chunks: write fp32 O to acc, lse to lse
  //                    mode 2 = middle chunk: merge with (acc, lse), write back fp32
  //                    mode 3 = last chunk: merge with (acc, lse), write out in qo_dtype and lse
  int mode;
  int variant;               // matrix-core kernels: 0 = pick by grid size, 1 = 256-query work-groups, 2 = key-split, 4 = mixed
  int mix_halves;            // mixed launch: blocks per XCD run as two key-split halves (set by the launcher)
  int half_d;                // matrix-core kernels: d = 64: the rows of Q, K, V, `out` and acc are 64 wide (128 bytes), the kernels
                             // run their head-dimension loops over half the slices
  float* acc;                // fp32 [B,H,Sq,d] dense carried O (modes 1-3)
  void* out;                 // qo_dtype by os strides (modes 0, 3)
  float* lse;                // fp32 [B,H,Sq] dense
  // Matrix-core kernels, chunks with a key mask, FP8 scales or a length that is not a multiple of 64:
  // per-(batch, head, 64-key tile) records (attn_mfma_ext_bytes) and per-batch live tile counts [B],
  // filled by launch_attn_ext_prepare on the same stream before the attention launch
  float* ext;
  int* n_live;
  // Matrix-core kernels, several resident chunks in one launch (n_multi > 0; plain bf16 chunks whose
  // lengths are positive multiples of 64, no mask): their 64-key tiles form one stream in ring
  // order and the running (O~, m, l) stays in registers from the first tile to the last, which is
  // the merge of section 3.4 applied tile by tile.  k, v, Sc and ks above are then unused.
  //
  // With `arrive` set the launch also plays the ring's transfers (Algorithm 2 inside one launch): its
  // first copy_wgs work-groups copy chunk c = 1, 2, .. from k_src / v_src (bytes each) into k / v, a
  // staging buffer of its own per chunk, and count themselves on arrive[c] when their share of chunk
  // c is visible device-wide; an attention work-group waits for arrive[c] == copy_wgs before it
  // loads the first tile of chunk c.  Dependencies only point from the attention work-groups to the
  // copy work-groups, which are dispatched first and wait for nothing.
  //
  // multi_fp8: the sources are FP8 E4M3 chunks ([B,H,Sc,128] codes at k_src / v_src, per-(head, token)
  // scales at k_scale_src / v_scale_src; Algorithm 1 line 4 on arrival).  A copy work-group then
  // decodes while it copies: K's codes widened to bf16 as they are, V's multiplied by their scales,
  // and the per-tile records of the chunk (K's scales as per-key factors) written into `ext`, laid
  // out [B*H][tiles of all chunks in ring order].  Chunk 0 is decoded by a launch of its own
  // (launch_attn_fp8_chunk_prepare) before the attention launch.
  struct Chunk {
    const void* k; const void* v; int64_t ks0, ks1; int Sc;
    const void* k_src; const void* v_src; int64_t bytes;
    const float* k_scale_src; const float* v_scale_src;
    const uint8_t* mask_src;   // key mask [B,Sc] of the chunk (nonzero = key takes part), or null
  };
  static constexpr int kMaxMulti = 16;
  int n_multi;
  int multi_fp8;
  int multi_masked;          // some chunk has a key mask (Chunk::mask_src): the records may flag dead keys.  With bf16
                             // chunks (no multi_fp8) the records are those of launch_attn_multi_records
  int* arrive;               // [kMaxMulti] counters, zero when the launch starts; or null
  // what an attention work-group waits for on arrive[c], and for how long: the launcher sets the
  // count to copy_wgs plus arrive_need_extra and the poll limit to its default when arrive_polls is
  // 0.  Both exist so that a host-side test can make the bounded wait give up (a count that is never
  // reached, a short limit) with every kernel still running to its end.
  int arrive_need_extra;
  int arrive_need;
  int arrive_polls;
  Chunk chunk[kMaxMulti];
  // Prefetch carried by this launch (Algorithm 2, the transfer of the next chunk): the last
  // copy_wgs work-groups of the grid copy the n_copy segments and exit; they are dispatched after
  // the attention work-groups, onto the CU slots those leave free.  The launcher fills copy_wgs (0 when n_copy == 0).
  struct CopySeg { const void* src; void* dst; int64_t bytes; };
  int n_copy;
  int copy_wgs;
  CopySeg copy[4];
};
static_assert(sizeof(AttnStep) <= 4096, "AttnStep is passed by value as the kernels' only argument");
// Copy work-groups appended to a launch of attn_wgs attention work-groups, slots_per_cu of which
// fit on a CU: the CU slots the attention grid leaves free, as a multiple of 8 in [16, 64]
// (one work-group moves about 50 GB/s).
inline int prefetch_wg_count(const AttnStep& s, int attn_wgs, int slots_per_cu) {
  if (s.n_copy <= 0) return 0;
  const int spare = 256 * slots_per_cu - attn_wgs % (256 * slots_per_cu);
  const int n = spare / 8 * 8;
  return n < 16 ? 16 : (n > 64 ? 64 : n);
}
usp_status launch_attn_generic(const AttnStep& s, hipStream_t st);
usp_status launch_attn_mfma(const AttnStep& s, hipStream_t st);
bool attn_mfma_supported(const AttnStep& s);
bool attn_mfma_needs_ext(const AttnStep& s);
size_t attn_mfma_ext_bytes(int B, int H, int Sc);
usp_status launch_attn_ext_prepare(const AttnStep& s, hipStream_t st);
usp_status launch_attn_arrive_reset(int* arrive, hipStream_t st);
// per-tile records (AttnStep::ext, [B*H][tiles in ring order]) of a step over several bf16 chunks some of
// which have a key mask (Chunk::mask_src, multi_masked); precedes the attention launch on the stream
usp_status launch_attn_multi_records(const AttnStep& s, hipStream_t st);
// chunk c of a step over several FP8 chunks decoded by a launch of its own; reset_arrive: the same
// launch zeroes the arrival counters (it precedes the attention launch on the stream)
usp_status launch_attn_fp8_chunk_prepare(const AttnStep& s, int c, bool reset_arrive, hipStream_t st);
// One FP8 chunk of a launch-per-chunk step (s describes it as the only chunk of a several-chunk launch): bf16 K
// and V, the per-tile records and n_live[B] in one launch
usp_status launch_attn_fp8_step_prepare(const AttnStep& s, int* n_live, hipStream_t st);


// What usp_ring_attn_fwd does, with the knobs the ABI does not carry.
struct CallOptions {
  int arrive_need_extra = 0;  // see AttnStep (tests of the give-up path only)
  int arrive_polls = 0;
};
usp_status ring_attn_fwd_impl(const usp_attn_desc* desc, const void* q, const void* const* k_chunks,
                              const void* const* v_chunks, const float* const* k_scales,
                              const float* const* v_scales, const uint8_t* const* key_mask, void* out,
                              float* lse, void* workspace, size_t workspace_bytes, void* compute_stream,
                              void* copy_stream, const CallOptions& opt);

}  // namespace usp
