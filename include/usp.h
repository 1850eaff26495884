/*
 * usp.h - C ABI of the MI355X (gfx950) hot path of Unified Sequence Parallel
 * attention: one rank's blockwise ring attention with log-sum-exp merging, and
 * the FP8 (E4M3) pack/unpack of the All-to-All and ring payloads.
 *
 * Paper: FastUSP (arXiv 2602.10940).  Each entry point names the passage that
 * defines what it computes.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers unless a parameter says "host".
 *   - `stream` parameters are hipStream_t values passed as void* (NULL = the
 *     default stream).  Calls only enqueue work; results are valid once the
 *     compute stream has completed.  The host never blocks inside a call.
 *   - The caller owns every buffer.  The library allocates no device memory
 *     and frees nothing; it keeps a small pool of HIP events per process.
 *   - Return value is a usp_status; on failure nothing has been enqueued
 *     unless the status is USP_ERR_HIP (a launch or event call failed midway).
 *     usp_last_error() gives a thread-local message for the last failure.
 *   - Inputs are assumed finite; NaN/Inf inputs are not checked.
 *   - Calls on different streams may run concurrently, except that two
 *     usp_ring_attn_fwd calls sharing a workspace must not overlap.
 */
#ifndef USP_H
#define USP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  USP_OK = 0,
  USP_ERR_INVALID_ARG = -1, /* null pointer, bad size, misaligned pointer or stride */
  USP_ERR_UNSUPPORTED = -2, /* a combination this build has no kernel for */
  USP_ERR_WORKSPACE = -3,   /* workspace missing or smaller than required */
  USP_ERR_HIP = -4          /* a HIP runtime call failed */
} usp_status;

typedef enum {
  USP_F32 = 0,
  USP_BF16 = 1,
  USP_FP8_E4M3FN = 2 /* 1 byte per element; only valid as kv_dtype */
} usp_dtype;

/* usp_attn_desc.flags */
#define USP_ATTN_DOUBLE_BUFFER 1u /* stage chunks 1..W-1 through two internal buffers on copy_stream */
#define USP_ATTN_UNFUSED_MERGE 2u /* per-chunk (O_i, lse_i) then usp_lse_merge, as Algorithm 2 is written;
                                     default folds the merge into the attention kernel's epilogue */
#define USP_ATTN_FUSED_PREFETCH 16u /* Algorithm 2 without a second stream: the transfers are done by extra
                                      work-groups of the attention launches on compute_stream;
                                      copy_stream is ignored.  Excludes USP_ATTN_DOUBLE_BUFFER.  Two forms:
                                      - one launch per chunk (always with USP_ATTN_STEPWISE or a chunk length
                                        that is not a multiple of 64): step
                                        r's launch carries the transfer of chunk r+1 into the idle one
                                        of two internal buffers, in work-groups that occupy the CUs the
                                        attention grid leaves free.  Same buffers and results as
                                        USP_ATTN_DOUBLE_BUFFER.
                                      - otherwise one launch for the whole ring (see USP_ATTN_STEPWISE):
                                        its first work-groups copy chunks 1..W-1, each into an internal
                                        buffer of its own, and count themselves on a per-chunk arrival
                                        counter; an attention work-group waits for a chunk's count
                                        before it loads that chunk's first keys.  Same result as the
                                        plain call on resident chunks.  FP8 K/V (Algorithm 1 line 4 on
                                        arrival): the same work-groups decode each chunk while they
                                        copy it, into bf16 K (the codes as they are), bf16 V (codes
                                        times scales) and K's scales as per-key factors of the exponent;
                                        the first chunk is decoded by a launch of its own in front;
                                        key masks go into the records as well. */
/* Work decomposition of the bf16 d=128 matrix-core kernel on unmasked chunks whose length is a
 * multiple of 64.  Default (neither bit): chosen from the number of work-groups the Q shard gives.
 * All variants meet the same accuracy bar; the bits exist for tuning and for tests. */
#define USP_ATTN_KERNEL_WIDE 4u   /* 256 queries per work-group, every wave visits every key */
#define USP_ATTN_KERNEL_SPLIT 8u  /* 128 queries per work-group, the two wave groups take alternate
                                     64-key tiles and combine their partial results at the end */
#define USP_ATTN_STEPWISE 64u     /* one attention launch per chunk even where one launch could cover the
                                     whole ring: without USP_ATTN_DOUBLE_BUFFER and USP_ATTN_UNFUSED_MERGE,
                                     bf16 or FP8 chunks (bf16 Q, d = 128), with or without key masks, whose
                                     lengths are multiples of 64 (2 to 16 of them non-empty) are otherwise
                                     taken as one stream of key tiles by a single launch (when the Q
                                     shard's 256-query blocks fit one round of work-groups on the chip,
                                     or the transfers are asked to ride inside the launch), the running
                                     softmax state staying in registers from the first chunk to the last
                                     (no carried state in the workspace); FP8 chunks are decoded by
                                     work-groups of that launch as described under
                                     USP_ATTN_FUSED_PREFETCH, which for them is the same launch.  Same
                                     result up to rounding order. */
#define USP_ATTN_KERNEL_MIXED 32u /* one launch of both: 256-query work-groups, and the blocks of the
                                     last, partly filled round as pairs of key-split work-groups
                                     (forced: the second half of all blocks) */

/*
 * Shape of one ring-attention call (paper section 2.2: Q, K, V are [B, H, S, D]).
 * Strides are in ELEMENTS for the (B, H, token) axes; the head dimension d is
 * always contiguous (stride 1).  Every KV chunk shares kv_stride; chunk r holds
 * chunk_len[r] tokens.  kv_stride = {0,0,0} means "each chunk is a dense
 * [B,H,chunk_len[r],d] array" (the only way to describe dense chunks of unequal length).
 */
typedef struct usp_attn_desc {
  int32_t B, H, d;          /* B*H at most 65535.  d: a multiple of 8 up to 256.  bf16 Q with d = 128 or d = 64 runs on the
                               matrix-core kernels (K and V read in place); every other combination on a slower
                               general kernel */
  int32_t Sq;               /* tokens of the local Q shard */
  int32_t n_chunks;         /* ring degree W >= 1 */
  const int32_t* chunk_len; /* HOST array [n_chunks] */
  int32_t qo_dtype;         /* usp_dtype of q and out: USP_BF16 or USP_F32 */
  int32_t kv_dtype;         /* USP_BF16 / USP_F32 (must equal qo_dtype) or USP_FP8_E4M3FN (with qo BF16) */
  int64_t q_stride[3];      /* elements, (B, H, token) */
  int64_t kv_stride[3];
  int64_t o_stride[3];
  float softmax_scale;      /* multiplies q.k; 0 selects 1/sqrt(d) */
  uint32_t flags;           /* USP_ATTN_* */
} usp_attn_desc;

/*
 * Bytes of device workspace usp_ring_attn_fwd needs for this descriptor
 * (0 is possible, e.g. one f32 chunk; bf16 with d = 128 or 64 always asks for a little, 1 KB per
 * 64 keys of a head).  Returns (size_t)-1 if the descriptor is invalid.
 */
size_t usp_ring_attn_workspace_bytes(const usp_attn_desc* desc);

/*
 * Ring attention of the local Q shard over W KV chunks (section 2.2.2 and
 * Algorithm 2, "Pipelined Ring Attention"): for every chunk r in order,
 *   O_r, lse_r = attn(Q, K_r, V_r)          softmax(Q K_r^T * scale) V_r, lse_r = log sum exp
 *   O, lse     = merge(O, lse, O_r, lse_r)  the two merge equations of section 3.4
 * so that the result equals full attention over the concatenated keys.
 *
 *   q          [B,H,Sq,d] by q_stride, dtype qo_dtype
 *   k_chunks   HOST array of n_chunks device pointers; chunk r is [B,H,chunk_len[r],d]
 *              by kv_stride, dtype kv_dtype.  With FP8 the bytes are dense E4M3 codes.
 *   v_chunks   same for V.  With USP_ATTN_DOUBLE_BUFFER or USP_ATTN_FUSED_PREFETCH the chunks
 *              after the first (and their scales) are only read by the transfers, so they may
 *              also sit in pinned host memory that the device can address (hipHostMalloc): the
 *              transfers then cross the host link, which stands in for a slow ring link.
 *   k_scales / v_scales   NULL unless kv_dtype is FP8: HOST arrays of device pointers,
 *              chunk r -> float [B,H,chunk_len[r]] dense, one scale per (b,h,token)
 *              (value = code * scale, as produced by usp_fp8_quant on the
 *              [B*H*chunk_len, d] view when the chunk is dense).  With bf16 Q and d = 128 or 64
 *              K enters exactly (codes, scale applied to the fp32 scores) and V as
 *              bf16(code * scale); otherwise both products are taken in fp32.
 *   key_mask   NULL, or HOST array of n_chunks device pointers (entries may be NULL):
 *              uint8 [B,chunk_len[r]], nonzero = key takes part.  A query whose keys
 *              are all masked gets O = 0, lse = -inf.
 *   out        [B,H,Sq,d] by o_stride, dtype qo_dtype
 *   lse        float [B,H,Sq] dense, natural log
 *   workspace  device memory, >= usp_ring_attn_workspace_bytes(desc), 256-byte aligned
 *   compute_stream   all kernels run here
 *   copy_stream      used only with USP_ATTN_DOUBLE_BUFFER: chunk r+1 is copied into an
 *              internal buffer here while chunk r is computed (the one-GPU stand-in for
 *              the ring's recv; Algorithm 2 lines 3, 6, 7).  Must differ from compute_stream.
 * Pointers must be 16-byte aligned, strides multiples of 8 elements (bf16) / 4 (f32).
 */
usp_status usp_ring_attn_fwd(const usp_attn_desc* desc, const void* q,
                             const void* const* k_chunks, const void* const* v_chunks,
                             const float* const* k_scales, const float* const* v_scales,
                             const uint8_t* const* key_mask,
                             void* out, float* lse,
                             void* workspace, size_t workspace_bytes,
                             void* compute_stream, void* copy_stream);

/*
 * usp_ring_attn_fwd for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results as usp_ring_attn_fwd (same kernels, same order: bit-identical outputs), minus the
 * workspace and the copy stream: the workspace is an array of USP_NOALLOC_SCRATCH_BYTES that the
 * library holds in device memory on every GPU it runs on, from the first such call on that GPU until
 * the process ends.  The call allocates and frees nothing (no hipMalloc, no events).
 *   - A descriptor whose usp_ring_attn_workspace_bytes() exceeds USP_NOALLOC_SCRATCH_BYTES is refused
 *     with USP_ERR_WORKSPACE and nothing is enqueued (e.g. the FLUX-1024 ring shard needs 17 MB, the
 *     Qwen-Image-like FP8 shard 0.5 GB: the latter has to bring its own workspace).
 *   - USP_ATTN_DOUBLE_BUFFER (side stream and events) is refused with USP_ERR_UNSUPPORTED; the
 *     transfers inside the launches (USP_ATTN_FUSED_PREFETCH) are available.
 *   - Every call on one GPU uses that GPU's one array: calls that overlap in time on one GPU (two
 *     streams, two host threads) race and give undefined results; calls ordered on one stream are
 *     safe.  Nothing is carried from call to call: whatever a call needs to start at zero it clears
 *     itself, on compute_stream.
 *   - The first call on a device looks up the array's address for that device (no allocation); make
 *     that call outside graph capture.
 */
#define USP_NOALLOC_SCRATCH_BYTES (64u << 20)
usp_status usp_ring_attn_fwd_noalloc(const usp_attn_desc* desc, const void* q,
                                     const void* const* k_chunks, const void* const* v_chunks,
                                     const float* const* k_scales, const float* const* v_scales,
                                     const uint8_t* const* key_mask,
                                     void* out, float* lse, void* compute_stream);

/*
 * Merge two partial attention results (section 3.4, the two equations under
 * Algorithm 2; same as the pair in section 2.2.2):
 *   lse = log(exp(lse1) + exp(lse2))
 *   O   = exp(lse1 - lse) * O1 + exp(lse2 - lse) * O2
 * o1, o2, o_out: [rows, d] dense, dtype dt (USP_BF16 or USP_F32); lse*: float [rows].
 * o_out may alias o1 or o2, lse_out may alias lse1 or lse2.  lse = -inf on both
 * sides gives lse = -inf, O = 0.  d must be a multiple of 8.
 */
usp_status usp_lse_merge(int64_t rows, int32_t d, int32_t dt,
                         const void* o1, const float* lse1,
                         const void* o2, const float* lse2,
                         void* o_out, float* lse_out, void* stream);

/*
 * FP8 pack (Algorithm 1 lines 1-2, "FP8 Quantized All-to-All"), one scale per
 * row of the [rows, cols] view (per token; rows = 1 is the per-tensor scale of
 * the algorithm as printed):
 *   a = max_c |x[r,c]|;  s[r] = a / 448 (IEEE float32; a zero quotient is replaced by 1)
 *   q[r,c] = e4m3( x[r,c] / s[r] )   true float32 division, round to nearest even,
 *                                    saturating at +-448, sign of zero kept
 * x: [rows, cols] dense row-major, in_dt USP_BF16 or USP_F32; q: uint8 [rows, cols];
 * scales: float [rows].  cols must be a multiple of 8; rows or cols may be 0.
 */
usp_status usp_fp8_quant(int64_t rows, int64_t cols, int32_t in_dt, const void* x,
                         uint8_t* q, float* scales, void* stream);

/*
 * FP8 unpack (Algorithm 1 line 4):  y[r,c] = float32(decode(q[r,c])) * scales[r],
 * stored as out_dt (USP_F32, or USP_BF16 rounded to nearest even).
 */
usp_status usp_fp8_dequant(int64_t rows, int64_t cols, int32_t out_dt, const uint8_t* q,
                           const float* scales, void* y, void* stream);

/*
 * The same pack / unpack with the rows taken from, or delivered to, the layouts on either side of
 * the All-to-All of section 2.2.1 ([B, H, S/N, D] on the sequence-sharded side, [B, H/N, S, D] on
 * the head-sharded side), so that the send buffer is written, and the receive buffer read, one
 * contiguous block per peer with no separate transposition pass.  Rows are visited as a 4-D index
 * (i0, i1, i2, i3), i3 fastest, n[k] values each (for the exchange: peer, batch, head, token).
 *   usp_fp8_quant_mapped:   row (i0..i3) starts at element  sum_k i_k * src_stride[k]  of x and its
 *                           codes / scale go to row  sum_k i_k * dst_stride[k]  of q [rows, cols] /
 *                           scales [rows]  (rows = n[0]*n[1]*n[2]*n[3]; the destination rows must be
 *                           a permutation of 0 .. rows-1)
 *   usp_fp8_dequant_mapped: row (i0..i3) is read at row  sum_k i_k * src_stride[k]  of q / scales and
 *                           written from element  sum_k i_k * dst_stride[k]  of y on
 * Arithmetic exactly as in usp_fp8_quant / usp_fp8_dequant.  cols: a multiple of 8, at most 4096;
 * element strides must keep every row 16-byte aligned.  Strides are not checked for overlap.
 */
typedef struct usp_row_map {
  int64_t n[4];
  int64_t src_stride[4];
  int64_t dst_stride[4];
} usp_row_map;
usp_status usp_fp8_quant_mapped(const usp_row_map* map, int64_t cols, int32_t in_dt, const void* x,
                                uint8_t* q, float* scales, void* stream);
usp_status usp_fp8_dequant_mapped(const usp_row_map* map, int64_t cols, int32_t out_dt, const uint8_t* q,
                                  const float* scales, void* y, void* stream);

/* Thread-local, statically stored description of the last failure ("" if none). */
const char* usp_last_error(void);

/* Library version string, e.g. "usp-gfx950 0.1". */
const char* usp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* USP_H */
