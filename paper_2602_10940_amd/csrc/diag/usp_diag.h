/*
 * usp_diag.h - entry points of libusp_diag.so: diagnostics for the benchmark and the tests.  Not part
 * of the library's ABI (include/usp.h); conventions (device pointers, streams as void*, usp_status,
 * usp_last_error() of libusp.so) are the same.
 */
#ifndef USP_DIAG_H
#define USP_DIAG_H

#include "usp.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The dense bf16 MFMA rate the device sustains when nothing else is issued: the measured ceiling
 * that the attention kernels' rate can be read against.  wgs work-groups of 8 waves each execute
 * iters * 32 * 32768 flop of MFMAs per wave (shape 0: 32 of 32x32x16; shape 1: 64 of 16x16x32, the
 * shape the attention kernels use; fp32 accumulate) on operands held in registers: pseudo-random
 * values in [-1, 1] if random_data != 0, constants otherwise (the clock the chip holds under load
 * depends on the data and on the shape).
 *   out    : device, wgs * 512 floats, receives per-thread sums (so the work cannot be dropped)
 *   clocks : device, 2 x uint64: shader cycles and 100 MHz ticks that work-group 0 spent in its
 *            loop (their ratio x 100 = shader clock in MHz)
 * Asynchronous on stream.  Limits: 1 <= wgs <= 65536, 1 <= iters <= 1000000. */
usp_status usp_diag_mfma_rate(int32_t wgs, int32_t iters, int32_t random_data, int32_t shape, float* out,
                              uint64_t* clocks, void* stream);

/* The pack kernels cast bf16 rows with a division sequence one correction step shorter than the IEEE
 * one (Algorithm 1 line 2 fixes a true division).  This runs both over EVERY pair (a, x) of bf16 values
 * with a > 0 finite as the row's |x| maximum (scale a / 448) and |x| <= a, both signs, and counts:
 *   counts[0] pairs checked, counts[1] E4M3 codes that differ (must be 0), counts[2] quotients that
 *   differ in some bit (harmless: never across a rounding boundary), counts[3] values of a whose
 *   scale lies outside the range the short sequence is used in.
 * counts: device, 4 x uint64, zeroed by the caller.  Asynchronous on stream. */
usp_status usp_diag_check_bf16_division(uint64_t* counts, void* stream);

/* What a pack launch over a [rows, 3072] bf16 payload costs before any arithmetic, on the pack's own
 * grid (one wave per row): kind 0 = nothing at all (x, q, scales may be NULL), 1 = read every row
 * (its |x| maximum goes to scales[row]), 2 = write rows * 3072 bytes to q.  x: rows * 3072 bf16. */
usp_status usp_diag_payload_floor(int32_t kind, int32_t rows, const void* x, uint8_t* q, float* scales,
                                  void* stream);

/* reps back-to-back calls on one stream, issued from C so that the host's per-call cost (a few
 * microseconds through an interpreter) does not bound what a timing loop measures: call i uses buffer
 * set i % n_sets of the host arrays of device pointers x, q, scales, y (bf16 [rows, cols] payloads).
 *   kind 0: usp_fp8_quant(x -> q, scales)     kind 1: usp_fp8_dequant(q, scales -> y)
 *   kind 2, 3, 4: usp_diag_payload_floor with kind 0, 1, 2 (cols must be 3072)
 * Time it with events around the call. */
usp_status usp_diag_repeat_payload_calls(int32_t kind, int32_t reps, int32_t n_sets, int64_t rows, int64_t cols,
                                         const void* const* x, uint8_t* const* q, float* const* scales,
                                         void* const* y, void* stream);

/* The same for usp_lse_merge on bf16 [rows, d] states: call i uses set i % n_sets of the host arrays. */
usp_status usp_diag_repeat_merge_calls(int32_t reps, int32_t n_sets, int64_t rows, int32_t d, const void* const* o1,
                                       const float* const* lse1, const void* const* o2, const float* const* lse2,
                                       void* const* o_out, float* const* lse_out, void* stream);

/* usp_ring_attn_fwd (same arguments, no copy stream) with the two knobs of the bounded wait that an
 * attention work-group of the one-launch ring makes for a chunk's arrival counter:
 *   arrive_need_extra : added to the count it waits for (> 0: a count that is never reached)
 *   arrive_polls      : poll limit (0 = the library's default, about a second)
 * With a count that is never reached every waiting work-group gives up after arrive_polls polls and
 * returns its rows as NaN in out and lse; every kernel still runs to its end.  Calls that do not take
 * the one-launch form with transfers inside ignore both. */
usp_status usp_diag_ring_attn_fwd_wait(const usp_attn_desc* desc, const void* q,
                                       const void* const* k_chunks, const void* const* v_chunks,
                                       const float* const* k_scales, const float* const* v_scales,
                                       const uint8_t* const* key_mask, void* out, float* lse,
                                       void* workspace, size_t workspace_bytes, void* compute_stream,
                                       int32_t arrive_need_extra, int32_t arrive_polls);

#ifdef __cplusplus
}
#endif
#endif /* USP_DIAG_H */
