// bf16 MFMA attention step for gfx950 (head dimension 128 or 64): for one KV chunk,
//   O_r = softmax(Q K^T * scale) V,   lse_r = log sum_j exp(q.k_j * scale)
// (FastUSP section 2.2 and 2.2.2), with the carried (O, lse) of earlier chunks folded in
// by the merge equations of section 3.4 in the epilogue.
//
// Shape of the computation (all choices are for 64-wide wavefronts and the 16x16x32 bf16 MFMA,
// whose A and B operands hold 8 consecutive contraction-index values per lane and whose 16 x 16
// result puts column (lane % 16), rows 4 * (lane / 16) .. +3 into a lane; under a full matrix load
// the chip holds a 13 % higher clock with this shape than with 32x32x16, which moves twice the
// accumulator data per flop):
//   * A work-group owns 256 queries of one (batch, head); each of its 8 waves owns 32, as two
//     16-query blocks.
//   * Scores are computed TRANSPOSED, S^T = K Q^T (keys are MFMA rows, queries columns), so
//     a lane owns one query column per block: the row max / row sum of the online softmax are in-lane
//     reductions plus two exchanges over the four lanes r, r+16, r+32, r+48.
//   * The exponentiated tile P^T, already in registers in the accumulator layout, is cast to
//     bf16 and used directly as the B operand of O^T += V^T P^T; it never touches LDS.  (The lane
//     that holds keys 16*mb + 4*g + i of a query is the lane that must supply contraction indices
//     8*g + j of the P.V step: the keys of a step are simply taken in that order on the V side.)
//   * K and V tiles (64 keys) sit in LDS row-major, XOR-swizzled instead of padded; the V^T
//     operand (8 keys of one head-dim column per lane) comes from the LDS transposing read.
//   * O and l are rescaled lazily: only when a row max has outgrown the exponent reference.
//   * exp is taken in base 2 with scale * log2(e) folded into one FMA.
#include <atomic>

#include "usp_common.h"
#include "prefetch_copy.h"

namespace usp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
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

// K and V tiles are row-major [key][128 bf16] in LDS without padding; bank conflicts are
// avoided by XOR-swizzling a row (SQ_LDS_BANK_CONFLICT reads 0 for both):
//   K: the 16-byte piece c of key r sits at piece c ^ (r & 15)   (16-byte MFMA operand reads: 16 lanes, 16 rows)
//   V: the 32-byte chunk c of key r sits at chunk c ^ (r & 7)     (transposing 8-byte reads: 32 lanes, 8 rows of 32 bytes)
// (head dimension 64, 128-byte rows: see attn_pp_body)
// Work-group -> (batch*head, query block) with the 8 XCDs of the chip in mind: consecutive
// work-group ids go to consecutive XCDs (id % 8), each with its own L2.  The (head, query block)
// items, head-major, are cut into 8 contiguous ranges of equal length, one per XCD: the query
// blocks of a head stay on one XCD (two where a range boundary falls inside a head), so its K/V
// is fetched from HBM once or twice instead of once per XCD, and every XCD gets the same number
// of work-groups whatever the head count.  The grid holds 8 * ceil(items / 8) ids; ids past the
// last item return false.
constexpr int kXcds = 8;
constexpr int kSplitBelowWGs = 128;   // use the key-split kernel when 256-query work-groups number at most this
__device__ __forceinline__ bool wg_to_tile(int copy_wgs, int nqb, int bh_total, int& bh, int& qb, int lead = 0) {
  const int id = blockIdx.x - lead;                   // the copy work-groups are the last ids of the grid, or the first `lead` (a multiple of 8)
  const int per_xcd = ((int)gridDim.x - copy_wgs) / kXcds;
  const int item = (id % kXcds) * per_xcd + id / kXcds;
  bh = item / nqb;
  qb = item - bh * nqb;
  return bh < bh_total;
}
static inline unsigned wg_grid_size(int nqb, int bh_total) {
  return (unsigned)(kXcds * ((bh_total * nqb + kXcds - 1) / kXcds));
}

// A query's values sit in the four lanes r, r + 16, r + 32, r + 48 (r = lane % 16): maximum / sum over them,
// left in all four (two swaps: rows of 16 lanes pairwise, then the halves of the wave).
__device__ __forceinline__ float xgroup_max(float x) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float xgroup_sum(float x) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// Chunk result of one query from its running state (reference m in log2 units, sum l), merged with the
// carried lse of earlier chunks by the section 3.4 equations: the factor for this chunk's O~ (c_cur), the
// weight of the carried O (w_prev) and the new lse.
// `invalid`: the rows are not to be trusted (a chunk of the ring never arrived): O and lse become NaN,
// which no valid result is (a query whose keys are all masked gets O = 0, lse = -inf).
struct RowFinish { float c_cur, w_prev, lse_new; };
__device__ __forceinline__ RowFinish finish_row(const AttnStep& s, float m, float l, int64_t lse_row, bool invalid) {
  RowFinish f;
  float lse_r = -INFINITY;
  f.c_cur = 0.0f;
  if (l > 0.0f) { lse_r = (m + log2f(l)) * 0.69314718055994530942f; f.c_cur = 1.0f / l; }
  f.w_prev = 0.0f;
  f.lse_new = lse_r;
  if (s.mode >= 2) {
    const float lse_p = s.lse[lse_row];
    const float mm = fmaxf(lse_p, lse_r);
    if (mm == -INFINITY) { f.w_prev = 0.0f; f.c_cur = 0.0f; f.lse_new = -INFINITY; }
    else {
      f.lse_new = mm + logf(expf(lse_p - mm) + expf(lse_r - mm));
      f.w_prev = expf(lse_p - f.lse_new);
      f.c_cur *= expf(lse_r - f.lse_new);
    }
  }
  if (invalid) { f.c_cur = __builtin_nanf(""); f.lse_new = f.c_cur; }
  return f;
}

// Chunk result, merge and store straight from the accumulator layout (a lane holds four consecutive head
// dims of a query: 8 bytes of bf16 or 16 bytes of the fp32 carry per store): what the key-split
// work-groups use, whose epilogue is too short for the detour through LDS to pay.
// kHalfD: head dimension 64: only the first four 16-wide blocks exist, rows are 64 wide everywhere.
template <bool kHalfD>
__device__ __forceinline__ void finish_and_store_direct(const AttnStep& s, f32x4 (&oacc)[8][2], const float (&m)[2],
                                                        const float (&lsum)[2], int b, int h, int q0, int r, int g, bool invalid) {
  constexpr int kDB = kHalfD ? 4 : 8;
  constexpr int kAccP = kHalfD ? 64 : kD;   // floats per row of the carried O
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const float l = xgroup_sum(lsum[nb]);
    const int qi = q0 + 16 * nb + r;
    const bool valid = qi < s.Sq;
    const int64_t row = ((int64_t)b * s.H + h) * s.Sq + (valid ? qi : s.Sq - 1);
    const RowFinish f = finish_row(s, m[nb], l, row, invalid);
    if (!valid) continue;
    float* accp = s.acc ? s.acc + row * kAccP : nullptr;
    bf16_t* outp = (bf16_t*)s.out + b * s.os[0] + h * s.os[1] + (int64_t)qi * s.os[2];
#pragma unroll
    for (int db = 0; db < kDB; ++db) {
      const int dcol = 16 * db + 4 * g;
      float o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = oacc[db][nb][e] * f.c_cur;
      if (s.mode >= 2) {
        const float4 p = *reinterpret_cast<const float4*>(accp + dcol);
        o[0] = fmaf(f.w_prev, p.x, o[0]); o[1] = fmaf(f.w_prev, p.y, o[1]);
        o[2] = fmaf(f.w_prev, p.z, o[2]); o[3] = fmaf(f.w_prev, p.w, o[3]);
      }
      if (s.mode == 1 || s.mode == 2)
        *reinterpret_cast<float4*>(accp + dcol) = make_float4(o[0], o[1], o[2], o[3]);
      else
        *reinterpret_cast<uint2*>(outp + dcol) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
    }
    if (g == 0) s.lse[row] = f.lse_new;
  }
}

// The same for the 256-query work-groups.  In the accumulator layout direct stores would touch 16 rows
// with 32 bytes each per instruction.  The wave therefore turns its 32 x 128 tile through its own LDS
// region (row pitch 528 bytes, so that rows do not all start in the same bank) and then moves
// whole rows: 32 lanes x 16 bytes (fp32 carry, read and write) or x 8 bytes (bf16 output) per row,
// two rows per instruction.  Only this wave touches the region; LDS operations of one wave complete
// in order, so no barrier is needed.
constexpr int kEpiPitch = kD * 4 + 16;                    // bytes per staged row
constexpr int kEpiWaveB = kQPerWave * kEpiPitch + 512;    // + per-row (scale of O~, weight of the carry, lse, unused)
template <bool kHalfD>
__device__ __forceinline__ void finish_and_store(const AttnStep& s, f32x4 (&oacc)[8][2], const float (&m)[2],
                                                 const float (&lsum)[2], int b, int h, int q0, int r, int g,
                                                 unsigned char* epi, bool invalid) {
  constexpr int kDB = kHalfD ? 4 : 8;
  constexpr int kAccP = kHalfD ? 64 : kD;                 // floats per row of the carried O
  const int lane = r + 16 * g;
  const int64_t row0 = ((int64_t)b * s.H + h) * s.Sq;     // first row of this (batch, head) in lse / acc
  float* info = reinterpret_cast<float*>(epi + kQPerWave * kEpiPitch);
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const float l = xgroup_sum(lsum[nb]);
    const int qr = 16 * nb + r;                           // row of the wave's tile
    const int qi = q0 + qr;
    const RowFinish f = finish_row(s, m[nb], l, row0 + min(qi, s.Sq - 1), invalid);
    if (g == 0 && qi < s.Sq) s.lse[row0 + qi] = f.lse_new;
    if (g == 0) { info[2 * qr] = f.c_cur; info[2 * qr + 1] = f.w_prev; }
    // stage: row qr, head dims 16*db + 4*g .. +3
#pragma unroll
    for (int db = 0; db < kDB; ++db)
      *reinterpret_cast<f32x4*>(epi + qr * kEpiPitch + (16 * db + 4 * g) * 4) = oacc[db][nb];
  }
  // rows: lane (r2, c) handles head dims 4c .. 4c+3 of rows 2*it + r2
  const int r2 = lane >> 5, c = lane & 31;
  const int rows_valid = min(kQPerWave, s.Sq - q0);       // <= 0: nothing to store
#pragma unroll 4
  for (int it = 0; it < kQPerWave / 2; ++it) {
    const int rr = 2 * it + r2;
    if (rr >= rows_valid || (kHalfD && c >= 16)) continue;   // kHalfD: rows are 64 wide
    const f32x4 v = *reinterpret_cast<const f32x4*>(epi + rr * kEpiPitch + c * 16);
    const float cc = info[2 * rr], wp = info[2 * rr + 1];
    float o[4] = {v[0] * cc, v[1] * cc, v[2] * cc, v[3] * cc};
    const int64_t row = row0 + q0 + rr;
    if (s.mode >= 2) {
      const float4 p = *reinterpret_cast<const float4*>(s.acc + row * kAccP + 4 * c);
      o[0] = fmaf(wp, p.x, o[0]); o[1] = fmaf(wp, p.y, o[1]);
      o[2] = fmaf(wp, p.z, o[2]); o[3] = fmaf(wp, p.w, o[3]);
    }
    if (s.mode == 1 || s.mode == 2)
      *reinterpret_cast<float4*>(s.acc + row * kAccP + 4 * c) = make_float4(o[0], o[1], o[2], o[3]);
    else {
      bf16_t* outp = (bf16_t*)s.out + b * s.os[0] + h * s.os[1] + (int64_t)(q0 + rr) * s.os[2];
      // the final output is not read again here: a streaming store leaves no dirty line for the
      // end of the kernel to write back (the fp32 carry above is re-read by the next step and stays cached)
      const u32x2 v2 = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
      __builtin_nontemporal_store(v2, reinterpret_cast<u32x2*>(outp + 4 * c));
    }
  }
}

// =============================================================================================
// Ping-pong kernels.
//
// The 8 waves form two groups (waves 0-3 = A, 4-7 = B; each SIMD hosts one wave of each; the
// register budget of 32 queries x 128 head dims per wave allows no more than these two).  A
// wave alternates between a softmax phase SM(t) (VALU only: scores of tile t -> bf16 P) and a
// matrix phase MM(t) (MFMA only: O += P(t) V(t), then the scores of its next tile).  The groups
// run half a period apart and a work-group barrier separates the phases, so in every phase one
// wave of each SIMD feeds the matrix core while the other does the exponentials.
//
// Two work decompositions (template parameter kSplit):
//   wide  : 256 queries per work-group, each wave its own 32; every wave visits every tile.
//             phase 2j   : A does SM(j),  B does MM(j-1)
//             phase 2j+1 : A does MM(j),  B does SM(j)
//   split : 128 queries per work-group, waves w and w+4 share 32 queries; group A takes the even
//           tiles, group B the odd ones, and B's partial (O~, m, l) is folded into A's through
//           LDS at the end.  Twice the work-groups for half the time each: for Q shards too
//           small to fill the chip with 256-query work-groups.
//             phase p : the owner of tile p does SM(p), the other group MM(p-1)
// K and V tiles go through three LDS stages each, written by direct global->LDS loads issued
// from the softmax phases (whose critical resource, the VALU, is not the matrix core's).
//
// Template parameter kExt adds what the plain kernels exclude: per-key scales of FP8 K/V
// (Algorithm 1, line 4, applied to the fp32 scores and to P instead of to K and V), a key mask,
// and a chunk length that is not a multiple of 64.  A small kernel run before the attention
// kernel turns scales, mask and length into four vectors of 64 floats per (batch, head, tile):
//   c    = k_scale * softmax_scale * log2(e)   (0 for a masked or out-of-range key)
//   bias = 0, or -inf for a masked or out-of-range key
//   flag = (flag[0] != 0) iff the tile has any such key
//   (a fourth, unused, vector keeps one 256-byte load per wave of the loading group)
// and the tile's record follows its K tile through the LDS stages.  The scales of FP8 V are not
// applied here: V is widened to bf16 as round(code * v_scale) before the kernel runs (the dequantise
// step of Algorithm 1 in the working precision), because a multiply per P element would make the
// softmax phase, which issues from a single wave per SIMD, the longer of the two phases.  K keeps
// its exact codes: its scale costs nothing inside the exponent's FMA, and rounding K would move
// the scores themselves.
//
// Template parameter kMulti lets one launch cover a whole ring (Algorithm 2): the 64-key tiles of up
// to 16 chunks (whole tiles only) form one stream in ring order, a cursor maps a tile index to
// its chunk's pointer, and the running (O~, m, l) stays in registers from the first tile to the
// last, which is the merge of section 3.4 applied tile by tile.  With AttnStep::arrive set the
// launch also plays the ring's transfers: its first work-groups copy the chunks into staging
// buffers and count themselves on a per-chunk arrival counter (prefetch_copy.h), and an attention
// work-group waits for a chunk's count before it loads the chunk's first tile (wait_arrival).
// FP8 chunks (AttnStep::multi_fp8) are decoded by those work-groups on the way (Algorithm 1 line 4:
// K widened, V dequantised, the records above written, masks included) and attended by the
// record-reading form; there the tiles of a chunk that came with a mask read their dead-key flag
// from the record in LDS (it cannot be fetched ahead from memory the launch is still writing).
//
// kNoDead: records that carry only per-key factors (no mask, whole tiles): flag and bias are never
// read.  kHalfD: head dimension 64 (see attn_pp_body).
// =============================================================================================
__device__ __forceinline__ void lds_dma16(const void* gbase, uint32_t lane_off, uint32_t lds_base) {
  // 64 lanes x 16 bytes from gbase (wave-uniform) + lane_off (per lane): lane i's 16 bytes land at
  // lds_base + 16*i.  Issued through inline asm so the compiler does not serialise later LDS reads
  // behind it; completion is awaited with an explicit vmcnt wait before the barrier that
  // publishes the tile.
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_base), "v"(lane_off), "s"(gbase) : "memory", "m0");
}
__device__ __forceinline__ void lds_dma4(const void* gbase, uint32_t lane_off, uint32_t lds_base) {
  // the same with 4 bytes per lane: lane i's dword lands at lds_base + 4*i
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
               :: "s"(lds_base), "v"(lane_off), "s"(gbase) : "memory", "m0");
}
constexpr int kStages = 3;       // LDS tile buffers per tensor
constexpr int kExtTileB = 1024;  // bytes of one tile's record of the extended path: c | bias | flag | unused

struct SmemPP {
  unsigned char k[kStages][kTileB];
  unsigned char v[kStages][kTileB];
};
// The wide work-groups' epilogue stages each wave's O tile through LDS (eight regions from offset 0,
// over the tile stages, which are dead by then).
constexpr int kLdsBytes = 8 * kEpiWaveB;
struct SmemPPExt {
  unsigned char k[kStages][kTileB];
  unsigned char v[kStages][kTileB];
  unsigned char ext[4][kExtTileB];   // the 256-query kernel rotates its records over four stages
};

// LDS transposing read: the 16 lanes of a group each name 8 bytes; seen as a 4 x 16 matrix of
// bf16 (row i = the data of lanes 4i..4i+3), lane j of the group receives column j.
__device__ __forceinline__ u32x2 lds_read_tr3(const __attribute__((address_space(3))) unsigned char* p) {
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
  return __builtin_bit_cast(u32x2, r);
}


// One work-group of 64 threads per (tile, batch*head): the record described above.  Blocks of tile 0
// with h == 0 also count the tiles up to the last one that has a live key (n_live[b]); the
// attention kernel stops there.
__global__ __launch_bounds__(64) void attn_ext_prepare_kernel(AttnStep s, float* ext, int* n_live) {
  const int tile = blockIdx.x, bh = blockIdx.y, t = threadIdx.x;
  const int b = bh / s.H;
  const int nt_all = (s.Sc + kTile - 1) / kTile;   // the grid has max(nt_all, 1) tiles
  const uint8_t* mask = s.key_mask ? s.key_mask + (int64_t)b * s.Sc : nullptr;
  if (tile < nt_all) {
    const int key = tile * kTile + t;
    const bool keep = key < s.Sc && (!mask || mask[key] != 0);
    const int64_t srow = (int64_t)bh * s.Sc + key;
    float* rec = ext + ((int64_t)bh * nt_all + tile) * (kExtTileB / 4);
    const float scale2 = s.scale * 1.44269504088896340736f;
    rec[t] = keep ? (s.k_scale ? s.k_scale[srow] : 1.0f) * scale2 : 0.0f;
    rec[64 + t] = keep ? 0.0f : -INFINITY;
    rec[128 + t] = __builtin_amdgcn_ballot_w64(!keep) != 0ull ? 1.0f : 0.0f;
    rec[192 + t] = 0.0f;
  }
  if (tile == 0 && bh % s.H == 0) {
    int last = -1;   // last live key of this batch entry
    if (!mask) last = s.Sc - 1;
    else {
#pragma unroll 8
      for (int k0 = t; k0 < s.Sc; k0 += 64)
        if (mask[k0] != 0) last = k0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) last = max(last, __shfl_xor(last, o, 64));
    if (t == 0) n_live[b] = last < 0 ? 0 : last / kTile + 1;
  }
}

// Records of a launch over several bf16 chunks of which some have a key mask: one work-group of 64
// threads per (tile of the ring's tile stream, batch*head), laid out [B*H][tiles in ring order] like
// the records the FP8 form writes while it decodes.  Masks are inputs of the call, not part of what
// the ring transfers, so the records of every chunk can be written before the attention launch.
__global__ __launch_bounds__(64) void attn_multi_records_kernel(AttnStep s) {
  int tile = blockIdx.x;
  const int bh = blockIdx.y, t = threadIdx.x;
  int nt_total = 0;
  for (int c = 0; c < s.n_multi; ++c) nt_total += s.chunk[c].Sc / kTile;
  int c = 0;
  while (tile >= s.chunk[c].Sc / kTile) { tile -= s.chunk[c].Sc / kTile; ++c; }   // (the grid has nt_total tiles)
  const AttnStep::Chunk& ch = s.chunk[c];
  const int key = tile * kTile + t;
  const bool keep = ch.mask_src == nullptr || ch.mask_src[(int64_t)(bh / s.H) * ch.Sc + key] != 0;
  float* rec = s.ext + ((int64_t)bh * nt_total + blockIdx.x) * (kExtTileB / 4);
  rec[t] = keep ? s.scale * 1.44269504088896340736f : 0.0f;
  rec[64 + t] = keep ? 0.0f : -INFINITY;
  rec[128 + t] = __builtin_amdgcn_ballot_w64(!keep) != 0ull ? 1.0f : 0.0f;
  rec[192 + t] = 0.0f;
}

// Wait of an attention work-group for a chunk that the copy work-groups of the same launch are still
// writing: polls the chunk's counter with device-scope loads until it reaches `need`.  The copy
// work-groups are dispatched before every attention work-group and wait for nothing, so the count
// is reached; the poll limit (of the order of a second by default) only keeps a launch from spinning
// forever should that ever not hold, at the price of a result the caller can recognise as invalid:
// every row of a work-group one of whose waves gave up is returned as NaN in out and lse.
constexpr int kArrivePolls = 1 << 21;
__device__ __forceinline__ bool wait_arrival(const int* counter, int need, int polls) {
  for (int i = 0; i < polls; ++i) {
    if (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= need) {
      asm volatile("" ::: "memory");
      return true;
    }
    __builtin_amdgcn_s_sleep(4);
  }
  return false;
}
__global__ __launch_bounds__(64) void attn_arrive_reset_kernel(int* arrive) {
  if (threadIdx.x < AttnStep::kMaxMulti) arrive[threadIdx.x] = 0;
}
// Chunk c of a launch over several FP8 chunks, decoded by a launch of its own (the first chunk,
// which no attention work-group could overlap with anything).
__global__ __launch_bounds__(256) void attn_fp8_chunk_prepare_kernel(AttnStep s, int c, int reset_arrive) {
  if (reset_arrive && blockIdx.x == 0 && threadIdx.x < AttnStep::kMaxMulti) s.arrive[threadIdx.x] = 0;
  fp8_chunk_prepare<false>(s, c, (int64_t)blockIdx.x * 256 + threadIdx.x, (int64_t)gridDim.x * 256);
}

// The same for a step of the launch-per-chunk form (the chunk is s.chunk[0] of a one-chunk description):
// codes -> bf16 K and V and the per-tile records in one launch instead of three, plus the count of tiles up
// to the last live key of every batch entry, which the attention kernel of a single chunk stops at.
__global__ __launch_bounds__(256) void attn_fp8_step_prepare_kernel(AttnStep s, int* n_live) {
  fp8_chunk_prepare<false>(s, 0, (int64_t)blockIdx.x * 256 + threadIdx.x, (int64_t)gridDim.x * 256);
  if (blockIdx.x == 0 && threadIdx.x < 64) {
    const AttnStep::Chunk& ch = s.chunk[0];
    const int t = threadIdx.x;
    for (int b = 0; b < s.B; ++b) {
      int last = ch.Sc - 1;
      if (ch.mask_src != nullptr) {
        last = -1;
        const uint8_t* mask = ch.mask_src + (int64_t)b * ch.Sc;
#pragma unroll 8
        for (int k0 = t; k0 < ch.Sc; k0 += 64)
          if (mask[k0] != 0) last = k0;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) last = max(last, __shfl_xor(last, o, 64));
      }
      if (t == 0) n_live[b] = last < 0 ? 0 : last / kTile + 1;
    }
  }
}

// One work-group's share: the queries q_base .. q_base + 255 (wide) or + 127 (split) of (batch, head) bh_.
// kNoDead (with kExt): the records carry per-key factors only, no key of the launch is dead (FP8
// scales on unmasked chunks of whole tiles): the per-tile flag is not read at all.
// kHalfD: head dimension 64: rows of Q, K, V and O are 128 bytes (K and V are read in place, their LDS
// tiles have 128-byte rows with swizzles of their own), the scores contract over two 32-wide slices
// of the head dimension and P.V produces four 16-wide blocks.
template <bool kSplit, bool kExt, bool kMulti = false, bool kNoDead = false, bool kHalfD = false>
__device__ __forceinline__ void attn_pp_body(const AttnStep& s, unsigned char* smem_raw, int bh_, int q_base) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it in an SGPR
  const int r = lane & 15, g = lane >> 4;   // MFMA column (a query) and 8-wide slice of the contraction index
  constexpr int kKS = kHalfD ? 2 : 4;        // 32-wide slices of the head dimension (contraction of the scores)
  constexpr int kNV = kHalfD ? 2 : 4;        // operands of either kind per block of the matrix phase
  constexpr int kDB = kHalfD ? 4 : 8;        // 16-wide blocks of the head dimension that P.V produces
  constexpr int kBurst = 1;                  // operands whose MFMAs are issued back to back before the next reads (1, 2, 4: no difference measured)
  const int h = bh_ % s.H, b = bh_ / s.H;
  // split: waves w and w+4 share their 32 queries
  const int q0 = q_base + (kSplit ? (wave & 3) : wave) * kQPerWave;
  const bool grpA = wave < 4;

  const bf16_t* qb = (const bf16_t*)s.q + b * s.qs[0] + h * s.qs[1];
  const unsigned char* kb = (const unsigned char*)((const bf16_t*)s.k + b * s.ks[0] + h * s.ks[1]);
  const unsigned char* vb = (const unsigned char*)((const bf16_t*)s.v + b * s.ks[0] + h * s.ks[1]);
  const float scale2 = s.scale * 1.44269504088896340736f;
  // plain: the host guarantees Sc % 64 == 0 and Sc > 0.  extended: tiles up to the last live key;
  // the last tile of the chunk may be ragged (tail_tile), none may be left (nt == 0).
  // several chunks per launch: full tiles only; with records (kExt) these follow the tile stream
  int nt_multi = 0;
  if (kMulti)
    for (int c = 0; c < s.n_multi; ++c) nt_multi += s.chunk[c].Sc / kTile;
  const int nt_all = kMulti ? nt_multi : (s.Sc + kTile - 1) / kTile;
  const int nt = kMulti ? nt_multi
                        : kExt ? min(nt_all, __builtin_amdgcn_readfirstlane(s.n_live[b])) : s.Sc / kTile;
  const int tail_tile = (kExt && !kMulti && (s.Sc % kTile) != 0) ? nt_all - 1 : -1;
  const int tail_last_row = s.Sc - (nt_all - 1) * kTile - 1;   // last valid row of the ragged tile

  f32x4 oacc[8][2];   // O~^T: [16-wide head-dim block db][16-query block nb]: head dims 16*db + 4*g + i of query 16*nb + r
#pragma unroll
  for (int db = 0; db < 8; ++db)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) oacc[db][nb] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  float m[2] = {-INFINITY, -INFINITY}, lsum[2] = {0.0f, 0.0f};   // per query block
  bool late = false;   // an awaited chunk never arrived (see wait_arrival): the results are replaced by NaN
  int arrived_upto = 0, probe_c = 0, probe_val = 0;   // chunks known to have arrived; the count read ahead for chunk probe_c
  constexpr int kProbeAheadTiles = 4;

  if (!kExt || nt > 0) {   // (uniform over the work-group)
  // ---- direct global->LDS tile loads, 4 rows (16 lanes each) per instruction.  wide: wave w moves
  // rows 8w..8w+7 of every tile.  split: only the group in its softmax phase loads, wave w its own
  // rows 8w..8w+7 and those of its partner w^4, 32 rows away (same swizzle: 32 is a multiple of
  // 16).  Per-lane byte offsets inside a tile are fixed; the tile base pointers advance as scalars.
  // kHalfD (head dimension 64): rows are 128 bytes in global memory and in LDS, so one instruction moves
  // 8 rows (8 lanes each) and a wave's share of a tile is a single load per tensor; the swizzles are
  //   K: piece c (of 8) of key r sits at piece c ^ ((r >> 1) & 7)   (two rows share a sweep of the banks)
  //   V: the 64-byte half h of key r sits at half h ^ ((r >> 1) & 1)
  constexpr int RB = kHalfD ? 128 : kRowB;   // bytes per K / V row in LDS
  const int dma_r0 = 8 * wave + (kHalfD ? (lane >> 3) : (lane >> 4)), dma_r1 = dma_r0 + 4;
  const int dma_p = kHalfD ? (lane & 7) : (lane & 15);
  const uint32_t rowB = (uint32_t)(s.ks[2] * 2);   // bytes between keys in global memory
  const int64_t tileB = (int64_t)kTile * rowB;
  const uint32_t ksw0 = kHalfD ? (uint32_t)((dma_p ^ ((dma_r0 >> 1) & 7)) << 4) : (uint32_t)((dma_p ^ (dma_r0 & 15)) << 4);
  const uint32_t ksw1 = (dma_p ^ (dma_r1 & 15)) << 4;
  // V: the 32-byte chunk c of key r sits at chunk c ^ (r & 7) (kHalfD: c ^ ((r >> 1) & 3)): in 16-byte pieces
  const uint32_t vsw0 = kHalfD ? (uint32_t)((dma_p ^ (((dma_r0 >> 1) & 3) << 1)) << 4) : (uint32_t)((dma_p ^ ((dma_r0 & 7) << 1)) << 4);
  const uint32_t vsw1 = (dma_p ^ ((dma_r1 & 7) << 1)) << 4;
  const uint32_t kg0 = dma_r0 * rowB + ksw0, kg1 = dma_r1 * rowB + ksw1;
  const uint32_t vg0 = dma_r0 * rowB + vsw0, vg1 = dma_r1 * rowB + vsw1;
  const uint32_t lds_base = (uint32_t)(uintptr_t)smem_raw;
  const uint32_t lds_k = __builtin_amdgcn_readfirstlane(lds_base + 8 * wave * RB);
  const uint32_t lds_v = __builtin_amdgcn_readfirstlane(lds_base + kStages * kTileB + 8 * wave * RB);
  const int pair_rows = kSplit ? (grpA ? 32 : -32) : 0;
  // rows past the end of a ragged last tile re-read its last valid row (finite data; their P is 0)
  auto row_off = [&](int r, int tile_idx) -> uint32_t {
    if (kExt && tile_idx == tail_tile) r = min(r, tail_last_row);
    return (uint32_t)r * rowB;
  };
  auto issue_k_half = [&](const unsigned char* tile, int tile_idx, int stage, int half, bool pair) {
    if (kHalfD && half) return;               // one load covers the wave's 8 rows
    const int dr = pair ? pair_rows : 0;
    uint32_t off = half ? kg1 : kg0;
    if (kExt && tile_idx == tail_tile) { off = row_off((half ? dma_r1 : dma_r0) + dr, tile_idx) + (half ? ksw1 : ksw0); }
    else tile += (int64_t)dr * rowB;
    lds_dma16(tile, off, lds_k + dr * RB + stage * kTileB + half * 4 * RB);
  };
  auto issue_v_half = [&](const unsigned char* tile, int tile_idx, int stage, int half, bool pair) {
    if (kHalfD && half) return;
    const int dr = pair ? pair_rows : 0;
    uint32_t off = half ? vg1 : vg0;
    if (kExt && tile_idx == tail_tile) { off = row_off((half ? dma_r1 : dma_r0) + dr, tile_idx) + (half ? vsw1 : vsw0); }
    else tile += (int64_t)dr * rowB;
    lds_dma16(tile, off, lds_v + dr * RB + stage * kTileB + half * 4 * RB);
  };
  // extended path: the four 64-float vectors of a tile's record, one per wave of the loading group
  const unsigned char* extb = kExt ? (const unsigned char*)(s.ext + (int64_t)bh_ * nt_all * (kExtTileB / 4)) : nullptr;
  const uint32_t lds_ext = lds_base + 2 * kStages * kTileB;
  // kMulti: the record of a tile is written by the copy work-groups together with its chunk
  int xcur_c = 0, xcur_first = 0;
  auto await_record = [&](int idx) {
    while (idx >= xcur_first + s.chunk[xcur_c].Sc / kTile) {
      xcur_first += s.chunk[xcur_c].Sc / kTile;
      ++xcur_c;
      if (s.arrive != nullptr && xcur_c > arrived_upto) {
        if (!wait_arrival(s.arrive + xcur_c, s.arrive_need, s.arrive_polls)) late = true;
        arrived_upto = xcur_c;
      }
    }
  };
  auto issue_ext = [&](int tile_idx, int stage) {
    if (kMulti) await_record(tile_idx);
    lds_dma4(extb + (int64_t)tile_idx * kExtTileB + (wave & 3) * 256, lane * 4,
             lds_ext + stage * kExtTileB + (wave & 3) * 256);
  };
  auto issue_k_tile = [&](const unsigned char* tile, int tile_idx, int stage) {   // this wave's share
    issue_k_half(tile, tile_idx, stage, 0, false); issue_k_half(tile, tile_idx, stage, 1, false);
    if (kSplit) { issue_k_half(tile, tile_idx, stage, 0, true); issue_k_half(tile, tile_idx, stage, 1, true); }
  };
  auto issue_v_tile = [&](const unsigned char* tile, int tile_idx, int stage) {
    issue_v_half(tile, tile_idx, stage, 0, false); issue_v_half(tile, tile_idx, stage, 1, false);
    if (kSplit) { issue_v_half(tile, tile_idx, stage, 0, true); issue_v_half(tile, tile_idx, stage, 1, true); }
  };

  // Where tile idx of the K (or V) stream starts.  kMulti: the tiles of the chunks follow one another;
  // a cursor (chunk, index of its first tile) moves forward with the indices asked for.
  struct TileCursor { int c, first; };
  auto tile_at = [&](TileCursor& cur, int idx, bool is_v) -> const unsigned char* {
    if (!kMulti) return (is_v ? vb : kb) + idx * tileB;
    while (idx >= cur.first + s.chunk[cur.c].Sc / kTile) {
      cur.first += s.chunk[cur.c].Sc / kTile;
      ++cur.c;
      if (s.arrive != nullptr && cur.c > arrived_upto) {
        // the count read a few tiles ago usually settles it; otherwise poll
        const bool seen = probe_c == cur.c && __builtin_amdgcn_readfirstlane(probe_val) >= s.arrive_need;
        if (!seen && !wait_arrival(s.arrive + cur.c, s.arrive_need, s.arrive_polls)) late = true;
        arrived_upto = cur.c;
      }
    }
    // a few tiles before the K stream leaves a chunk, read the next chunk's count without waiting
    // for the answer: a blocking poll at the boundary costs a round trip to memory on the critical path
    if (s.arrive != nullptr && !is_v && cur.c + 1 < s.n_multi && cur.c + 1 > arrived_upto && probe_c <= cur.c &&
        idx + kProbeAheadTiles >= cur.first + s.chunk[cur.c].Sc / kTile) {
      probe_c = cur.c + 1;
      probe_val = __hip_atomic_load(s.arrive + probe_c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const AttnStep::Chunk& ch = s.chunk[cur.c];
    const bf16_t* base = (const bf16_t*)(is_v ? ch.v : ch.k) + b * ch.ks0 + h * ch.ks1;
    return (const unsigned char*)base + (idx - cur.first) * tileB;
  };
  TileCursor kcur{0, 0}, vcur{0, 0};

  // Tiles needed before the first loads of the softmax phases land are fetched here.
  //   wide : A's SM(j) prefetches K(j+2) (with its record) and V(j+1); B's SM(j), one phase later,
  //          K(j+3) and V(j+2).
  //   split: the softmax phase p prefetches K(p+3), V(p+1) and the record of tile p+2.
  int kpre_idx, vpre_idx;   // next K / V tile this wave prefetches
  if (!kSplit) {
    { const unsigned char* t = tile_at(kcur, 0, false); issue_k_half(t, 0, 0, 0, false); issue_k_half(t, 0, 0, 1, false); }
    { const unsigned char* t = tile_at(vcur, 0, true); issue_v_half(t, 0, 0, 0, false); issue_v_half(t, 0, 0, 1, false); }
    if (nt > 1) { const unsigned char* t = tile_at(kcur, 1, false); issue_k_half(t, 1, 1, 0, false); issue_k_half(t, 1, 1, 1, false); }
    if (!grpA) {
      if (nt > 1) { const unsigned char* t = tile_at(vcur, 1, true); issue_v_half(t, 1, 1, 0, false); issue_v_half(t, 1, 1, 1, false); }
      if (nt > 2) { const unsigned char* t = tile_at(kcur, 2, false); issue_k_half(t, 2, 2, 0, false); issue_k_half(t, 2, 2, 1, false); }
    } else if (kExt) {
      issue_ext(0, 0);
      if (nt > 1) issue_ext(1, 1);
    }
    kpre_idx = grpA ? 2 : 3;
    vpre_idx = grpA ? 1 : 2;
  } else {
    if (grpA) {   // the loading lambdas of the split kernel move a wave pair's rows: one group suffices
      issue_k_tile(tile_at(kcur, 0, false), 0, 0);
      issue_v_tile(tile_at(vcur, 0, true), 0, 0);
      if (nt > 1) issue_k_tile(tile_at(kcur, 1, false), 1, 1);
      if (nt > 2) issue_k_tile(tile_at(kcur, 2, false), 2, 2);
      if (kExt) {
        issue_ext(0, 0);
        if (nt > 1) issue_ext(1, 1);
      }
    }
    kpre_idx = grpA ? 3 : 4;   // K(p+3) / V(p+1) of this group's first softmax phase, p = 0 (A) or 1 (B)
    vpre_idx = grpA ? 1 : 2;
  }
  const unsigned char* kpre = kMulti ? nullptr : kb + kpre_idx * tileB;   // kMulti: looked up when the load is issued
  const unsigned char* vpre = kMulti ? nullptr : vb + vpre_idx * tileB;
  constexpr int kPreStep = kSplit ? 2 : 1;   // tiles between two softmax phases of a wave

  // Q^T operand (B of S^T = K Q^T): lane (r, g) holds Q[q0 + 16*nb + r][32*ks + 8*g .. +7]
  bf16x8 qreg[2][4];
  {
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int qi = min(q0 + 16 * nb + r, s.Sq - 1);
      const bf16_t* qr = qb + (int64_t)qi * s.qs[2] + 8 * g;
#pragma unroll
      for (int ks = 0; ks < kKS; ++ks) qreg[nb][ks] = *reinterpret_cast<const bf16x8*>(qr + 32 * ks);
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int ks = 0; ks < kKS; ++ks) asm volatile("" : "+v"(qreg[nb][ks]));
  }

  f32x4 sacc[4][2];   // scores: [16-key block mb][16-query block nb]: keys 16*mb + 4*g + i of query 16*nb + r
  u32x4 pk[2][2];     // bf16 P as the B operand of P.V: [32-key step kk][nb]: keys 32*kk + 16*(j >> 2) + 4*g + (j & 3), j = 0..7

  // per-lane LDS read addresses (see the layout notes at the top): 4 for the K operand (one per 32-wide
  // slice of the head dimension), 8 for the V^T operand (one per 16-wide slice); stage, key block
  // and row offsets are compile-time immediates on top of these
  typedef const __attribute__((address_space(3))) unsigned char* lds_cptr;
  lds_cptr k_rd[4], v_rd[8];
  {
    const int vrow = 4 * g + (r >> 2);          // the key this lane names in a transposing read (plus 32*kk, plus 16)
    if (!kHalfD) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        k_rd[ks] = (lds_cptr)(uintptr_t)(lds_base + r * RB + (((4 * ks + g) ^ r) << 4));
#pragma unroll
      for (int db = 0; db < 8; ++db)
        v_rd[db] = (lds_cptr)(uintptr_t)(lds_base + kStages * kTileB + vrow * RB + ((db ^ (vrow & 7)) << 5) + 8 * (r & 3));
    } else {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        k_rd[ks] = (lds_cptr)(uintptr_t)(lds_base + r * RB + ((((4 * ks + g) & 7) ^ ((r >> 1) & 7)) << 4));
#pragma unroll
      for (int db = 0; db < 8; ++db)
        v_rd[db] = (lds_cptr)(uintptr_t)(lds_base + kStages * kTileB + vrow * RB + (((db & 3) ^ ((vrow >> 1) & 3)) << 5) + 8 * (r & 3));
    }
  }
  // extended path: this lane's keys of a tile are rows 16*mb + 4*g + (0..3), mb = 0..3
  const lds_cptr x_rd = (lds_cptr)(uintptr_t)(lds_ext + 16 * g);

  // LDS operands.  K: keys 16*mb .. +15 (MFMA rows), head dims 32*ks + 8*g .. +7: one 16-byte read.
  // V^T: head dims 16*db .. +15 (MFMA rows), keys of step kk in the order of pk: two transposing reads of
  // four keys each (rows 32*kk + 4*g + i and 32*kk + 16 + 4*g + i).
  auto k_operand = [&](int stage, int mb, int ks) -> bf16x8 {
    return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(k_rd[ks] + stage * kTileB + 16 * mb * RB);
  };
  auto v_operand = [&](int stage, int kk, int db) -> bf16x8 {
    const u32x2 lo = lds_read_tr3(v_rd[db] + stage * kTileB + 32 * kk * RB);
    const u32x2 hi = lds_read_tr3(v_rd[db] + stage * kTileB + (32 * kk + 16) * RB);
    return __builtin_bit_cast(bf16x8, u32x4{lo[0], lo[1], hi[0], hi[1]});
  };
  const f32x4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
  // matrix phase: O += P V (V tile in stage sv) interleaved with the scores of the next tile (K in
  // stage sk), in four blocks of sixteen MFMAs: block b takes kNV V^T operands (key step b >> 1, head-dim
  // blocks kNV * (b & 1) ..) and kNV K operands (key block b, all head-dim slices), each operand feeding
  // two MFMAs (the wave's two 16-query blocks), so that consecutive MFMAs share their A operand.
  // Only this wave feeds the SIMD's matrix core during the phase, so its LDS operand reads run one
  // block ahead of their use.  The order is written out and pinned (sched_barrier after every operand's
  // MFMAs and the reads issued behind them) rather than left to the instruction scheduler.
  auto MM_full = [&](int sv, int sk) {
    __builtin_amdgcn_s_setprio(2);
    bf16x8 va[2][kNV], ka[2][kNV];
#pragma unroll
    for (int i = 0; i < kNV; ++i) va[0][i] = v_operand(sv, 0, i);
#pragma unroll
    for (int i = 0; i < kNV; ++i) ka[0][i] = k_operand(sk, 0, i);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      const int c = blk & 1, kk = blk >> 1;
      const bf16x8 pb0 = __builtin_bit_cast(bf16x8, pk[kk][0]), pb1 = __builtin_bit_cast(bf16x8, pk[kk][1]);
#pragma unroll
      for (int i = 0; i < kNV; i += kBurst) {
#pragma unroll
        for (int j = i; j < i + kBurst; ++j) {
          const int db = kNV * (blk & 1) + j;
          oacc[db][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[c][j], pb0, oacc[db][0], 0, 0, 0);
          oacc[db][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[c][j], pb1, oacc[db][1], 0, 0, 0);
        }
#pragma unroll
        for (int j = i; j < i + kBurst; ++j)
          if (blk < 3) va[c ^ 1][j] = v_operand(sv, (blk + 1) >> 1, kNV * ((blk + 1) & 1) + j);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < kNV; i += kBurst) {     // (kNV == kKS: the head-dim slices of the scores)
#pragma unroll
        for (int ks = i; ks < i + kBurst; ++ks) {
          sacc[blk][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[c][ks], qreg[0][ks], ks == 0 ? zero4 : sacc[blk][0], 0, 0, 0);
          sacc[blk][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[c][ks], qreg[1][ks], ks == 0 ? zero4 : sacc[blk][1], 0, 0, 0);
        }
#pragma unroll
        for (int ks = i; ks < i + kBurst; ++ks)
          if (blk < 3) ka[c ^ 1][ks] = k_operand(sk, blk + 1, ks);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __builtin_amdgcn_s_setprio(0);
  };
  auto MM_last = [&](int sv) {   // last tile: no further scores; the reads run two blocks ahead
    __builtin_amdgcn_s_setprio(2);
    bf16x8 va[4][kNV];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int i = 0; i < kNV; ++i) va[blk][i] = v_operand(sv, blk >> 1, kNV * (blk & 1) + i);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      const int kk = blk >> 1;
      const bf16x8 pb0 = __builtin_bit_cast(bf16x8, pk[kk][0]), pb1 = __builtin_bit_cast(bf16x8, pk[kk][1]);
#pragma unroll
      for (int i = 0; i < kNV; ++i) {
        const int db = kNV * (blk & 1) + i;
        oacc[db][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[blk][i], pb0, oacc[db][0], 0, 0, 0);
        oacc[db][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[blk][i], pb1, oacc[db][1], 0, 0, 0);
        if (blk < 2) va[blk + 2][i] = v_operand(sv, (blk + 2) >> 1, kNV * (blk & 1) + i);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __builtin_amdgcn_s_setprio(0);
  };
  // softmax phase: sacc (scores of one tile) -> pk (bf16 P), running references m and sums l of the
  // lane's two queries.
  // Fast path: exponentials are taken against the current reference m without first looking for
  // the tile's maximum; the row sum then certifies the result: if this lane's sum of P is at most
  // 2^60, no P exceeded 2^60, and neither l (at most 2^60 per key) nor O~ (at most 2^60 |v| per key)
  // leaves the fp32 range (2^127) over 2^20 keys with |v| up to 2^40; a reference that lags the
  // maximum by D only scales P, l and O~ by 2^D, which floating point carries without loss.  Only
  // when some lane fails that test (always on the first tile, where m = -inf makes every P inf)
  // does the wave find the true maximum, move m, rescale O and l, and redo the exponentials.
  // While it runs, the wave also issues its tile loads, spread between the exponential blocks so
  // that the waves do not hit the load path at once.
  // Extended path: the per-key factor c replaces the uniform scale, and in a tile with dead keys
  // their bias (-inf) is added to the exponent.
  auto x_vec = [&](int stage, int which, int mb) -> f32x4 {   // which: 0 c, 1 bias; keys 16*mb + 4*g + (0..3)
    return *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(
        x_rd + stage * kExtTileB + which * 256 + 64 * mb);
  };
  // c of the second key step is fetched while the first is computed
  f32x4 xc[2][2];
  auto x_load = [&](int kk, int xs) {
#pragma unroll
    for (int a = 0; a < 2; ++a) xc[kk][a] = x_vec(xs, 0, 2 * kk + a);
  };
  // one block: the 8 scores of query block nb over key step kk -> pk[kk][nb]
  auto exp_block = [&](int kk, int nb, float& psum, int xs, bool dead_keys, bool fetch_ahead) {
    float p[8];
    if (!kExt) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          p[4 * a + e] = __builtin_amdgcn_exp2f(fmaf(sacc[2 * kk + a][nb][e], scale2, -m[nb]));
          psum += p[4 * a + e];
        }
    } else {
      if (fetch_ahead && kk == 0 && nb == 1) x_load(1, xs);   // blocks run in the order (0,0) (0,1) (1,0) (1,1)
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        f32x4 t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = fmaf(sacc[2 * kk + a][nb][e], xc[kk][a][e], -m[nb]);
        if (dead_keys) {
          const f32x4 bias = x_vec(xs, 1, 2 * kk + a);
#pragma unroll
          for (int e = 0; e < 4; ++e) t[e] += bias[e];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          p[4 * a + e] = __builtin_amdgcn_exp2f(t[e]);
          psum += p[4 * a + e];
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) pk[kk][nb][j] = pack_bf16x2(p[2 * j], p[2 * j + 1]);
    // anchor the block here, between the tile loads that surround it in program order
    asm volatile("" : "+v"(pk[kk][nb]));
  };
  // largest exponent argument (before the reference is subtracted) of each of this lane's two queries over the tile
  auto tile_max = [&](int xs, float (&tmax)[2]) {
    tmax[0] = tmax[1] = -INFINITY;
    if (!kExt) {
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int e = 0; e < 4; ++e) tmax[nb] = fmaxf(tmax[nb], sacc[mb][nb][e]);
      tmax[0] = xgroup_max(tmax[0]) * scale2;
      tmax[1] = xgroup_max(tmax[1]) * scale2;
      return;
    }
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      const f32x4 c = x_vec(xs, 0, mb), bias = x_vec(xs, 1, mb);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int e = 0; e < 4; ++e) tmax[nb] = fmaxf(tmax[nb], fmaf(sacc[mb][nb][e], c[e], bias[e]));
    }
    tmax[0] = xgroup_max(tmax[0]);
    tmax[1] = xgroup_max(tmax[1]);
  };
  auto rescale = [&](int nb, float alpha) {   // O~ and l of query block nb
    lsum[nb] *= alpha;
#pragma unroll
    for (int db = 0; db < 8; ++db)
#pragma unroll
      for (int e = 0; e < 4; ++e) oacc[db][nb][e] *= alpha;
  };
  // Tiles still to be handled maximum-first (wave-uniform).  After a failed certification with a
  // reference already in place, the next kMaxFirstTiles softmax phases of the wave find the tile's
  // maximum before the exponentials and move the reference if it is outgrown by more than 2^8; every
  // such move re-arms the counter.  Scores with heavy tails then cost one maximum pass per tile
  // instead of a second round of exponentials on most tiles; ordinary scores never arm it.
  constexpr float kCertifiedSum = 1152921504606846976.0f;   // 2^60
  // A reference that moves is set this far ABOVE the maximum that moved it: the largest P is then 2^-32
  // instead of 1, which fp32 sums and bf16 P carry as well (every P, l and O~ is scaled by the same
  // power of two), and a later score has to exceed the maximum seen so far by 2^92, not 2^60, before
  // the reference has to move again.  With heavy-tailed scores (x20 outliers in Q and K) that is the
  // difference between a second round of exponentials on many tiles and on few.
  constexpr float kRefMargin = 32.0f;
  constexpr int kMaxFirstTiles = 8;
  int max_first = 0;
  // "some key of the tile is dead", read from the tile's record in global memory through the scalar
  // path (uniform address, written by an earlier launch) one softmax phase ahead of its use, so that
  // no softmax phase starts by waiting for it
  auto tile_flag = [&](int tile) -> float {
    typedef const __attribute__((address_space(4))) float* const_fptr;
    const float* p = s.ext + ((int64_t)bh_ * nt_all + min(tile, nt_all - 1)) * (kExtTileB / 4) + 128;
    return *(const_fptr)(uintptr_t)p;
  };
  // several chunks per launch: the records are written while the launch runs, so a tile's flag cannot
  // be fetched ahead from global memory; tiles of chunks that came with a key mask read it from their
  // record in LDS when the softmax phase starts (a short wait), tiles of other chunks skip it
  int sm_c = 0, sm_first = 0;   // chunk of sm_tile and the index of its first tile
  auto chunk_masked = [&](int tile) -> bool {
    while (sm_c + 1 < s.n_multi && tile >= sm_first + s.chunk[sm_c].Sc / kTile) {
      sm_first += s.chunk[sm_c].Sc / kTile;
      ++sm_c;
    }
    return s.chunk[sm_c].mask_src != nullptr;
  };
  int sm_tile = (kSplit && !grpA) ? 1 : 0;   // tile of this wave's next softmax phase
  float flag_next = 0.0f;
  // SM of the tile whose record sits in stage xs; loads K tile kpre_idx into stage sk (if do_k, with
  // the record of tile xpre_idx into stage xst if do_x) and V tile vpre_idx into stage sv (if do_v)
  auto SM = [&](int xs, int sk, int sv, bool do_k, bool do_v, bool do_x, int xpre_idx, int xst) {
    float psum[2] = {0.0f, 0.0f};
    bool dead_keys = false;
    if (kExt) x_load(0, xs);
    if (kExt && !kNoDead) {
      // this tile's flag was fetched during the wave's previous softmax phase; fetch the next one
      if (kMulti) {
        // a tile of a chunk that came with a mask: its flag, from the record in LDS
        if (chunk_masked(sm_tile)) {
          const float f = *reinterpret_cast<const __attribute__((address_space(3))) float*>(
              (lds_cptr)(uintptr_t)(lds_ext + xs * kExtTileB + 512));
          dead_keys = __builtin_amdgcn_readfirstlane(__float_as_uint(f)) != 0u;
        }
        sm_tile += kPreStep;
      } else {
        dead_keys = flag_next != 0.0f;
        sm_tile += kPreStep;
        flag_next = tile_flag(sm_tile);
      }
    }
    if (max_first > 0) {
      --max_first;
      float tmax[2];
      tile_max(xs, tmax);
      const bool jump0 = tmax[0] > m[0] + 8.0f, jump1 = tmax[1] > m[1] + 8.0f;
      if (__builtin_amdgcn_ballot_w64(jump0 || jump1) != 0ull) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          const bool jump = nb ? jump1 : jump0;
          const float m_new = tmax[nb] + kRefMargin;
          const float alpha = jump ? __builtin_amdgcn_exp2f(m[nb] - m_new) : 1.0f;   // m = -inf gives 0
          m[nb] = jump ? m_new : m[nb];
          rescale(nb, alpha);
        }
        max_first = kMaxFirstTiles;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (kMulti) {
      if (do_k) kpre = tile_at(kcur, kpre_idx, false);
      if (do_v) vpre = tile_at(vcur, vpre_idx, true);
    }
    // sched_barrier: keep each load between two blocks of arithmetic (the scheduler would
    // otherwise hoist all of them to the top, where they queue behind one another)
    if (!kSplit) {
      if (do_k) issue_k_half(kpre, kpre_idx, sk, 0, false);
      exp_block(0, 0, psum[0], xs, dead_keys, true);
      __builtin_amdgcn_sched_barrier(0);
      if (do_k) issue_k_half(kpre, kpre_idx, sk, 1, false);
      exp_block(0, 1, psum[1], xs, dead_keys, true);
      __builtin_amdgcn_sched_barrier(0);
      if (do_v) issue_v_half(vpre, vpre_idx, sv, 0, false);
      exp_block(1, 0, psum[0], xs, dead_keys, true);
      __builtin_amdgcn_sched_barrier(0);
      if (do_v) issue_v_half(vpre, vpre_idx, sv, 1, false);
      if (kExt && do_x) issue_ext(xpre_idx, xst);
      exp_block(1, 1, psum[1], xs, dead_keys, true);
      __builtin_amdgcn_sched_barrier(0);
    } else {
      if (do_v) { issue_v_half(vpre, vpre_idx, sv, 0, false); issue_v_half(vpre, vpre_idx, sv, 0, true); }
      exp_block(0, 0, psum[0], xs, dead_keys, true);
      __builtin_amdgcn_sched_barrier(0);
      if (do_v) { issue_v_half(vpre, vpre_idx, sv, 1, false); issue_v_half(vpre, vpre_idx, sv, 1, true); }
      exp_block(0, 1, psum[1], xs, dead_keys, true);
      __builtin_amdgcn_sched_barrier(0);
      if (do_k) { issue_k_half(kpre, kpre_idx, sk, 0, false); issue_k_half(kpre, kpre_idx, sk, 0, true); }
      exp_block(1, 0, psum[0], xs, dead_keys, true);
      __builtin_amdgcn_sched_barrier(0);
      if (do_k) { issue_k_half(kpre, kpre_idx, sk, 1, false); issue_k_half(kpre, kpre_idx, sk, 1, true); }
      if (kExt && do_x) issue_ext(xpre_idx, xst);
      exp_block(1, 1, psum[1], xs, dead_keys, true);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (!kMulti) { kpre += kPreStep * tileB; vpre += kPreStep * tileB; }
    kpre_idx += kPreStep;
    vpre_idx += kPreStep;
    // (per query block: a block all of whose lanes passed keeps its exponentials and its reference)
    const bool redo0 = __builtin_amdgcn_ballot_w64(!(psum[0] <= kCertifiedSum)) != 0ull;
    const bool redo1 = __builtin_amdgcn_ballot_w64(!(psum[1] <= kCertifiedSum)) != 0ull;
    if (redo0 || redo1) {
      // a reference that was already set and still failed: scores with heavy tails; look for the
      // maximum first on the next tiles instead of paying for the exponentials twice
      if (__builtin_amdgcn_ballot_w64(m[0] != -INFINITY || m[1] != -INFINITY) != 0ull) max_first = kMaxFirstTiles;
      float tmax[2];
      tile_max(xs, tmax);
      if (kExt) { x_load(0, xs); x_load(1, xs); }
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        if (!(nb ? redo1 : redo0)) continue;
        const float m_new = tmax[nb] > m[nb] ? tmax[nb] + kRefMargin : m[nb];
        // m = -inf (first live tile) gives alpha 0; no live key so far: nothing to rescale, P = 0
        const float alpha = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m[nb] - m_new);
        m[nb] = m_new;
        rescale(nb, alpha);
        psum[nb] = 0.0f;
        if (kExt && m_new == -INFINITY) {
          pk[0][nb] = u32x4{0u, 0u, 0u, 0u};
          pk[1][nb] = u32x4{0u, 0u, 0u, 0u};
        } else {
          exp_block(0, nb, psum[nb], xs, dead_keys, false);
          exp_block(1, nb, psum[nb], xs, dead_keys, false);
        }
      }
    }
    lsum[0] += psum[0];
    lsum[1] += psum[1];
    // pin the results here: without a use in this phase the optimiser sinks the exponentials past
    // the barrier, next to their first use in the matrix phase
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) asm volatile("" : "+v"(pk[kk][nb]));
    asm volatile("" : "+v"(lsum[0]), "+v"(lsum[1]));
  };
  auto nxt = [](int x) { return x == 2 ? 0 : x + 1; };
  if (kExt && !kNoDead && !kMulti) flag_next = tile_flag(sm_tile);
  auto first_scores = [&](int stage) {
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      sacc[mb][0] = zero4;
      sacc[mb][1] = zero4;
#pragma unroll
      for (int ks = 0; ks < kKS; ++ks) {
        const bf16x8 a = k_operand(stage, mb, ks);
        sacc[mb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qreg[0][ks], sacc[mb][0], 0, 0, 0);
        sacc[mb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qreg[1][ks], sacc[mb][1], 0, 0, 0);
      }
    }
  };

  // prologue: the first tiles have landed
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  __builtin_amdgcn_s_barrier();

  if (!kSplit) {
    first_scores(0);   // scores of tile 0 in both groups
    // Both groups execute the same barrier sequence (two per tile index j = 0..nt); the steady-state
    // bodies are straight-line code so the accumulators stay in place.
    // sched_barrier(0): nothing may be moved across a phase boundary (the compiler would otherwise
    // sink the softmax arithmetic below the barrier, into the matrix phase of the same wave).
    // A wave waits for its own tile loads at the end of its softmax phases: the batch issued one
    // softmax phase earlier must have landed, the batch just issued (if full: 4 loads, 5 with a
    // record) may be in flight.
    // Only the barrier in front of A's matrix phase / B's softmax phase is needed (the other phase
    // boundaries pass needed = false and only order the instruction stream): with
    // three stages no load of the half-period after it overwrites what that half-period or the one
    // before the next barrier still reads, and every tile is waited for by its loaders before the
    // barrier in front of its first reader.  The second barrier only kept the groups in step, which
    // equal phase lengths do by themselves.  The key records are read in the softmax phases of both
    // halves, so they go round four stages (tile j in stage j % 4): record j+2 then replaces record
    // j-2, last read in phase 2j-3, in phase 2j, with the barrier of tile j-1 between the two.
    auto phase_barrier = [&](int wait_mode, bool needed = true) {   // 0: no wait, 1: all but the last full batch, 2: vmcnt(0)
      __builtin_amdgcn_sched_barrier(0);
      if (wait_mode == 1) {
        // a full batch is 4 loads (2 with 128-byte rows), plus the record's in the group that loads it
        if (kExt && grpA) __builtin_amdgcn_s_waitcnt(kHalfD ? 0x0F73 : 0x0F75);   // vmcnt(3) / vmcnt(5)
        else __builtin_amdgcn_s_waitcnt(kHalfD ? 0x0F72 : 0x0F74);                // vmcnt(2) / vmcnt(4)
      } else if (wait_mode == 2) __builtin_amdgcn_s_waitcnt(0x0F70);
      if (needed) __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
    };
    int st = 0;                            // LDS stage of tile j, j % 3
    if (grpA) {
      // tile j: phase 2j = SM(j), prefetching K(j+2) and its record -> stage st+2, V(j+1) -> stage st+1;
      //         phase 2j+1 = MM(j) with V(j) in stage st, K(j+1) in stage st+1
      for (int j = 0; j < nt - 1; ++j) {
        const int s1 = nxt(st), s2 = nxt(s1);
        SM(j & 3, s2, s1, j + 2 < nt, true, j + 2 < nt, j + 2, (j + 2) & 3);
        phase_barrier(j + 2 < nt ? 1 : 2);
        MM_full(st, s1);
        phase_barrier(0, false);
        st = s1;
      }
      SM((nt - 1) & 3, 0, 0, false, false, false, 0, 0);
      phase_barrier(2);
      MM_last(st);
      phase_barrier(0, false);
      phase_barrier(0);
      phase_barrier(0, false);
    } else {
      // tile j: phase 2j = MM(j-1) with V(j-1) in stage st-1, K(j) in stage st;
      //         phase 2j+1 = SM(j), prefetching K(j+3) -> stage st, V(j+2) -> stage st+2
      phase_barrier(0);                                 // phase 0: nothing to do yet
      SM(0, 0, 2, 3 < nt, 2 < nt, false, 0, 0);         // phase 1 (tile 0)
      phase_barrier(3 < nt ? 1 : 2, false);
      for (int j = 1; j < nt; ++j) {
        const int sp = st;                              // stage of tile j-1
        st = nxt(st);
        MM_full(sp, st);
        phase_barrier(0);
        SM(j & 3, st, sp, j + 3 < nt, j + 2 < nt, false, 0, 0);   // st+2 == sp (mod 3)
        phase_barrier(j + 3 < nt ? 1 : 2, false);
      }
      MM_last(st);
      phase_barrier(0);
      phase_barrier(0, false);
    }
  } else {
    // scores of tile 0 (group A) / tile 1 (group B)
    if (grpA || nt > 1) first_scores(grpA ? 0 : 1);
    // Phases p = 0..nt, one work-group barrier each; both groups execute nt + 1 of them.
    //   reads in phase p : V(p-1) from stage (p-1)%3, K(p+1) from stage (p+1)%3, record p from p%3
    //   batch of phase p : K(p+3) -> stage p%3 (last read, as K(p), in phase p-1),
    //                      V(p+1) -> stage (p+1)%3 (last read, as V(p-2), in phase p-1),
    //                      record p+2 -> stage (p+2)%3 (last read, as record p-1, in phase p-1)
    //   end of phase p   : the batch of phase p-1 must have landed (first read in phase p+1); its
    //                      issuers are the group now ending a matrix phase, which waits for all of
    //                      its loads; the other group has only this phase's batch in flight
    auto end_phase = [&](bool wait_loads) {
      __builtin_amdgcn_sched_barrier(0);
      if (wait_loads) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
    };
    int t = grpA ? 0 : 1;                  // this group's current tile; SM(t) runs in phase t
    int st = t;                            // t % 3
    if (!grpA) end_phase(false);           // phase 0: group B has no scores yet
    while (t + 2 < nt) {
      const int s1 = nxt(st), s2 = nxt(s1);                // (t + 1) % 3, (t + 2) % 3
      SM(st, st, s1, t + 3 < nt, true, true, t + 2, s2);   // phase t (t + 1 < nt holds here)
      end_phase(false);
      MM_full(st, s2);                                     // phase t + 1
      end_phase(true);
      t += 2;
      st = s2;
    }
    if (t < nt) {                                          // this group's last tile
      SM(st, st, nxt(st), false, t + 1 < nt, false, 0, 0);
      end_phase(false);
      MM_last(st);
      end_phase(true);
      t += 2;
    }
    // the group whose last matrix phase was phase nt-1 sits out phase nt
    if ((grpA && (nt % 2 == 0)) || (!grpA && (nt % 2 == 1))) end_phase(false);
  }
  }  // nt > 0
  // A wave that gave up waiting for a chunk loaded its rows of the tiles too early, and every wave of
  // the work-group has read those rows: the flag belongs to the work-group.
  if (kMulti) {
    if (s.arrive != nullptr) late = __syncthreads_or(late ? 1 : 0) != 0;
  }

  if (kSplit) {
    // ---- fold group B's partial state into group A's (same queries, disjoint keys) --------------
    // all tile reads are behind the last barrier, so the tile buffers are reused for the exchange:
    // float slot i of wave w, lane l sits at x[(w * 66 + i) * 64 + l]
    float* xch = reinterpret_cast<float*>(smem_raw);
    constexpr int kSlots = 8 * 2 * 4 + 4;   // O~, the two references, the two sums
    if (!grpA) {
      float* dst = xch + ((wave - 4) * kSlots) * 64 + lane;
#pragma unroll
      for (int db = 0; db < kDB; ++db)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int e = 0; e < 4; ++e) dst[((db * 2 + nb) * 4 + e) * 64] = oacc[db][nb][e];
      dst[64 * 64] = m[0]; dst[65 * 64] = m[1];
      dst[66 * 64] = lsum[0]; dst[67 * 64] = lsum[1];
    }
    __syncthreads();
    if (!grpA) return;
    const float* src = xch + (wave * kSlots) * 64 + lane;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const float mB = src[(64 + nb) * 64], lB = src[(66 + nb) * 64];
      const float mm = fmaxf(m[nb], mB);
      const float wa = (mm == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(m[nb] - mm);
      const float wb = (mm == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mB - mm);
#pragma unroll
      for (int db = 0; db < kDB; ++db)
#pragma unroll
        for (int e = 0; e < 4; ++e) oacc[db][nb][e] = wa * oacc[db][nb][e] + wb * src[((db * 2 + nb) * 4 + e) * 64];
      lsum[nb] = wa * lsum[nb] + wb * lB;
      m[nb] = mm;
    }
  }

  // every tile read of the work-group is behind a barrier here (the one after the last matrix phase)
  if (kSplit) finish_and_store_direct<kHalfD>(s, oacc, m, lsum, b, h, q0, r, g, kMulti && late);
  else finish_and_store<kHalfD>(s, oacc, m, lsum, b, h, q0, r, g, smem_raw + wave * kEpiWaveB, kMulti && late);
}

template <bool kSplit, bool kExt, bool kMulti = false, bool kNoDead = false, bool kHalfD = false>
__global__ __launch_bounds__(kThreads, 2) void attn_pp_kernel(AttnStep s) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  if (!kMulti && s.copy_wgs > 0 && blockIdx.x >= gridDim.x - s.copy_wgs) {   // prefetch work-group: copy and leave
    prefetch_copy(s, blockIdx.x - (gridDim.x - s.copy_wgs), threadIdx.x, kThreads);
    return;
  }
  constexpr int kQBlock = kSplit ? kQPerWGSplit : kQPerWG;
  int bh_, qb_;
  int lead = 0;
  if (kMulti && s.arrive != nullptr) {   // the whole ring's transfers ride in this launch, in its first work-groups
    if ((int)blockIdx.x < s.copy_wgs) {
      if (kExt && s.multi_fp8) stream_chunks_fp8(s, blockIdx.x, threadIdx.x, kThreads);
      else stream_chunks(s, blockIdx.x, threadIdx.x, kThreads);   // bf16 chunks (their records, if any, were written before the launch)
      return;
    }
    lead = s.copy_wgs;
  }
  if (!wg_to_tile(s.copy_wgs, (s.Sq + kQBlock - 1) / kQBlock, s.B * s.H, bh_, qb_, lead)) return;   // whole work-group
  attn_pp_body<kSplit, kExt, kMulti, kNoDead, kHalfD>(s, smem_raw, bh_, qb_ * kQBlock);
}

// Mixed launch: when the 256-query blocks do not fill the last round of work-groups on the 256 CUs
// (one work-group per CU at a time), the blocks of that round are run as two key-split work-groups
// of 128 queries each, which take about 0.55 of a wide work-group's time.  Per XCD (ids go round
// robin) the contiguous, head-major range of blocks is dispatched wide blocks first, then the
// halves of its last s.mix_halves blocks.
template <bool kExt>
__global__ __launch_bounds__(kThreads, 2) void attn_pp_mixed_kernel(AttnStep s) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  if (s.copy_wgs > 0 && blockIdx.x >= gridDim.x - s.copy_wgs) {
    prefetch_copy(s, blockIdx.x - (gridDim.x - s.copy_wgs), threadIdx.x, kThreads);
    return;
  }
  const int nqb = (s.Sq + kQPerWG - 1) / kQPerWG;
  const int items = nqb * s.B * s.H;
  const int per = (items + kXcds - 1) / kXcds;
  const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  const int first = xcd * per;
  const int count = min(per, items - first);          // blocks of this XCD (may be <= 0 on the last ones)
  const int halves = min(s.mix_halves, count);
  const int wide = count - halves;
  if (slot < wide) {
    const int item = first + slot;
    const int bh_ = item / nqb;
    attn_pp_body<false, kExt>(s, smem_raw, bh_, (item - bh_ * nqb) * kQPerWG);
  } else {
    const int hs = slot - wide;
    if (hs >= 2 * halves) return;
    const int item = first + wide + (hs >> 1);
    const int bh_ = item / nqb;
    const int q_base = (item - bh_ * nqb) * kQPerWG + (hs & 1) * kQPerWGSplit;
    if (q_base >= s.Sq) return;                        // second half of a ragged last block
    attn_pp_body<true, kExt>(s, smem_raw, bh_, q_base);
  }
}

}  // namespace

bool attn_mfma_supported(const AttnStep& s) {
  return s.qo_dtype == USP_BF16 && s.kv_dtype == USP_BF16 && (s.d == kD || (s.d == 64 && s.half_d)) && s.Sq > 0;
}

size_t attn_mfma_ext_bytes(int B, int H, int Sc) {
  const size_t nt_all = (size_t)(Sc + kTile - 1) / kTile;
  return (size_t)B * H * nt_all * kExtTileB;
}

bool attn_mfma_needs_ext(const AttnStep& s) {
  return !(s.Sc > 0 && s.Sc % kTile == 0 && !s.key_mask && !s.k_scale);
}

usp_status launch_attn_ext_prepare(const AttnStep& s, hipStream_t st) {
  const unsigned nt_all = (unsigned)((s.Sc + kTile - 1) / kTile);
  hipLaunchKernelGGL(attn_ext_prepare_kernel, dim3(nt_all > 0 ? nt_all : 1, (unsigned)(s.B * s.H)), dim3(64), 0, st,
                     s, s.ext, s.n_live);
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

usp_status launch_attn_fp8_chunk_prepare(const AttnStep& s, int c, bool reset_arrive, hipStream_t st) {
  if (!s.multi_fp8 || c < 0 || c >= s.n_multi || !s.ext || (reset_arrive && !s.arrive)) {
    set_error("FP8 chunk preparation needs a step over several FP8 chunks with its records");
    return USP_ERR_INVALID_ARG;
  }
  const int64_t units = (int64_t)s.B * s.H * s.chunk[c].Sc * (s.d / 16);   // 16 codes each
  const int64_t blocks = (units + 255) / 256;                          // one unit per thread while the chunk is small
  hipLaunchKernelGGL(attn_fp8_chunk_prepare_kernel, dim3((unsigned)(blocks < 1 ? 1 : blocks > 8192 ? 8192 : blocks)), dim3(256),
                     0, st, s, c, reset_arrive ? 1 : 0);
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

usp_status launch_attn_fp8_step_prepare(const AttnStep& s, int* n_live, hipStream_t st) {
  if (!s.multi_fp8 || s.n_multi != 1 || !s.ext || !n_live || s.chunk[0].Sc <= 0 || s.chunk[0].Sc % kTile != 0) {
    set_error("FP8 step preparation needs one FP8 chunk of whole tiles with room for its records");
    return USP_ERR_INVALID_ARG;
  }
  const int64_t units = (int64_t)s.B * s.H * s.chunk[0].Sc * (s.d / 16);   // 16 codes each
  const int64_t blocks = (units + 255) / 256;
  hipLaunchKernelGGL(attn_fp8_step_prepare_kernel, dim3((unsigned)(blocks < 1 ? 1 : blocks > 8192 ? 8192 : blocks)), dim3(256),
                     0, st, s, n_live);
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

usp_status launch_attn_multi_records(const AttnStep& s, hipStream_t st) {
  int nt_total = 0;
  for (int c = 0; c < s.n_multi; ++c) {
    if (s.chunk[c].Sc <= 0 || s.chunk[c].Sc % kTile != 0) {
      set_error("records of a launch over several chunks need chunk lengths that are positive multiples of %d", kTile);
      return USP_ERR_INVALID_ARG;
    }
    nt_total += s.chunk[c].Sc / kTile;
  }
  if (s.n_multi <= 0 || s.n_multi > AttnStep::kMaxMulti || !s.ext || s.multi_fp8) {
    set_error("records of a launch over several bf16 chunks need the chunks and room for the records");
    return USP_ERR_INVALID_ARG;
  }
  hipLaunchKernelGGL(attn_multi_records_kernel, dim3((unsigned)nt_total, (unsigned)(s.B * s.H)), dim3(64), 0, st, s);
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

usp_status launch_attn_arrive_reset(int* arrive, hipStream_t st) {
  hipLaunchKernelGGL(attn_arrive_reset_kernel, dim3(1), dim3(64), 0, st, arrive);
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}

namespace {
// More than 64 KB of dynamic LDS has to be allowed per kernel, and the setting belongs to the device
// that is current when it is made: once per (kernel, device ordinal below 64), every launch beyond.
template <void (*kKernel)(AttnStep)>
hipError_t allow_large_lds(int bytes) {
  static std::atomic<uint64_t> done{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < 64;
  if (tracked && ((done.load(std::memory_order_acquire) >> dev) & 1u) != 0) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(kKernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && tracked) done.fetch_or((uint64_t)1 << dev, std::memory_order_release);
  return e;
}
template <bool kSplit, bool kExt, bool kMulti = false, bool kNoDead = false, bool kHalfD = false>
usp_status launch_pp_d(const AttnStep& s, unsigned wgs, hipStream_t st) {
  static_assert(kLdsBytes >= (int)sizeof(SmemPPExt) && kLdsBytes <= 160 * 1024, "LDS plan");
  constexpr int lds = kLdsBytes;
  USP_CHECK_HIP((allow_large_lds<attn_pp_kernel<kSplit, kExt, kMulti, kNoDead, kHalfD>>(lds)));
  hipLaunchKernelGGL((attn_pp_kernel<kSplit, kExt, kMulti, kNoDead, kHalfD>), dim3(wgs + s.copy_wgs), dim3(kThreads), lds, st, s);
  USP_CHECK_HIP(hipGetLastError());
  return USP_OK;
}
template <bool kSplit, bool kExt, bool kMulti = false, bool kNoDead = false>
usp_status launch_pp(const AttnStep& s, unsigned wgs, hipStream_t st) {
  return s.half_d ? launch_pp_d<kSplit, kExt, kMulti, kNoDead, true>(s, wgs, st)
                  : launch_pp_d<kSplit, kExt, kMulti, kNoDead, false>(s, wgs, st);
}
}  // namespace

usp_status launch_attn_mfma(const AttnStep& step, hipStream_t st) {
  AttnStep s = step;
  if (s.n_multi > 0) {
    // several resident chunks, one launch: the same two work decompositions, by the same rule
    if (s.n_multi > AttnStep::kMaxMulti || s.mode != 0 || s.n_copy != 0 || s.key_mask || s.k_scale || s.v_scale) {   // (n_copy: the per-step form of the transfers)
      set_error("a launch over several chunks takes at most %d unmasked chunks and finishes the result", AttnStep::kMaxMulti);
      return USP_ERR_INVALID_ARG;
    }
    if (s.multi_fp8 && (!s.arrive || !s.ext)) {
      set_error("a launch over several FP8 chunks needs arrival counters and per-tile records");
      return USP_ERR_INVALID_ARG;
    }
    if (!s.multi_fp8 && s.multi_masked && !s.ext) {
      set_error("a launch over several chunks with key masks needs their per-tile records");
      return USP_ERR_INVALID_ARG;
    }
    for (int c = 0; c < s.n_multi; ++c)
      if (s.chunk[c].Sc <= 0 || s.chunk[c].Sc % kTile != 0 || !s.chunk[c].k || !s.chunk[c].v) {
        set_error("a launch over several chunks needs chunk lengths that are positive multiples of %d", kTile);
        return USP_ERR_INVALID_ARG;
      }
    const unsigned w256 = wg_grid_size((s.Sq + kQPerWG - 1) / kQPerWG, s.B * s.H);
    const unsigned w128 = wg_grid_size((s.Sq + kQPerWGSplit - 1) / kQPerWGSplit, s.B * s.H);
    // There is no mixed form of this launch: between the two decompositions, take the one whose
    // rounds of work-groups over the 256 CUs cost less (a key-split work-group takes about 0.55 of a
    // 256-query one)
    const double cost256 = (double)((w256 + 255) / 256), cost128 = 0.55 * (double)((w128 + 255) / 256);
    const bool split = s.variant == 2 || (s.variant != 1 && ((int)w256 <= kSplitBelowWGs || cost128 < cost256));
    const unsigned wgs = split ? w128 : w256;
    s.copy_wgs = 0;
    if (s.arrive != nullptr) {
      for (int c = s.multi_fp8 ? 0 : 1; c < s.n_multi; ++c)
        if (!s.chunk[c].k_src || !s.chunk[c].v_src || s.chunk[c].bytes <= 0 || s.chunk[c].bytes % 16 != 0 ||
            !aligned16(s.chunk[c].k_src) || !aligned16(s.chunk[c].v_src) || !aligned16(s.chunk[c].k) || !aligned16(s.chunk[c].v) ||
            (s.multi_fp8 && (!s.chunk[c].k_scale_src || !s.chunk[c].v_scale_src || !aligned16(s.chunk[c].k_scale_src) ||
                             ((uintptr_t)s.chunk[c].mask_src & 3u) != 0))) {
          set_error("transfers inside a launch over several chunks need 16-byte aligned sources and buffers");
          return USP_ERR_INVALID_ARG;
        }
      s.n_copy = 1;                                    // (only asks prefetch_wg_count for a count)
      s.copy_wgs = prefetch_wg_count(s, (int)wgs, 1);
      s.n_copy = 0;
      s.arrive_need = s.copy_wgs + (s.arrive_need_extra > 0 ? s.arrive_need_extra : 0);
      if (s.arrive_polls <= 0 || s.arrive_polls > kArrivePolls) s.arrive_polls = kArrivePolls;
    }
    if (s.multi_fp8 && s.multi_masked)
      return split ? launch_pp<true, true, true, false>(s, wgs, st) : launch_pp<false, true, true, false>(s, wgs, st);
    if (s.multi_fp8) return split ? launch_pp<true, true, true, true>(s, wgs, st) : launch_pp<false, true, true, true>(s, wgs, st);
    if (s.multi_masked)   // bf16 chunks, records written by launch_attn_multi_records
      return split ? launch_pp<true, true, true, false>(s, wgs, st) : launch_pp<false, true, true, false>(s, wgs, st);
    if (split) return launch_pp<true, false, true>(s, wgs, st);
    return launch_pp<false, false, true>(s, wgs, st);
  }
  const bool ext = attn_mfma_needs_ext(s);
  // Few query blocks (a small Q shard of a ring step): 256-query work-groups would leave CUs idle;
  // 128-query work-groups whose two wave groups split the keys fill twice as many.
  const unsigned wgs256 = wg_grid_size((s.Sq + kQPerWG - 1) / kQPerWG, s.B * s.H);
  const bool split = s.variant == 2 || (s.variant == 0 && (int)wgs256 <= kSplitBelowWGs);
  if (ext && (s.ext == nullptr || s.n_live == nullptr)) {
    set_error("attention step with a key mask, FP8 scales or a ragged chunk needs its per-tile records");
    return USP_ERR_INVALID_ARG;
  }
  if (s.v_scale != nullptr) {
    set_error("the bf16 matrix-core kernels take V already multiplied by its scales");
    return USP_ERR_INVALID_ARG;
  }
  // Mixed launch when the last round of 256-query work-groups would be at most half full
  const int items = (int)((s.Sq + kQPerWG - 1) / kQPerWG) * s.B * s.H;
  const int rem = items % 256;
  int mix_blocks = 0;
  if (s.half_d) mix_blocks = 0;                                           // (the mixed kernel has no half-head-dimension form)
  else if (s.variant == 4) mix_blocks = (items + 1) / 2;                  // forced: the second half of the blocks
  else if (s.variant == 0 && !split && rem > 0 && rem <= 128) mix_blocks = rem;
  if (mix_blocks > 0) {
    s.mix_halves = (mix_blocks + kXcds - 1) / kXcds;
    const int per = (items + kXcds - 1) / kXcds;
    const unsigned wgs_mixed = (unsigned)(kXcds * (per + s.mix_halves));
    s.copy_wgs = prefetch_wg_count(s, (int)wgs_mixed, 1);
    constexpr int lds = kLdsBytes;
    if (ext) {
      USP_CHECK_HIP(allow_large_lds<attn_pp_mixed_kernel<true>>(lds));
      hipLaunchKernelGGL((attn_pp_mixed_kernel<true>), dim3(wgs_mixed + s.copy_wgs), dim3(kThreads), lds, st, s);
    } else {
      USP_CHECK_HIP(allow_large_lds<attn_pp_mixed_kernel<false>>(lds));
      hipLaunchKernelGGL((attn_pp_mixed_kernel<false>), dim3(wgs_mixed + s.copy_wgs), dim3(kThreads), lds, st, s);
    }
    USP_CHECK_HIP(hipGetLastError());
    return USP_OK;
  }
  const unsigned wgs = split ? wg_grid_size((s.Sq + kQPerWGSplit - 1) / kQPerWGSplit, s.B * s.H) : wgs256;
  s.copy_wgs = prefetch_wg_count(s, (int)wgs, 1);
  // records only because of FP8 scales: no key is dead
  if (ext && !s.key_mask && s.Sc % kTile == 0)
    return split ? launch_pp<true, true, false, true>(s, wgs, st) : launch_pp<false, true, false, true>(s, wgs, st);
  if (split) return ext ? launch_pp<true, true>(s, wgs, st) : launch_pp<true, false>(s, wgs, st);
  return ext ? launch_pp<false, true>(s, wgs, st) : launch_pp<false, false>(s, wgs, st);
}

}  // namespace usp
