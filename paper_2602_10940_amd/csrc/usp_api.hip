// C ABI entry points: argument validation, workspace carving, and the stream / event
// schedule of pipelined ring attention (FastUSP Algorithm 2).  No device memory is
// allocated here and the host never blocks.
#include <mutex>
#include <vector>
#include <math.h>
#include <string.h>

#include "usp_common.h"

namespace usp {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
void clear_error() { g_err[0] = 0; }

namespace {

size_t elt_size(int dt) { return dt == USP_F32 ? 4 : dt == USP_BF16 ? 2 : 1; }
size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Per-thread, per-device pool of timing-free events used to order the two streams.
struct EventPool {
  int device = -1;
  std::vector<hipEvent_t> ev;
  size_t next = 0;
  hipError_t get(hipEvent_t* out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev != device) { ev.clear(); next = 0; device = dev; }  // events of another device are abandoned
    if (ev.size() < 64) {
      hipEvent_t x;
      e = hipEventCreateWithFlags(&x, hipEventDisableTiming | hipEventReleaseToDevice);
      if (e != hipSuccess) return e;
      ev.push_back(x);
      *out = x;
      return hipSuccess;
    }
    *out = ev[next++ % ev.size()];
    return hipSuccess;
  }
};
thread_local EventPool g_events;

struct Plan {
  bool valid = false;
  int W = 0;
  int max_len = 0;
  bool fp8 = false, dbuf = false, unfused = false, mfma = false, dequant_stage = false;
  bool fused_pf = false;      // dbuf with the transfers riding in the attention launches
  size_t rows_q = 0;          // B*H*Sq
  size_t off_acc = 0;         // fp32 carried O            (fused, W > 1)
  size_t off_tmp_o = 0;       // per-chunk O_i             (unfused, W > 1)
  size_t off_tmp_lse = 0;     // per-chunk lse_i           (unfused, W > 1)
  size_t off_buf[2] = {0, 0}; // staged chunk: K | V | k_scale | v_scale
  size_t buf_k = 0, buf_v = 0, buf_ks = 0, buf_vs = 0;  // offsets inside a staging buffer
  size_t off_deq_k = 0, off_deq_v = 0;  // bf16 K/V after dequantisation (FP8 + MFMA kernel)
  size_t off_ext = 0, off_nlive = 0;    // per-tile key records and live tile counts (MFMA kernel, masks / scales / ragged chunks)
  bool ring1 = false;                   // fused prefetch as one launch over the whole ring: a staging buffer per chunk
  size_t off_ring1 = 0, off_arrive = 0; // K | V of chunk 1, K | V of chunk 2, ... (dense, 256-byte aligned each); arrival counters
  bool ring8 = false;                   // FP8 chunks decoded inside one launch over the whole ring
  size_t off_ring8 = 0, off_ext8 = 0;   // bf16 K | V of every live chunk; records of all their tiles
  bool ext = false;
  bool multi_rec = false;               // room for the records of a one-launch ring over bf16 chunks with key masks
  size_t off_multi_rec = 0;
  size_t total = 0;
};

bool kv_auto(const usp_attn_desc* d) {  // all-zero kv_stride: every chunk is dense for its own length
  return d->kv_stride[0] == 0 && d->kv_stride[1] == 0 && d->kv_stride[2] == 0;
}
bool kv_dense(const usp_attn_desc* d, int len) {
  if (kv_auto(d)) return true;
  return d->kv_stride[2] == d->d && d->kv_stride[1] == (int64_t)len * d->d &&
         d->kv_stride[0] == (int64_t)d->H * len * d->d;
}
bool o_dense(const usp_attn_desc* d) {
  return d->o_stride[2] == d->d && d->o_stride[1] == (int64_t)d->Sq * d->d &&
         d->o_stride[0] == (int64_t)d->H * d->Sq * d->d;
}

usp_status make_plan(const usp_attn_desc* d, Plan* p) {
  USP_CHECK_ARG(d != nullptr, "desc is NULL");
  USP_CHECK_ARG(d->B > 0 && d->H > 0 && d->Sq > 0, "B, H, Sq must be positive (B=%d H=%d Sq=%d)", d->B, d->H, d->Sq);
  USP_CHECK_ARG(d->d > 0 && d->d % 8 == 0 && d->d <= 256, "d must be a multiple of 8 in [8, 256] (got %d)", d->d);
  // launch grids: (batch, head) pairs ride in a 16-bit grid dimension, query blocks times pairs in a 32-bit one
  USP_CHECK_ARG((int64_t)d->B * d->H <= 65535, "B*H=%lld exceeds 65535", (long long)d->B * d->H);
  USP_CHECK_ARG((int64_t)d->B * d->H * d->Sq < ((int64_t)1 << 37), "B*H*Sq=%lld is too large", (long long)d->B * d->H * d->Sq);
  USP_CHECK_ARG(d->n_chunks >= 1 && d->chunk_len != nullptr, "n_chunks must be >= 1 with chunk_len set");
  USP_CHECK_ARG(d->qo_dtype == USP_F32 || d->qo_dtype == USP_BF16, "qo_dtype must be USP_F32 or USP_BF16");
  USP_CHECK_ARG(d->kv_dtype == d->qo_dtype || d->kv_dtype == USP_FP8_E4M3FN,
                "kv_dtype must equal qo_dtype or be USP_FP8_E4M3FN");
  USP_CHECK_ARG(d->softmax_scale >= 0.0f && isfinite(d->softmax_scale), "softmax_scale must be finite and >= 0");
  const int64_t al = d->qo_dtype == USP_F32 ? 4 : 8;
  for (int i = 0; i < 3; ++i) {
    USP_CHECK_ARG(d->q_stride[i] >= 0 && d->q_stride[i] % al == 0, "q_stride[%d]=%lld must be a non-negative multiple of %lld", i, (long long)d->q_stride[i], (long long)al);
    USP_CHECK_ARG(d->o_stride[i] >= 0 && d->o_stride[i] % al == 0, "o_stride[%d]=%lld must be a non-negative multiple of %lld", i, (long long)d->o_stride[i], (long long)al);
    const int64_t kal = d->kv_dtype == USP_F32 ? 4 : d->kv_dtype == USP_BF16 ? 8 : 16;
    USP_CHECK_ARG(d->kv_stride[i] >= 0 && d->kv_stride[i] % kal == 0, "kv_stride[%d]=%lld must be a non-negative multiple of %lld", i, (long long)d->kv_stride[i], (long long)kal);
  }
  USP_CHECK_ARG(d->q_stride[2] >= d->d && d->o_stride[2] >= d->d && (kv_auto(d) || d->kv_stride[2] >= d->d),
                "token strides must be >= d");
  p->W = d->n_chunks;
  p->max_len = 0;
  for (int r = 0; r < p->W; ++r) {
    USP_CHECK_ARG(d->chunk_len[r] >= 0, "chunk_len[%d]=%d is negative", r, d->chunk_len[r]);
    if (d->chunk_len[r] > p->max_len) p->max_len = d->chunk_len[r];
  }
  {
    const uint32_t kf = d->flags & (USP_ATTN_KERNEL_WIDE | USP_ATTN_KERNEL_SPLIT | USP_ATTN_KERNEL_MIXED);
    USP_CHECK_ARG((kf & (kf - 1)) == 0, "the USP_ATTN_KERNEL_* flags exclude one another");
  }
  p->fp8 = d->kv_dtype == USP_FP8_E4M3FN;
  USP_CHECK_ARG(!((d->flags & USP_ATTN_DOUBLE_BUFFER) && (d->flags & USP_ATTN_FUSED_PREFETCH)),
                "USP_ATTN_DOUBLE_BUFFER and USP_ATTN_FUSED_PREFETCH exclude each other");
  p->dbuf = (d->flags & (USP_ATTN_DOUBLE_BUFFER | USP_ATTN_FUSED_PREFETCH)) != 0 && p->W > 1;
  p->fused_pf = p->dbuf && (d->flags & USP_ATTN_FUSED_PREFETCH) != 0;
  p->unfused = (d->flags & USP_ATTN_UNFUSED_MERGE) != 0 && p->W > 1;
  p->mfma = d->qo_dtype == USP_BF16 && (d->d == 128 || d->d == 64);   // the matrix-core kernels: 256- or 128-byte K / V rows
  p->dequant_stage = p->fp8 && p->mfma;
  if (p->fp8 || p->dbuf) {
    for (int r = 0; r < p->W; ++r)
      if (d->chunk_len[r] > 0 && !kv_dense(d, d->chunk_len[r])) {
        set_error("FP8 K/V and the double-buffered modes need dense [B,H,chunk_len,d] chunks (chunk %d is strided)", r);
        return USP_ERR_UNSUPPORTED;
      }
  }
  if (p->unfused && !o_dense(d)) {
    set_error("USP_ATTN_UNFUSED_MERGE needs a dense [B,H,Sq,d] out");
    return USP_ERR_UNSUPPORTED;
  }
  p->rows_q = (size_t)d->B * d->H * d->Sq;
  size_t off = 0;
  if (p->W > 1 && !p->unfused) { p->off_acc = off; off += align_up(p->rows_q * d->d * 4); }
  if (p->unfused) {
    p->off_tmp_o = off; off += align_up(p->rows_q * d->d * elt_size(d->qo_dtype));
    p->off_tmp_lse = off; off += align_up(p->rows_q * 4);
  }
  const size_t chunk_elems = (size_t)d->B * d->H * p->max_len * d->d;
  const size_t chunk_tok = (size_t)d->B * d->H * p->max_len;
  if (p->dbuf) {
    size_t b = 0;
    p->buf_k = b; b += align_up(chunk_elems * elt_size(d->kv_dtype));
    p->buf_v = b; b += align_up(chunk_elems * elt_size(d->kv_dtype));
    if (p->fp8) {
      p->buf_ks = b; b += align_up(chunk_tok * 4);
      p->buf_vs = b; b += align_up(chunk_tok * 4);
    }
    p->off_buf[0] = off; off += b;
    p->off_buf[1] = off; off += b;
  }
  if (p->dequant_stage) {
    p->off_deq_k = off; off += align_up(chunk_elems * 2);
    p->off_deq_v = off; off += align_up(chunk_elems * 2);
  }
  if (p->mfma) {
    // Records are needed by chunks with FP8 scales, a key mask (not known here: assume one) or a
    // length that is not a multiple of 64; they are small (1 KB per 64 keys of a head).
    p->ext = true;
    p->off_ext = off; off += align_up(attn_mfma_ext_bytes(d->B, d->H, p->max_len));
    p->off_nlive = off; off += align_up((size_t)d->B * 4);
  }
  // Transfers inside a single launch over the whole ring (see usp_ring_attn_fwd): every chunk after
  // the first gets a staging buffer of its own, because a buffer that is reused inside one launch
  // would make the copy work-groups wait for the attention work-groups.
  p->ring1 = p->fused_pf && p->mfma && !p->fp8 && !p->unfused && !(d->flags & USP_ATTN_STEPWISE);
  if (p->ring1) {
    int live = 0;
    for (int r = 0; r < p->W; ++r) {
      if (d->chunk_len[r] == 0) continue;
      if (d->chunk_len[r] % 64 != 0) p->ring1 = false;
      ++live;
    }
    if (live < 2 || live > AttnStep::kMaxMulti) p->ring1 = false;
  }
  if (p->ring1) {
    p->off_ring1 = off;
    for (int r = 1; r < p->W; ++r) off += 2 * align_up((size_t)d->B * d->H * d->chunk_len[r] * d->d * 2);
    p->off_arrive = off; off += align_up(AttnStep::kMaxMulti * sizeof(int));
  }
  // FP8 chunks, all of them at hand or with the transfers inside the launches: the decoding of
  // Algorithm 1 line 4 rides in the one launch over the ring (copy work-groups decode chunk r+1
  // while chunk r is computed on), each live chunk into bf16 buffers of its own; key masks go into the
  // records the same work-groups write.
  p->ring8 = p->fp8 && p->mfma && !p->unfused && !(d->flags & (USP_ATTN_STEPWISE | USP_ATTN_DOUBLE_BUFFER)) &&
             (p->fused_pf || (int64_t)d->B * d->H * ((d->Sq + 255) / 256) <= 256);   // short ring steps (see usp_ring_attn_fwd)
  if (p->ring8) {
    int live = 0;
    size_t tiles = 0;
    for (int r = 0; r < p->W; ++r) {
      if (d->chunk_len[r] == 0) continue;
      if (d->chunk_len[r] % 64 != 0) p->ring8 = false;
      tiles += (size_t)d->chunk_len[r] / 64;
      ++live;
    }
    if (live < 2 || live > AttnStep::kMaxMulti) p->ring8 = false;
    if (p->ring8) {
      p->off_ring8 = off;
      for (int r = 0; r < p->W; ++r) off += 2 * align_up((size_t)d->B * d->H * d->chunk_len[r] * d->d * 2);
      p->off_ext8 = off; off += align_up((size_t)d->B * d->H * tiles * 1024);
      p->off_arrive = off; off += align_up(AttnStep::kMaxMulti * sizeof(int));
    }
  }
  // bf16 chunks that one launch could take (see usp_ring_attn_fwd): should some of them come with a key
  // mask (not known here), that launch reads per-tile records, 1 KB per 64 keys of a head
  p->multi_rec = p->mfma && !p->fp8 && (!p->dbuf || p->ring1) && !p->unfused && p->W > 1 && !(d->flags & USP_ATTN_STEPWISE);
  if (p->multi_rec) {
    int live = 0;
    size_t tiles = 0;
    for (int r = 0; r < p->W; ++r) {
      if (d->chunk_len[r] == 0) continue;
      if (d->chunk_len[r] % 64 != 0) p->multi_rec = false;
      tiles += (size_t)d->chunk_len[r] / 64;
      ++live;
    }
    if (live < 2 || live > AttnStep::kMaxMulti) p->multi_rec = false;
    if (p->multi_rec) { p->off_multi_rec = off; off += align_up((size_t)d->B * d->H * tiles * 1024); }
  }
  p->total = off;
  p->valid = true;
  return USP_OK;
}

}  // namespace
}  // namespace usp

using namespace usp;

// ---- the workspace of usp_ring_attn_fwd_noalloc: one array per GPU, held until the process ends ----
// In host code the array's name is only a handle for hipGetSymbolAddress; its device address, one per
// device, is looked up once with that device current and is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[USP_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

usp_status scratch_for_current_device(void** out) {
  int dev = -1;
  USP_CHECK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) {
    set_error("device ordinal %d is outside [0, %d)", dev, kMaxDevices);
    return USP_ERR_UNSUPPORTED;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    USP_CHECK_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (ptr == nullptr || (reinterpret_cast<uintptr_t>(ptr) & 255u) != 0) {
      set_error("the scratch array of device %d has no usable address", dev);
      return USP_ERR_HIP;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return USP_OK;
}
}  // namespace

extern "C" {

usp_status usp_ring_attn_fwd_noalloc(const usp_attn_desc* desc, const void* q, const void* const* k_chunks,
                                     const void* const* v_chunks, const float* const* k_scales,
                                     const float* const* v_scales, const uint8_t* const* key_mask, void* out,
                                     float* lse, void* compute_stream) {
  clear_error();
  Plan p;
  usp_status st = make_plan(desc, &p);
  if (st != USP_OK) return st;
  if ((desc->flags & USP_ATTN_DOUBLE_BUFFER) != 0) {
    set_error("usp_ring_attn_fwd_noalloc has no copy stream: USP_ATTN_DOUBLE_BUFFER is not available "
              "(USP_ATTN_FUSED_PREFETCH is)");
    return USP_ERR_UNSUPPORTED;
  }
  if (p.total > (size_t)USP_NOALLOC_SCRATCH_BYTES) {
    set_error("this call needs %zu bytes of workspace, the built-in scratch holds %zu: use usp_ring_attn_fwd "
              "with a workspace of the caller's", p.total, (size_t)USP_NOALLOC_SCRATCH_BYTES);
    return USP_ERR_WORKSPACE;
  }
  void* ws = nullptr;
  if (p.total > 0 && (st = scratch_for_current_device(&ws)) != USP_OK) return st;
  return ring_attn_fwd_impl(desc, q, k_chunks, v_chunks, k_scales, v_scales, key_mask, out, lse, ws,
                            p.total > 0 ? (size_t)USP_NOALLOC_SCRATCH_BYTES : 0, compute_stream, nullptr, CallOptions());
}

const char* usp_last_error(void) { return g_err; }
const char* usp_version(void) { return "usp-gfx950 0.1"; }

size_t usp_ring_attn_workspace_bytes(const usp_attn_desc* desc) {
  Plan p;
  if (make_plan(desc, &p) != USP_OK) return (size_t)-1;
  return p.total;
}

usp_status usp_fp8_quant(int64_t rows, int64_t cols, int32_t in_dt, const void* x, uint8_t* q,
                         float* scales, void* stream) {
  clear_error();
  USP_CHECK_ARG(rows >= 0 && cols >= 0, "rows and cols must be >= 0");
  USP_CHECK_ARG(in_dt == USP_F32 || in_dt == USP_BF16, "in_dt must be USP_F32 or USP_BF16");
  USP_CHECK_ARG(cols % 8 == 0, "cols=%lld must be a multiple of 8", (long long)cols);
  USP_CHECK_ARG(rows <= (int64_t)1 << 31, "rows=%lld too large", (long long)rows);
  if (rows == 0) return USP_OK;
  USP_CHECK_ARG(scales != nullptr, "scales is NULL");
  if (cols > 0) {
    USP_CHECK_ARG(x != nullptr && q != nullptr, "x or q is NULL");
    USP_CHECK_ARG(aligned16(x) && aligned16(q), "x and q must be 16-byte aligned");
  }
  return launch_fp8_quant(rows, cols, in_dt, x, q, scales, (hipStream_t)stream);
}

usp_status usp_fp8_dequant(int64_t rows, int64_t cols, int32_t out_dt, const uint8_t* q,
                           const float* scales, void* y, void* stream) {
  clear_error();
  USP_CHECK_ARG(rows >= 0 && cols >= 0, "rows and cols must be >= 0");
  USP_CHECK_ARG(out_dt == USP_F32 || out_dt == USP_BF16, "out_dt must be USP_F32 or USP_BF16");
  USP_CHECK_ARG(cols % 8 == 0, "cols=%lld must be a multiple of 8", (long long)cols);
  if (rows == 0 || cols == 0) return USP_OK;
  USP_CHECK_ARG(rows * (cols / 8) < ((int64_t)1 << 39), "tensor too large");
  USP_CHECK_ARG(q != nullptr && scales != nullptr && y != nullptr, "q, scales or y is NULL");
  USP_CHECK_ARG(aligned16(q) && aligned16(y), "q and y must be 16-byte aligned");
  return launch_fp8_dequant(rows, cols, out_dt, q, scales, y, (hipStream_t)stream);
}

namespace {
// Validates a row map and turns it into the kernels' form; *rows receives n0*n1*n2*n3.
usp_status check_row_map(const usp_row_map* map, int64_t cols, int64_t elt_src, int64_t elt_dst, RowMap* m, int64_t* rows) {
  USP_CHECK_ARG(map != nullptr, "map is NULL");
  USP_CHECK_ARG(cols >= 0 && cols % 8 == 0 && cols <= 4096, "cols=%lld must be a multiple of 8, at most 4096", (long long)cols);
  int64_t total = 1;
  for (int k = 0; k < 4; ++k) {
    USP_CHECK_ARG(map->n[k] >= 0 && map->n[k] < ((int64_t)1 << 31), "n[%d]=%lld out of range", k, (long long)map->n[k]);
    USP_CHECK_ARG(map->src_stride[k] >= 0 && map->dst_stride[k] >= 0, "strides must be >= 0");
    // element strides must keep rows 16-byte aligned (elt_* = bytes per element, 0 for row strides)
    USP_CHECK_ARG(elt_src == 0 || (map->src_stride[k] * elt_src) % 16 == 0, "src_stride[%d] breaks 16-byte row alignment", k);
    USP_CHECK_ARG(elt_dst == 0 || (map->dst_stride[k] * elt_dst) % 16 == 0, "dst_stride[%d] breaks 16-byte row alignment", k);
    total *= map->n[k];
    USP_CHECK_ARG(total < ((int64_t)1 << 40), "too many rows");
    m->src[k] = map->src_stride[k];
    m->dst[k] = map->dst_stride[k];
  }
  m->n1 = (uint32_t)(map->n[1] > 0 ? map->n[1] : 1);
  m->n2 = (uint32_t)(map->n[2] > 0 ? map->n[2] : 1);
  m->n3 = (uint32_t)(map->n[3] > 0 ? map->n[3] : 1);
  *rows = total;
  return USP_OK;
}
}  // namespace

usp_status usp_fp8_quant_mapped(const usp_row_map* map, int64_t cols, int32_t in_dt, const void* x,
                                uint8_t* q, float* scales, void* stream) {
  clear_error();
  USP_CHECK_ARG(in_dt == USP_F32 || in_dt == USP_BF16, "in_dt must be USP_F32 or USP_BF16");
  RowMap m;
  int64_t rows = 0;
  usp_status st = check_row_map(map, cols, in_dt == USP_F32 ? 4 : 2, 0, &m, &rows);
  if (st != USP_OK) return st;
  if (rows == 0 || cols == 0) return USP_OK;
  USP_CHECK_ARG(x != nullptr && q != nullptr && scales != nullptr, "x, q or scales is NULL");
  USP_CHECK_ARG(aligned16(x) && aligned16(q), "x and q must be 16-byte aligned");
  return launch_fp8_quant_mapped(m, rows, cols, in_dt, x, q, scales, (hipStream_t)stream);
}

usp_status usp_fp8_dequant_mapped(const usp_row_map* map, int64_t cols, int32_t out_dt, const uint8_t* q,
                                  const float* scales, void* y, void* stream) {
  clear_error();
  USP_CHECK_ARG(out_dt == USP_F32 || out_dt == USP_BF16, "out_dt must be USP_F32 or USP_BF16");
  RowMap m;
  int64_t rows = 0;
  usp_status st = check_row_map(map, cols, 0, out_dt == USP_F32 ? 4 : 2, &m, &rows);
  if (st != USP_OK) return st;
  if (rows == 0 || cols == 0) return USP_OK;
  USP_CHECK_ARG(q != nullptr && scales != nullptr && y != nullptr, "q, scales or y is NULL");
  USP_CHECK_ARG(aligned16(q) && aligned16(y), "q and y must be 16-byte aligned");
  return launch_fp8_dequant_mapped(m, rows, cols, out_dt, q, scales, y, (hipStream_t)stream);
}

usp_status usp_lse_merge(int64_t rows, int32_t d, int32_t dt, const void* o1, const float* lse1,
                         const void* o2, const float* lse2, void* o_out, float* lse_out, void* stream) {
  clear_error();
  USP_CHECK_ARG(rows >= 0, "rows must be >= 0");
  USP_CHECK_ARG(d > 0 && d % 8 == 0 && d <= 512, "d must be a multiple of 8 in [8, 512] (got %d)", d);
  USP_CHECK_ARG(dt == USP_F32 || dt == USP_BF16, "dt must be USP_F32 or USP_BF16");
  USP_CHECK_ARG(rows <= (int64_t)1 << 31, "rows=%lld too large", (long long)rows);
  if (rows == 0) return USP_OK;
  USP_CHECK_ARG(o1 && o2 && o_out && lse1 && lse2 && lse_out, "a required pointer is NULL");
  USP_CHECK_ARG(aligned16(o1) && aligned16(o2) && aligned16(o_out), "o1, o2 and o_out must be 16-byte aligned");
  return launch_lse_merge(rows, d, dt, o1, lse1, o2, lse2, o_out, lse_out, (hipStream_t)stream);
}

usp_status usp_ring_attn_fwd(const usp_attn_desc* desc, const void* q, const void* const* k_chunks,
                             const void* const* v_chunks, const float* const* k_scales,
                             const float* const* v_scales, const uint8_t* const* key_mask, void* out,
                             float* lse, void* workspace, size_t workspace_bytes, void* compute_stream,
                             void* copy_stream) {
  clear_error();
  return ring_attn_fwd_impl(desc, q, k_chunks, v_chunks, k_scales, v_scales, key_mask, out, lse, workspace,
                            workspace_bytes, compute_stream, copy_stream, CallOptions());
}

}  // extern "C"

usp_status usp::ring_attn_fwd_impl(const usp_attn_desc* desc, const void* q, const void* const* k_chunks,
                                   const void* const* v_chunks, const float* const* k_scales,
                                   const float* const* v_scales, const uint8_t* const* key_mask, void* out,
                                   float* lse, void* workspace, size_t workspace_bytes, void* compute_stream,
                                   void* copy_stream, const CallOptions& opt) {
  Plan p;
  usp_status st = make_plan(desc, &p);
  if (st != USP_OK) return st;
  USP_CHECK_ARG(q && out && lse && k_chunks && v_chunks, "q, out, lse, k_chunks or v_chunks is NULL");
  USP_CHECK_ARG(aligned16(q) && aligned16(out), "q and out must be 16-byte aligned");
  USP_CHECK_ARG(!p.fp8 || (k_scales && v_scales), "FP8 K/V needs k_scales and v_scales");
  for (int r = 0; r < p.W; ++r) {
    if (desc->chunk_len[r] == 0) continue;
    USP_CHECK_ARG(k_chunks[r] && v_chunks[r], "K or V pointer of chunk %d is NULL", r);
    USP_CHECK_ARG(aligned16(k_chunks[r]) && aligned16(v_chunks[r]), "K/V of chunk %d must be 16-byte aligned", r);
    USP_CHECK_ARG(!p.fp8 || (k_scales[r] && v_scales[r]), "scale pointer of chunk %d is NULL", r);
  }
  if (p.total > 0) {
    if (workspace == nullptr || workspace_bytes < p.total) {
      set_error("workspace of %zu bytes needed, %zu given", p.total, workspace ? workspace_bytes : (size_t)0);
      return USP_ERR_WORKSPACE;
    }
    USP_CHECK_ARG((reinterpret_cast<uintptr_t>(workspace) & 255u) == 0, "workspace must be 256-byte aligned");
  }
  hipStream_t cs = (hipStream_t)compute_stream, xs = (hipStream_t)copy_stream;
  if (p.dbuf && !p.fused_pf)
    USP_CHECK_ARG(xs != cs, "USP_ATTN_DOUBLE_BUFFER needs a copy_stream different from compute_stream");

  char* ws = (char*)workspace;
  const int d = desc->d;
  const float scale = desc->softmax_scale > 0.0f ? desc->softmax_scale : 1.0f / sqrtf((float)d);
  const size_t kv_es = elt_size(desc->kv_dtype);

  // ---- Algorithm 2, lines 1-3: the first prefetch is issued before the local chunk is computed
  std::vector<hipEvent_t> copied(p.W, nullptr), computed(p.W, nullptr);
  auto stage_chunk = [&](int r) -> usp_status {  // "recv" chunk r (r >= 1) into buffer (r-1)%2 on xs
    const int len = desc->chunk_len[r];
    char* buf = ws + p.off_buf[(r - 1) & 1];
    if (len > 0) {
      const size_t bytes = (size_t)desc->B * desc->H * len * d * kv_es;
      USP_CHECK_HIP(hipMemcpyAsync(buf + p.buf_k, k_chunks[r], bytes, hipMemcpyDefault, xs));
      USP_CHECK_HIP(hipMemcpyAsync(buf + p.buf_v, v_chunks[r], bytes, hipMemcpyDefault, xs));
      if (p.fp8) {
        const size_t sb = (size_t)desc->B * desc->H * len * 4;
        USP_CHECK_HIP(hipMemcpyAsync(buf + p.buf_ks, k_scales[r], sb, hipMemcpyDefault, xs));
        USP_CHECK_HIP(hipMemcpyAsync(buf + p.buf_vs, v_scales[r], sb, hipMemcpyDefault, xs));
      }
    }
    USP_CHECK_HIP(g_events.get(&copied[r]));
    USP_CHECK_HIP(hipEventRecord(copied[r], xs));
    return USP_OK;
  };
  // The same transfer as a list of segments for the work-groups that ride in step r-1's launch.
  auto prefetch_segments = [&](int r, AttnStep* a) {
    const int len = desc->chunk_len[r];
    char* buf = ws + p.off_buf[(r - 1) & 1];
    a->n_copy = 0;
    if (len <= 0) return;
    const int64_t bytes = (int64_t)desc->B * desc->H * len * d * (int64_t)kv_es;
    a->copy[a->n_copy++] = {k_chunks[r], buf + p.buf_k, bytes};
    a->copy[a->n_copy++] = {v_chunks[r], buf + p.buf_v, bytes};
    if (p.fp8) {
      const int64_t sb = (int64_t)desc->B * desc->H * len * 4;
      a->copy[a->n_copy++] = {k_scales[r], buf + p.buf_ks, sb};
      a->copy[a->n_copy++] = {v_scales[r], buf + p.buf_vs, sb};
    }
  };
  if (p.dbuf && !p.fused_pf) {
    hipEvent_t entry;
    USP_CHECK_HIP(g_events.get(&entry));
    USP_CHECK_HIP(hipEventRecord(entry, cs));            // inputs were produced on the compute stream
    USP_CHECK_HIP(hipStreamWaitEvent(xs, entry, 0));     // ... and earlier calls are done with the buffers
    if ((st = stage_chunk(1)) != USP_OK) return st;
  }

  // One launch over the ring pays when a ring step is short (launch, pipeline fill and the carried
  // state's round trip weigh on it).  Where the Q shard's 256-query blocks need more than one round of
  // work-groups on the 256 CUs, a step is long, its per-chunk launch can mix the two work
  // decompositions to fill its last round, and the plain call keeps one launch per chunk; a call
  // that asks for the transfers inside the launches takes the one launch at any size.
  const int64_t q_blocks = (int64_t)desc->B * desc->H * ((desc->Sq + 255) / 256);
  const bool short_steps = q_blocks <= 256 || p.fused_pf;
  // Every chunk resident, whole tiles, merge fused: one launch over the whole ring (chunks with a key
  // mask through per-tile records written just before it).
  {
    bool one_launch = p.mfma && !p.fp8 && (!p.dbuf || p.ring1) && !p.unfused && p.W > 1 && !(desc->flags & USP_ATTN_STEPWISE) &&
                      short_steps;
    int n_live = 0, n_masked = 0;
    int64_t keys = 0;
    for (int r = 0; one_launch && r < p.W; ++r) {
      const int len = desc->chunk_len[r];
      if (len == 0) continue;
      if (len % 64 != 0) one_launch = false;
      if (key_mask && key_mask[r]) ++n_masked;
      keys += len;
      ++n_live;
    }
    // Key masks: the one launch then reads per-tile records for every chunk, which costs it about a
    // third (96 against 73 us on a FLUX-1024 ring of four with one masked chunk), while the per-chunk
    // form pays for records only in the masked chunks' launches.  The one launch still wins where the
    // ring steps are short (below about 40 million query-key pairs per step) or every chunk is masked.
    if (one_launch && n_masked > 0 && n_masked < n_live &&
        (double)desc->B * desc->H * desc->Sq * ((double)keys / n_live) > 40e6)
      one_launch = false;
    if (one_launch && n_live >= 2 && n_live <= AttnStep::kMaxMulti && p.multi_rec) {
      AttnStep a;
      memset(&a, 0, sizeof(a));
      a.B = desc->B; a.H = desc->H; a.d = d; a.Sq = desc->Sq;
      a.qo_dtype = desc->qo_dtype; a.half_d = d == 64 ? 1 : 0; a.kv_dtype = desc->kv_dtype;
      a.q = q; a.out = out; a.lse = lse; a.scale = scale; a.mode = 0;
      for (int i = 0; i < 3; ++i) { a.qs[i] = desc->q_stride[i]; a.ks[i] = desc->kv_stride[i]; a.os[i] = desc->o_stride[i]; }
      if (kv_auto(desc)) a.ks[2] = d;
      a.variant = (desc->flags & USP_ATTN_KERNEL_SPLIT) ? 2 : (desc->flags & USP_ATTN_KERNEL_WIDE) ? 1 : 0;
      const bool transfers = p.dbuf;                      // (ring1) Algorithm 2 inside the launch
      if (transfers) a.ks[2] = d;                         // the double-buffered modes take dense chunks only
      size_t stage = p.off_ring1;
      for (int r = 0; r < p.W; ++r) {
        const int len = desc->chunk_len[r];
        const size_t bytes = (size_t)desc->B * desc->H * len * d * 2;
        if (len > 0) {
          AttnStep::Chunk& c = a.chunk[a.n_multi++];
          c.k = k_chunks[r]; c.v = v_chunks[r]; c.Sc = len;
          c.ks0 = kv_auto(desc) || transfers ? (int64_t)desc->H * len * d : desc->kv_stride[0];
          c.ks1 = kv_auto(desc) || transfers ? (int64_t)len * d : desc->kv_stride[1];
          if (transfers && a.n_multi > 1) {               // every live chunk but the first arrives through its buffer
            c.k_src = k_chunks[r]; c.v_src = v_chunks[r]; c.bytes = (int64_t)bytes;
            c.k = ws + stage; c.v = ws + stage + align_up(bytes);
          }
          if (key_mask && key_mask[r]) { c.mask_src = key_mask[r]; a.multi_masked = 1; }
        }
        if (r >= 1) stage += 2 * align_up(bytes);
      }
      if (transfers) {
        a.arrive = (int*)(ws + p.off_arrive);
        a.arrive_need_extra = opt.arrive_need_extra; a.arrive_polls = opt.arrive_polls;
        if ((st = launch_attn_arrive_reset(a.arrive, cs)) != USP_OK) return st;
      }
      if (a.multi_masked) {   // some chunk has a key mask: the launch reads per-tile records
        a.ext = (float*)(ws + p.off_multi_rec);
        if ((st = launch_attn_multi_records(a, cs)) != USP_OK) return st;
      }
      return launch_attn_mfma(a, cs);
    }
  }

  // FP8 chunks: one launch over the ring that decodes them as it goes
  if (p.ring8 && short_steps) {
    bool ok = true;
    for (int r = 0; r < p.W; ++r)
      if (desc->chunk_len[r] > 0 && (((uintptr_t)k_scales[r] & 15) != 0 || (key_mask && ((uintptr_t)key_mask[r] & 3) != 0))) ok = false;
    if (ok) {
      AttnStep a;
      memset(&a, 0, sizeof(a));
      a.B = desc->B; a.H = desc->H; a.d = d; a.Sq = desc->Sq;
      a.qo_dtype = desc->qo_dtype; a.half_d = d == 64 ? 1 : 0; a.kv_dtype = USP_BF16;   // what the attention work-groups read
      a.q = q; a.out = out; a.lse = lse; a.scale = scale; a.mode = 0;
      for (int i = 0; i < 3; ++i) { a.qs[i] = desc->q_stride[i]; a.os[i] = desc->o_stride[i]; }
      a.ks[2] = d;
      a.variant = (desc->flags & USP_ATTN_KERNEL_SPLIT) ? 2 : (desc->flags & USP_ATTN_KERNEL_WIDE) ? 1 : 0;
      a.multi_fp8 = 1;
      a.ext = (float*)(ws + p.off_ext8);
      a.arrive = (int*)(ws + p.off_arrive);
      a.arrive_need_extra = opt.arrive_need_extra; a.arrive_polls = opt.arrive_polls;
      size_t stage = p.off_ring8;
      for (int r = 0; r < p.W; ++r) {
        const int len = desc->chunk_len[r];
        const size_t bytes = (size_t)desc->B * desc->H * len * d * 2;
        if (len > 0) {
          AttnStep::Chunk& c = a.chunk[a.n_multi++];
          c.Sc = len;
          c.ks0 = (int64_t)desc->H * len * d; c.ks1 = (int64_t)len * d;
          c.k = ws + stage; c.v = ws + stage + align_up(bytes);
          c.k_src = k_chunks[r]; c.v_src = v_chunks[r]; c.bytes = (int64_t)(bytes / 2);
          c.k_scale_src = k_scales[r]; c.v_scale_src = v_scales[r];
          c.mask_src = key_mask ? key_mask[r] : nullptr;
          if (c.mask_src) a.multi_masked = 1;
        }
        stage += 2 * align_up(bytes);
      }
      if ((st = launch_attn_fp8_chunk_prepare(a, 0, true, cs)) != USP_OK) return st;   // also zeroes the counters
      return launch_attn_mfma(a, cs);
    }
  }

  for (int r = 0; r < p.W; ++r) {
    const int len = desc->chunk_len[r];
    const void* kp = k_chunks[r];
    const void* vp = v_chunks[r];
    const float* ksp = p.fp8 ? k_scales[r] : nullptr;
    const float* vsp = p.fp8 ? v_scales[r] : nullptr;
    if (p.dbuf && r >= 1) {
      // line 6: the chunk must have arrived; line 7: start the next transfer, which may only
      // overwrite the other buffer once the step that read it (r-1) has finished.  With the
      // transfers inside the attention launches, stream order alone gives both.
      if (!p.fused_pf) {
        USP_CHECK_HIP(hipStreamWaitEvent(cs, copied[r], 0));
        if (r + 1 < p.W) {
          if (r >= 2) USP_CHECK_HIP(hipStreamWaitEvent(xs, computed[r - 1], 0));
          if ((st = stage_chunk(r + 1)) != USP_OK) return st;
        }
      }
      char* buf = ws + p.off_buf[(r - 1) & 1];
      kp = buf + p.buf_k;
      vp = buf + p.buf_v;
      if (p.fp8) { ksp = (const float*)(buf + p.buf_ks); vsp = (const float*)(buf + p.buf_vs); }
    }

    AttnStep a;
    memset(&a, 0, sizeof(a));
    a.B = desc->B; a.H = desc->H; a.d = d; a.Sq = desc->Sq; a.Sc = len;
    a.qo_dtype = desc->qo_dtype; a.half_d = d == 64 ? 1 : 0; a.kv_dtype = desc->kv_dtype;
    a.q = q; a.k = kp; a.v = vp; a.k_scale = ksp; a.v_scale = vsp;
    a.key_mask = key_mask ? key_mask[r] : nullptr;
    for (int i = 0; i < 3; ++i) { a.qs[i] = desc->q_stride[i]; a.ks[i] = desc->kv_stride[i]; a.os[i] = desc->o_stride[i]; }
    if (p.fp8 || (p.dbuf && r >= 1) || kv_auto(desc)) {  // dense chunk
      a.ks[2] = d; a.ks[1] = (int64_t)len * d; a.ks[0] = (int64_t)desc->H * len * d;
    }
    if (p.fused_pf && r + 1 < p.W) prefetch_segments(r + 1, &a);
    a.scale = scale;
    a.variant = (desc->flags & USP_ATTN_KERNEL_SPLIT) ? 2 : (desc->flags & USP_ATTN_KERNEL_WIDE) ? 1 :
                (desc->flags & USP_ATTN_KERNEL_MIXED) ? 4 : 0;
    a.lse = lse;
    a.out = out;
    a.acc = p.W > 1 && !p.unfused ? (float*)(ws + p.off_acc) : nullptr;
    if (p.W == 1) a.mode = 0;
    else if (p.unfused) {
      a.mode = 0;
      if (r > 0) {
        a.out = ws + p.off_tmp_o;
        a.lse = (float*)(ws + p.off_tmp_lse);
        a.os[2] = d; a.os[1] = (int64_t)desc->Sq * d; a.os[0] = (int64_t)desc->H * desc->Sq * d;
      }
    } else a.mode = r == 0 ? 1 : (r == p.W - 1 ? 3 : 2);

    bool records_ready = false;
    if (p.dequant_stage && len > 0 && len % 64 == 0 && aligned16(kp) && aligned16(vp) && aligned16(ksp) && aligned16(vsp) &&
        ((uintptr_t)a.key_mask & 3u) == 0) {
      // Algorithm 1 line 4 for a chunk of whole tiles, in one launch: K widened exactly, V dequantised to
      // bf16(code * scale), the per-tile records (K's scales as per-key factors, the mask) and the live-tile
      // counts; the same arithmetic as the three launches of the general case below, bit for bit
      AttnStep m;
      memset(&m, 0, sizeof(m));
      m.B = desc->B; m.H = desc->H; m.d = d; m.scale = scale;
      m.n_multi = 1; m.multi_fp8 = 1;
      m.ext = (float*)(ws + p.off_ext);
      AttnStep::Chunk& c = m.chunk[0];
      c.k = ws + p.off_deq_k; c.v = ws + p.off_deq_v; c.Sc = len;
      c.ks0 = (int64_t)desc->H * len * d; c.ks1 = (int64_t)len * d;
      c.k_src = kp; c.v_src = vp; c.k_scale_src = ksp; c.v_scale_src = vsp;
      c.mask_src = a.key_mask;
      if ((st = launch_attn_fp8_step_prepare(m, (int*)(ws + p.off_nlive), cs)) != USP_OK) return st;
      a.k = c.k; a.v = c.v;
      a.v_scale = nullptr;
      a.kv_dtype = USP_BF16;
      a.ext = m.ext;
      a.n_live = (int*)(ws + p.off_nlive);
      records_ready = true;
    } else if (p.dequant_stage && len > 0) {
      // Algorithm 1 line 4.  K: the codes are widened to bf16 exactly here (scale 1) and the MFMA
      // kernel multiplies the fp32 scores by the per-token scales, so the exponents see no rounding
      // beyond the quantisation itself.  V: dequantised to the working precision, bf16(code * scale).
      const int64_t rows = (int64_t)desc->B * desc->H * len;
      if ((st = launch_fp8_dequant(rows, d, USP_BF16, (const uint8_t*)kp, nullptr, ws + p.off_deq_k, cs)) != USP_OK) return st;
      if ((st = launch_fp8_dequant(rows, d, USP_BF16, (const uint8_t*)vp, vsp, ws + p.off_deq_v, cs)) != USP_OK) return st;
      a.k = ws + p.off_deq_k; a.v = ws + p.off_deq_v;
      a.v_scale = nullptr;
      a.kv_dtype = USP_BF16;
    } else if (p.dequant_stage) {
      // an empty chunk still merges and stores (its epilogue mode): keep it on the matrix-core kernel,
      // which reads no key of it
      a.k_scale = nullptr; a.v_scale = nullptr;
      a.kv_dtype = USP_BF16;
    }
    if (!records_ready && attn_mfma_supported(a) && attn_mfma_needs_ext(a)) {
      a.ext = (float*)(ws + p.off_ext);
      a.n_live = (int*)(ws + p.off_nlive);
      if ((st = launch_attn_ext_prepare(a, cs)) != USP_OK) return st;
    }
    st = attn_mfma_supported(a) ? launch_attn_mfma(a, cs) : launch_attn_generic(a, cs);
    if (st != USP_OK) return st;
    if (p.unfused && r > 0) {
      st = launch_lse_merge((int64_t)p.rows_q, d, desc->qo_dtype, out, lse, ws + p.off_tmp_o,
                            (const float*)(ws + p.off_tmp_lse), out, lse, cs);
      if (st != USP_OK) return st;
    }
    if (p.dbuf && !p.fused_pf && r >= 1 && r + 2 < p.W) {  // a later transfer will reuse this step's buffer
      USP_CHECK_HIP(g_events.get(&computed[r]));
      USP_CHECK_HIP(hipEventRecord(computed[r], cs));
    }
  }
  return USP_OK;
}
