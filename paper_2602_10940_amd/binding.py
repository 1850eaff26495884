"""ctypes binding of libusp.so: same names as the C ABI in include/usp.h.

Marshalling only: every step of the path runs in the library's HIP kernels.  torch is
used for device memory and stream handles, nothing else.  There is no CPU fallback:
if the library is missing or a call fails, a UspError is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libusp.so")

USP_OK, USP_ERR_INVALID_ARG, USP_ERR_UNSUPPORTED, USP_ERR_WORKSPACE, USP_ERR_HIP = 0, -1, -2, -3, -4
USP_F32, USP_BF16, USP_FP8_E4M3FN = 0, 1, 2
USP_ATTN_DOUBLE_BUFFER, USP_ATTN_UNFUSED_MERGE = 1, 2
USP_ATTN_KERNEL_WIDE, USP_ATTN_KERNEL_SPLIT = 4, 8
USP_ATTN_FUSED_PREFETCH = 16
USP_ATTN_KERNEL_MIXED = 32
USP_ATTN_STEPWISE = 64
USP_NOALLOC_SCRATCH_BYTES = 64 << 20

EXPORTS = ("usp_ring_attn_workspace_bytes", "usp_ring_attn_fwd", "usp_ring_attn_fwd_noalloc", "usp_lse_merge", "usp_fp8_quant",
           "usp_fp8_dequant", "usp_fp8_quant_mapped", "usp_fp8_dequant_mapped",
           "usp_last_error", "usp_version")


class RowMap(ctypes.Structure):
    """usp_row_map: rows visited as (i0..i3), i3 fastest; offsets sum i_k * stride[k]."""
    _fields_ = [("n", ctypes.c_int64 * 4), ("src_stride", ctypes.c_int64 * 4), ("dst_stride", ctypes.c_int64 * 4)]


def make_row_map(n, src_stride, dst_stride) -> "RowMap":
    m = RowMap()
    for k in range(4):
        m.n[k], m.src_stride[k], m.dst_stride[k] = int(n[k]), int(src_stride[k]), int(dst_stride[k])
    return m


class UspError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("usp status %d: %s" % (status, msg))
        self.status = status


class AttnDesc(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("d", ctypes.c_int32),
        ("Sq", ctypes.c_int32), ("n_chunks", ctypes.c_int32),
        ("chunk_len", ctypes.POINTER(ctypes.c_int32)),
        ("qo_dtype", ctypes.c_int32), ("kv_dtype", ctypes.c_int32),
        ("q_stride", ctypes.c_int64 * 3), ("kv_stride", ctypes.c_int64 * 3),
        ("o_stride", ctypes.c_int64 * 3),
        ("softmax_scale", ctypes.c_float), ("flags", ctypes.c_uint32),
    ]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libusp.so (built in-tree by paper_2602_10940_amd.build). Fails loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise UspError(USP_ERR_HIP, "%s not found: run `python -m paper_2602_10940_amd.build` "
                       "(or __graft_entry__.build()) first; there is no fallback path" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    lib.usp_last_error.restype = ctypes.c_char_p
    lib.usp_version.restype = ctypes.c_char_p
    lib.usp_ring_attn_workspace_bytes.restype = sz
    lib.usp_ring_attn_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc)]
    lib.usp_ring_attn_fwd.restype = i32
    lib.usp_ring_attn_fwd.argtypes = [ctypes.POINTER(AttnDesc), vp, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                      ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                      vp, vp, vp, sz, vp, vp]
    lib.usp_ring_attn_fwd_noalloc.restype = i32
    lib.usp_ring_attn_fwd_noalloc.argtypes = [ctypes.POINTER(AttnDesc), vp, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                              ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp, vp, vp]
    lib.usp_lse_merge.restype = i32
    lib.usp_lse_merge.argtypes = [i64, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.usp_fp8_quant.restype = i32
    lib.usp_fp8_quant.argtypes = [i64, i64, i32, vp, vp, vp, vp]
    lib.usp_fp8_dequant.restype = i32
    lib.usp_fp8_dequant.argtypes = [i64, i64, i32, vp, vp, vp, vp]
    lib.usp_fp8_quant_mapped.restype = i32
    lib.usp_fp8_quant_mapped.argtypes = [ctypes.POINTER(RowMap), i64, i32, vp, vp, vp, vp]
    lib.usp_fp8_dequant_mapped.restype = i32
    lib.usp_fp8_dequant_mapped.argtypes = [ctypes.POINTER(RowMap), i64, i32, vp, vp, vp, vp]
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != USP_OK:
        raise UspError(status, load_library().usp_last_error().decode())


def _dt(t: torch.dtype) -> int:
    if t == torch.float32:
        return USP_F32
    if t == torch.bfloat16:
        return USP_BF16
    if t == torch.uint8:
        return USP_FP8_E4M3FN
    raise UspError(USP_ERR_INVALID_ARG, "unsupported torch dtype %s" % t)


def _stream_handle(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _ptr_array(ts: Optional[Sequence[Optional[torch.Tensor]]]):
    if ts is None:
        return None
    return (ctypes.c_void_p * len(ts))(*[_ptr(t) for t in ts])


# ---------------------------------------------------------------------------------------
def usp_version() -> str:
    return load_library().usp_version().decode()


def usp_fp8_quant(x: torch.Tensor, q: Optional[torch.Tensor] = None,
                  scales: Optional[torch.Tensor] = None, stream=None
                  ) -> Tuple[torch.Tensor, torch.Tensor]:
    """x [rows, cols] (bf16 or f32, dense) -> (codes uint8 [rows, cols], scales f32 [rows])."""
    lib = load_library()
    assert x.dim() == 2 and x.is_contiguous() and x.is_cuda
    rows, cols = x.shape
    if q is None:
        q = torch.empty((rows, cols), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows,), dtype=torch.float32, device=x.device)
    _check(lib.usp_fp8_quant(rows, cols, _dt(x.dtype), _ptr(x), _ptr(q), _ptr(scales), _stream_handle(stream)))
    return q, scales


def usp_fp8_dequant(q: torch.Tensor, scales: torch.Tensor, out_dtype: torch.dtype = torch.bfloat16,
                    y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    lib = load_library()
    assert q.dim() == 2 and q.is_contiguous() and q.dtype == torch.uint8 and q.is_cuda
    rows, cols = q.shape
    if y is None:
        y = torch.empty((rows, cols), dtype=out_dtype, device=q.device)
    _check(lib.usp_fp8_dequant(rows, cols, _dt(y.dtype), _ptr(q), _ptr(scales), _ptr(y), _stream_handle(stream)))
    return y


def usp_fp8_quant_mapped(x: torch.Tensor, n, src_stride, dst_stride, cols: int,
                         q: Optional[torch.Tensor] = None, scales: Optional[torch.Tensor] = None,
                         stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """x: any contiguous tensor (flat element offsets); returns q uint8 [rows, cols], scales f32 [rows]
    with rows = prod(n).  src_stride in elements of x, dst_stride in rows of q."""
    lib = load_library()
    assert x.is_contiguous() and x.is_cuda
    rows = int(n[0]) * int(n[1]) * int(n[2]) * int(n[3])
    if q is None:
        q = torch.empty((rows, cols), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows,), dtype=torch.float32, device=x.device)
    m = make_row_map(n, src_stride, dst_stride)
    _check(lib.usp_fp8_quant_mapped(ctypes.byref(m), cols, _dt(x.dtype), _ptr(x), _ptr(q), _ptr(scales),
                                    _stream_handle(stream)))
    return q, scales


def usp_fp8_dequant_mapped(q: torch.Tensor, scales: torch.Tensor, n, src_stride, dst_stride, y: torch.Tensor,
                           stream=None) -> torch.Tensor:
    """q uint8 [rows, cols] and scales read by row (src_stride in rows); rows written into the contiguous
    tensor y (bf16 or f32) at element offsets sum i_k * dst_stride[k]."""
    lib = load_library()
    assert q.dim() == 2 and q.is_contiguous() and q.dtype == torch.uint8 and y.is_contiguous()
    m = make_row_map(n, src_stride, dst_stride)
    _check(lib.usp_fp8_dequant_mapped(ctypes.byref(m), q.shape[1], _dt(y.dtype), _ptr(q), _ptr(scales), _ptr(y),
                                      _stream_handle(stream)))
    return y


def usp_lse_merge(o1: torch.Tensor, lse1: torch.Tensor, o2: torch.Tensor, lse2: torch.Tensor,
                  o_out: Optional[torch.Tensor] = None, lse_out: Optional[torch.Tensor] = None,
                  stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """o* [..., d] dense, lse* [...] f32.  Outputs may alias inputs."""
    lib = load_library()
    assert o1.is_contiguous() and o2.is_contiguous() and o1.shape == o2.shape and o1.dtype == o2.dtype
    d = o1.shape[-1]
    rows = o1.numel() // d if d else 0
    if o_out is None:
        o_out = torch.empty_like(o1)
    if lse_out is None:
        lse_out = torch.empty_like(lse1)
    _check(lib.usp_lse_merge(rows, d, _dt(o1.dtype), _ptr(o1), _ptr(lse1), _ptr(o2), _ptr(lse2),
                             _ptr(o_out), _ptr(lse_out), _stream_handle(stream)))
    return o_out, lse_out


def make_attn_desc(q: torch.Tensor, k_chunks: Sequence[torch.Tensor], out: torch.Tensor,
                   softmax_scale: float = 0.0, flags: int = 0):
    """Fill a usp_attn_desc from [B,H,S,d] tensors (any B/H/token strides, d contiguous)."""
    B, H, Sq, d = q.shape
    lens = (ctypes.c_int32 * len(k_chunks))(*[int(k.shape[2]) for k in k_chunks])
    desc = AttnDesc()
    desc.B, desc.H, desc.d, desc.Sq, desc.n_chunks = B, H, d, Sq, len(k_chunks)
    desc.chunk_len = ctypes.cast(lens, ctypes.POINTER(ctypes.c_int32))
    desc.qo_dtype = _dt(q.dtype)
    desc.kv_dtype = _dt(k_chunks[0].dtype)
    assert q.stride(3) == 1 and out.stride(3) == 1
    live = [k for k in k_chunks if k.shape[2] > 0]
    dense = all(k.is_contiguous() for k in live)
    for i in range(3):
        desc.q_stride[i] = q.stride(i)
        desc.o_stride[i] = out.stride(i)
        # all-zero kv_stride = every chunk dense for its own length
        desc.kv_stride[i] = 0 if (dense or not live) else live[0].stride(i)
    if not dense:
        assert all(k.stride() == live[0].stride() and k.stride(3) == 1 for k in live), \
            "strided KV chunks must share one stride triple"
    desc.softmax_scale = float(softmax_scale)
    desc.flags = int(flags)
    desc._keepalive = lens
    return desc


def usp_ring_attn_workspace_bytes(desc: AttnDesc) -> int:
    n = load_library().usp_ring_attn_workspace_bytes(ctypes.byref(desc))
    if n == ctypes.c_size_t(-1).value:
        raise UspError(USP_ERR_INVALID_ARG, load_library().usp_last_error().decode())
    return int(n)


def usp_ring_attn_fwd(q: torch.Tensor, k_chunks: Sequence[torch.Tensor], v_chunks: Sequence[torch.Tensor],
                      k_scales: Optional[Sequence[torch.Tensor]] = None,
                      v_scales: Optional[Sequence[torch.Tensor]] = None,
                      key_mask: Optional[Sequence[Optional[torch.Tensor]]] = None,
                      softmax_scale: float = 0.0, flags: int = 0,
                      out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                      workspace: Optional[torch.Tensor] = None,
                      compute_stream=None, copy_stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Ring attention of q [B,H,Sq,d] over KV chunks [B,H,Sc_r,d]; returns (out, lse [B,H,Sq])."""
    lib = load_library()
    B, H, Sq, d = q.shape
    if out is None:
        out = torch.empty((B, H, Sq, d), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((B, H, Sq), dtype=torch.float32, device=q.device)
    desc = make_attn_desc(q, k_chunks, out, softmax_scale, flags)
    need = usp_ring_attn_workspace_bytes(desc)
    if workspace is None and need > 0:
        workspace = torch.empty((need,), dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    cs = _stream_handle(compute_stream)
    xs = None if copy_stream is None else _stream_handle(copy_stream)
    _check(lib.usp_ring_attn_fwd(ctypes.byref(desc), _ptr(q), _ptr_array(k_chunks), _ptr_array(v_chunks),
                                 _ptr_array(k_scales), _ptr_array(v_scales), _ptr_array(key_mask),
                                 _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes, cs, xs))
    out._usp_workspace = workspace  # keep the workspace alive as long as the result
    return out, lse


def usp_ring_attn_fwd_noalloc(q: torch.Tensor, k_chunks: Sequence[torch.Tensor], v_chunks: Sequence[torch.Tensor],
                              out: torch.Tensor, lse: torch.Tensor,
                              k_scales: Optional[Sequence[torch.Tensor]] = None,
                              v_scales: Optional[Sequence[torch.Tensor]] = None,
                              key_mask: Optional[Sequence[Optional[torch.Tensor]]] = None,
                              softmax_scale: float = 0.0, flags: int = 0, compute_stream=None
                              ) -> Tuple[torch.Tensor, torch.Tensor]:
    """usp_ring_attn_fwd on the library's built-in scratch: the caller passes every input and output
    (out [B,H,Sq,d], lse [B,H,Sq]); nothing is allocated, here or in the library."""
    lib = load_library()
    desc = make_attn_desc(q, k_chunks, out, softmax_scale, flags)
    _check(lib.usp_ring_attn_fwd_noalloc(ctypes.byref(desc), _ptr(q), _ptr_array(k_chunks), _ptr_array(v_chunks),
                                         _ptr_array(k_scales), _ptr_array(v_scales), _ptr_array(key_mask),
                                         _ptr(out), _ptr(lse), _stream_handle(compute_stream)))
    return out, lse
