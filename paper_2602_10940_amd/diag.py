"""ctypes binding of libusp_diag.so (csrc/diag/usp_diag.h): diagnostics for the benchmark and the
tests, outside the library's ABI.  Marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

from . import binding as B

DIAG_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libusp_diag.so")
_diag = None


def load_diag_library() -> ctypes.CDLL:
    global _diag
    if _diag is not None:
        return _diag
    B.load_library()   # libusp_diag.so is linked against libusp.so
    if not os.path.exists(DIAG_LIB_PATH):
        raise B.UspError(B.USP_ERR_HIP, "%s not found: run `python -m paper_2602_10940_amd.build` first" % DIAG_LIB_PATH)
    lib = ctypes.CDLL(DIAG_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.usp_diag_mfma_rate.restype = i32
    lib.usp_diag_mfma_rate.argtypes = [i32, i32, i32, i32, vp, vp, vp]
    lib.usp_diag_check_bf16_division.restype = i32
    lib.usp_diag_check_bf16_division.argtypes = [vp, vp]
    lib.usp_diag_payload_floor.restype = i32
    lib.usp_diag_payload_floor.argtypes = [i32, i32, vp, vp, vp, vp]
    lib.usp_diag_repeat_payload_calls.restype = i32
    lib.usp_diag_repeat_payload_calls.argtypes = [i32, i32, i32, ctypes.c_int64, ctypes.c_int64, ctypes.POINTER(vp),
                                                  ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp]
    lib.usp_diag_repeat_merge_calls.restype = i32
    lib.usp_diag_repeat_merge_calls.argtypes = [i32, i32, ctypes.c_int64, i32] + [ctypes.POINTER(vp)] * 6 + [vp]
    lib.usp_diag_ring_attn_fwd_wait.restype = i32
    lib.usp_diag_ring_attn_fwd_wait.argtypes = [ctypes.POINTER(B.AttnDesc), vp, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                                ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                                vp, vp, vp, sz, vp, i32, i32]
    _diag = lib
    return lib


def usp_diag_mfma_rate(wgs: int, iters: int, random_data: bool, out: torch.Tensor, clocks: torch.Tensor,
                       stream=None, shape: int = 0) -> None:
    """out: f32 device tensor of wgs*512 elements; clocks: int64 device tensor of 2 (shader cycles, 100 MHz ticks)."""
    lib = load_diag_library()
    assert out.dtype == torch.float32 and out.numel() >= wgs * 512 and out.is_contiguous()
    assert clocks.dtype == torch.int64 and clocks.numel() >= 2 and clocks.is_contiguous()
    B._check(lib.usp_diag_mfma_rate(int(wgs), int(iters), 1 if random_data else 0, int(shape), B._ptr(out), B._ptr(clocks),
                                    B._stream_handle(stream)))


def usp_diag_check_bf16_division(stream=None):
    """(pairs checked, codes that differ, quotients that differ, absmax values outside the fast range)."""
    lib = load_diag_library()
    counts = torch.zeros((4,), dtype=torch.int64, device="cuda")
    B._check(lib.usp_diag_check_bf16_division(B._ptr(counts), B._stream_handle(stream)))
    return tuple(int(v) for v in counts.cpu())


def usp_diag_payload_floor(kind: int, x: torch.Tensor, q: torch.Tensor, scales: torch.Tensor, stream=None) -> None:
    """kind 0 empty launch, 1 read-only, 2 write-only, on the pack's grid for x [rows, 3072] bf16."""
    lib = load_diag_library()
    assert x.dim() == 2 and x.shape[1] == 3072 and x.dtype == torch.bfloat16 and x.is_contiguous()
    assert q.numel() >= x.numel() and scales.numel() >= x.shape[0]
    B._check(lib.usp_diag_payload_floor(int(kind), x.shape[0], B._ptr(x), B._ptr(q), B._ptr(scales), B._stream_handle(stream)))


def usp_diag_repeat_payload_calls(kind: int, reps: int, xs, qs, ss, ys, stream=None) -> None:
    """reps back-to-back library calls issued from C over the buffer sets (lists of tensors, bf16 [rows, cols])."""
    lib = load_diag_library()
    rows, cols = xs[0].shape
    assert all(t.shape == (rows, cols) and t.is_contiguous() for t in list(xs) + list(qs) + list(ys))
    B._check(lib.usp_diag_repeat_payload_calls(int(kind), int(reps), len(xs), rows, cols, B._ptr_array(xs), B._ptr_array(qs),
                                               B._ptr_array(ss), B._ptr_array(ys), B._stream_handle(stream)))


def usp_diag_repeat_merge_calls(reps: int, o1, l1, o2, l2, o, l, stream=None) -> None:
    """reps back-to-back usp_lse_merge calls issued from C over the buffer sets (lists of bf16 [rows, d] / f32 [rows])."""
    lib = load_diag_library()
    rows, d = o1[0].shape
    B._check(lib.usp_diag_repeat_merge_calls(int(reps), len(o1), rows, d, B._ptr_array(o1), B._ptr_array(l1), B._ptr_array(o2),
                                             B._ptr_array(l2), B._ptr_array(o), B._ptr_array(l), B._stream_handle(stream)))


def usp_diag_ring_attn_fwd_wait(q: torch.Tensor, k_chunks: Sequence[torch.Tensor], v_chunks: Sequence[torch.Tensor],
                                arrive_need_extra: int, arrive_polls: int,
                                k_scales: Optional[Sequence[torch.Tensor]] = None,
                                v_scales: Optional[Sequence[torch.Tensor]] = None,
                                key_mask: Optional[Sequence[Optional[torch.Tensor]]] = None,
                                softmax_scale: float = 0.0, flags: int = 0,
                                workspace: Optional[torch.Tensor] = None, compute_stream=None
                                ) -> Tuple[torch.Tensor, torch.Tensor]:
    """usp_ring_attn_fwd with the knobs of the one-launch ring's bounded arrival wait."""
    lib = load_diag_library()
    Bn, H, Sq, d = q.shape
    out = torch.empty((Bn, H, Sq, d), dtype=q.dtype, device=q.device)
    lse = torch.empty((Bn, H, Sq), dtype=torch.float32, device=q.device)
    desc = B.make_attn_desc(q, k_chunks, out, softmax_scale, flags)
    need = B.usp_ring_attn_workspace_bytes(desc)
    if workspace is None and need > 0:
        workspace = torch.empty((need,), dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    B._check(lib.usp_diag_ring_attn_fwd_wait(ctypes.byref(desc), B._ptr(q), B._ptr_array(k_chunks), B._ptr_array(v_chunks),
                                             B._ptr_array(k_scales), B._ptr_array(v_scales), B._ptr_array(key_mask),
                                             B._ptr(out), B._ptr(lse), B._ptr(workspace), ws_bytes,
                                             B._stream_handle(compute_stream), int(arrive_need_extra), int(arrive_polls)))
    out._usp_workspace = workspace
    return out, lse
