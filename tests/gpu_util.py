"""Helpers shared by the GPU parity tests (host<->device marshalling, error metrics)."""
import numpy as np
import torch

from paper_2602_10940_amd import workloads as W

DEV = "cuda:0"


def dev_bf16(x32: np.ndarray) -> torch.Tensor:
    """float32 array holding bf16-exact values -> bf16 device tensor (exact)."""
    bits = W.f32_to_bf16_bits(x32)
    t = torch.from_numpy(bits.view(np.int16).copy()).to(DEV)
    return t.view(torch.bfloat16).reshape(x32.shape)


def dev_f32(x32: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(DEV)


def host_f64(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return W.bf16_bits_to_f32(bits).astype(np.float64).reshape(t.shape)
    return t.detach().cpu().numpy().astype(np.float64)


def host_bits_bf16(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def attn_errors(got: np.ndarray, ref: np.ndarray):
    """(max-abs error, relative L2 error) of an attention output against the oracle."""
    diff = got - ref
    return float(np.max(np.abs(diff))), float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-300))


# parity bars (bf16 inputs): attention max-abs 2e-2 and rel-L2 5e-3, lse 1e-3
ATTN_MAX_ABS = 2e-2
ATTN_REL_L2 = 5e-3
LSE_ABS = 1e-3
