"""Seeded synthetic inputs for the USP hot path (ring attention + FP8 payloads).

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic (no softmax, no merge, no FP8 codec).  Both the CPU oracle's
tests and the HIP path's tests/bench draw their inputs from here so that both
sides see identical values.

Shapes stand in for one rank's attention shard of a FLUX / Qwen-Image style
multi-modal diffusion transformer under Unified Sequence Parallelism
(paper section 2.2: Q/K/V are [B, H, S, D]; a ring of degree W splits the KV
sequence into W chunks; the Ulysses All-to-All payload is a [tokens, H*D]
matrix).  No model weights or images are involved: values are N(0,1) draws with
the per-workload modifications listed in WORKLOADS.

Draw order for every workload, from numpy PCG64(seed), float32, C order:
  Q [B,H,Sq,d], then K [B,H,S,d], then V [B,H,S,d], then the auxiliary draws
  (per-head scales, outlier masks), then the FP8 payload matrix.
bf16 workloads round the fp32 draws to bf16 (round-to-nearest-even) and hand
out BOTH the bf16 bit patterns (uint16) and the exactly-equal float32 values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np


# ---------------------------------------------------------------------------
# bf16 <-> fp32 bit helpers (input preparation only)
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------------------
# workload table
# ---------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    B: int
    H: int
    d: int
    Sq: int                      # local Q shard tokens
    chunk_len: Tuple[int, ...]   # tokens per KV chunk, ring order
    dtype: str                   # "f32" or "bf16"
    k_mul: float = 1.0           # K multiplied by this before rounding
    head_scale: bool = False     # per-head c_h ~ U(0.5, 2) applied to Q, K, V
    outlier_frac: float = 0.0    # Bernoulli fraction of entries multiplied by outlier_mul
    outlier_mul: float = 1.0
    masked_keys: Tuple[int, int] = (0, 0)   # [lo, hi) global key positions masked out
    fp8_kv: bool = False         # K/V chunks travel as e4m3 bytes + per-(b,h,token) scales
    payload: Optional[Tuple[int, int]] = None  # FP8 All-to-All payload [rows, cols]
    payload_dtype: str = "bf16"

    @property
    def S(self) -> int:
        return int(sum(self.chunk_len))

    @property
    def W(self) -> int:
        return len(self.chunk_len)

    def attn_flops(self) -> float:
        """Algorithmic flops: two contractions, 2 flop per multiply-add."""
        return 4.0 * self.B * self.H * self.Sq * self.S * self.d


WORKLOADS: Dict[str, Workload] = {
    # tiny: ring degree 2, fp32 inputs, rank-0 Q shard
    "tiny": Workload("tiny", 0, 1, 2, 64, 128, (128, 128), "f32",
                     payload=(256, 128), payload_dtype="f32"),
    # FLUX-1024 shard, Ulysses only: 4096 image + 512 text tokens, one KV chunk
    "flux1024_u": Workload("flux1024_u", 1, 1, 24, 128, 4608, (4608,), "bf16",
                           k_mul=0.5, payload=(4608, 3072)),
    # FLUX-1024 shard, ring degree 4, K/V payload FP8 per step
    "flux1024_r4": Workload("flux1024_r4", 2, 1, 24, 128, 1152, (1152,) * 4, "bf16",
                            fp8_kv=True),
    # FLUX-2048 shard, Ulysses 2 x ring 8
    "flux2048_u2r8": Workload("flux2048_u2r8", 3, 1, 12, 128, 2112, (2112,) * 8, "bf16",
                              head_scale=True),
    # Qwen-Image-like shard: 6889 image + 1303 text tokens, last floor(0.3*1303)=390
    # text keys are padding, 1% of entries are x20 outliers, FP8 K/V
    "qwen_r2": Workload("qwen_r2", 4, 1, 24, 128, 4096, (4096, 4096), "bf16",
                        outlier_frac=0.01, outlier_mul=20.0,
                        masked_keys=(8192 - 390, 8192), fp8_kv=True),
}


@dataclass
class AttnInputs:
    wl: Workload
    q: np.ndarray                 # float32 [B,H,Sq,d] (bf16-exact when wl.dtype == "bf16")
    k: List[np.ndarray]           # per chunk float32 [B,H,Sc,d]
    v: List[np.ndarray]
    key_mask: Optional[List[np.ndarray]]  # per chunk uint8 [B,Sc], 1 = keep; None if no mask
    softmax_scale: np.float32 = field(default=np.float32(0))


def _draw(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.standard_normal(size=shape, dtype=np.float32)


def make_attention_inputs(wl: Workload, *, heads: Optional[int] = None,
                          sq: Optional[int] = None) -> AttnInputs:
    """Draw Q and the KV chunks for one workload.

    `heads` / `sq` shrink the number of heads / local queries (for sampled parity
    checks at full KV length); the draw then covers only that smaller shape.
    """
    H = wl.H if heads is None else heads
    Sq = wl.Sq if sq is None else sq
    rng = np.random.Generator(np.random.PCG64(wl.seed))
    q = _draw(rng, (wl.B, H, Sq, wl.d))
    k = _draw(rng, (wl.B, H, wl.S, wl.d))
    v = _draw(rng, (wl.B, H, wl.S, wl.d))
    if wl.k_mul != 1.0:
        k *= np.float32(wl.k_mul)
    if wl.head_scale:
        c = rng.uniform(0.5, 2.0, size=(1, H, 1, 1)).astype(np.float32)
        q *= c
        k *= c
        v *= c
    if wl.outlier_frac > 0.0:
        for t in (q, k, v):
            hit = rng.random(size=t.shape, dtype=np.float32) < np.float32(wl.outlier_frac)
            t[hit] *= np.float32(wl.outlier_mul)
    if wl.dtype == "bf16":
        q = bf16_bits_to_f32(f32_to_bf16_bits(q))
        k = bf16_bits_to_f32(f32_to_bf16_bits(k))
        v = bf16_bits_to_f32(f32_to_bf16_bits(v))
    ks, vs, ms = [], [], []
    lo = 0
    mlo, mhi = wl.masked_keys
    for L in wl.chunk_len:
        ks.append(np.ascontiguousarray(k[:, :, lo:lo + L, :]))
        vs.append(np.ascontiguousarray(v[:, :, lo:lo + L, :]))
        m = np.ones((wl.B, L), dtype=np.uint8)
        a, b = max(mlo, lo), min(mhi, lo + L)
        if b > a:
            m[:, a - lo:b - lo] = 0
        ms.append(m)
        lo += L
    has_mask = mhi > mlo
    scale = np.float32(1.0) / np.sqrt(np.float32(wl.d))
    return AttnInputs(wl, q, ks, vs, ms if has_mask else None, np.float32(scale))


def make_payload(wl: Workload, *, rows: Optional[int] = None) -> np.ndarray:
    """FP8 All-to-All payload matrix [rows, cols] as float32 (bf16-exact if bf16)."""
    assert wl.payload is not None
    R, C = wl.payload
    if rows is not None:
        R = rows
    rng = np.random.Generator(np.random.PCG64(wl.seed + 1000))
    x = _draw(rng, (R, C))
    if wl.payload_dtype == "bf16":
        x = bf16_bits_to_f32(f32_to_bf16_bits(x))
    return x


def make_matrix(seed: int, rows: int, cols: int, dtype: str = "bf16",
                kind: str = "normal") -> np.ndarray:
    """Generic seeded [rows, cols] matrix for FP8 edge-case tests.

    kind: "normal" N(0,1); "wide" N(0,1) * 2**U(-20,20) per row (tests the scale
    path over many binades); "zero_rows" N(0,1) with every third row all-zero.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    x = _draw(rng, (rows, cols))
    if kind == "wide":
        e = rng.integers(-20, 21, size=(rows, 1)).astype(np.float32)
        x = x * np.exp2(e).astype(np.float32)
    elif kind == "zero_rows":
        x[::3, :] = 0.0
    if dtype == "bf16":
        x = bf16_bits_to_f32(f32_to_bf16_bits(x))
    return x


def sample_rows(seed: int, n_total: int, n_pick: int) -> np.ndarray:
    """Sorted seeded sample (without replacement) of row indices in [0, n_total)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n_pick = min(n_pick, n_total)
    return np.sort(rng.choice(n_total, size=n_pick, replace=False)).astype(np.int64)
