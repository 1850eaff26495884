"""fp64 CPU oracle for one rank's share of USP attention and its FP8 payloads.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
module; only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg do.
It shares no code with the HIP path (no kernels, headers, tables or helpers) and
imports nothing from it.

Everything here is the plain definition written out with numpy in float64
(float32 only where the method itself fixes fp32: the FP8 scale arithmetic).
No tiling, no online softmax, no fusion.

What each function follows (paper = FastUSP, arXiv 2602.10940):
  attention()          section 2.2, softmax(Q K^T / sqrt(d)) V, plus the
                       log-sum-exp of each score row (section 2.2.2)
  lse_merge()          section 3.4, the two merge equations below Algorithm 2
                       (exponent-difference form)
  lse_merge_raw()      section 2.2.2, the same merge in its raw exp() form
  ring_attention()     section 2.2.2 / Algorithm 2: per-chunk attention folded
                       with the merge, chunks in a caller-chosen order
  e4m3fn_*             the FP8 E4M3 format named in section 3.3 (range +-448,
                       i.e. the OCP "fn" variant: no infinities, one NaN code)
  fp8_quant()/fp8_dequant()   Algorithm 1 lines 1-2 and 4, with one scale per
                       row of the 2-D view (per token)
  fp8_quant_mapped()/fp8_dequant_mapped()   the same two steps with the rows
                       gathered from / scattered to the layouts on either side
                       of the All-to-All of section 2.2.1 ([B,H,S/N,D] <->
                       [B,H/N,S,D]): a row permutation around fp8_quant /
                       fp8_dequant, nothing else

Readings taken where the paper is silent are listed in the repository's design
notes; the ones that matter here:
  * log is the natural log; lse is m + ln(sum exp(s - m)).
  * a row with every key masked has lse = -inf and O = 0.
  * scale s = absmax / 448 in IEEE float32; s == 0 (all-zero row) is replaced by
    1.0; x / s is a true IEEE float32 division; the cast rounds to nearest even
    and saturates to +-448; dequantisation multiplies in float32.

Pins (tests/test_oracle_*.py, none of them re-types these formulas): mpmath
brute force on tiny shapes, closed forms (equal keys, Q = 0, constant V, shift
invariance, a dominant key), torch's fp64 scaled_dot_product_attention and
logsumexp, chunk-order invariance over every permutation, merge-tree
associativity, raw-form == difference-form merge, the OCP E4M3 value table facts
(448, 2^-9, 2^-6, NaN codes, monotonicity), torch.float8_e4m3fn casts inside
+-448, encode(decode(b)) == b, tie and saturation cases, per-row invariants of
the quantiser and its provable round-trip bound; dequant_exact_f64 (what an FP8
K/V chunk means as numbers) against exact rationals, against the fp32
dequantiser it must round to in one step, and on a [B,H,L,d] case with a
different scale per (b, h, token); for the mapped variants the
identity with numpy transposes of the plain result, and a four-rank emulation
of the exchange of section 2.2.1 (8 heads, 1024 tokens: [B,8,256,D] ->
[B,2,1024,D] and back).
The paper's "<0.1% precision loss" has no stated metric: parity unpinned for
that figure (only aggregate readings of it are asserted).
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np

FP8_MAX = 448.0  # section 3.3: E4M3 dynamic range +-448


# ---------------------------------------------------------------------------
# attention, section 2.2
# ---------------------------------------------------------------------------
def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float,
              key_mask: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """One-shot attention of q [B,H,Sq,d] over k, v [B,H,S,d] (all widened to fp64).

    scale multiplies the scores (1/sqrt(d) in the paper).  key_mask [B,S], nonzero =
    keep, masks keys for every query.  Returns (O [B,H,Sq,d], lse [B,H,Sq]).
    Two passes per score row: max, then exp/sum; nothing is chunked.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, H, Sq, d = q.shape
    out = np.zeros((B, H, Sq, v.shape[-1]), dtype=np.float64)
    lse = np.full((B, H, Sq), -np.inf, dtype=np.float64)
    sc = np.float64(scale)
    for b in range(B):
        keep = None if key_mask is None else (np.asarray(key_mask[b]) != 0)
        for h in range(H):
            s = (q[b, h] @ k[b, h].T) * sc                     # [Sq, S]
            if keep is not None:
                s = np.where(keep[None, :], s, -np.inf)
            if s.shape[1] == 0:
                continue
            M = s.max(axis=1)                                   # [Sq]
            live = np.isfinite(M)                               # rows with >=1 unmasked key
            Msafe = np.where(live, M, 0.0)
            p = np.exp(s - Msafe[:, None])                      # masked keys -> exp(-inf) = 0
            L = p.sum(axis=1)
            o = p @ v[b, h]
            Lsafe = np.where(live, L, 1.0)
            out[b, h] = np.where(live[:, None], o / Lsafe[:, None], 0.0)
            lse[b, h] = np.where(live, Msafe + np.log(Lsafe), -np.inf)
    return out, lse


# ---------------------------------------------------------------------------
# LSE merge, section 3.4 (difference form) and section 2.2.2 (raw form)
# ---------------------------------------------------------------------------
def lse_merge(o1: np.ndarray, lse1: np.ndarray, o2: np.ndarray, lse2: np.ndarray
              ) -> Tuple[np.ndarray, np.ndarray]:
    """lse = log(e^lse1 + e^lse2);  O = e^(lse1-lse) O1 + e^(lse2-lse) O2.

    o* [..., d], lse* [...].  lse = -inf on both sides gives lse = -inf, O = 0.
    """
    o1 = np.asarray(o1, dtype=np.float64)
    o2 = np.asarray(o2, dtype=np.float64)
    a = np.asarray(lse1, dtype=np.float64)
    b = np.asarray(lse2, dtype=np.float64)
    m = np.maximum(a, b)
    dead = np.isneginf(m)
    ms = np.where(dead, 0.0, m)
    with np.errstate(divide="ignore"):
        lse = ms + np.log(np.exp(a - ms) + np.exp(b - ms))
    lse = np.where(dead, -np.inf, lse)
    ls = np.where(dead, 0.0, lse)
    w1 = np.where(dead, 0.0, np.exp(a - ls))
    w2 = np.where(dead, 0.0, np.exp(b - ls))
    return w1[..., None] * o1 + w2[..., None] * o2, lse


def lse_merge_raw(o1, lse1, o2, lse2):
    """The merge exactly as first printed: raw exp(lse) sums and a division.

    Only usable for moderate |lse| (it overflows past ~709 in fp64); kept as an
    independent second form to check lse_merge() against.
    """
    o1 = np.asarray(o1, dtype=np.float64)
    o2 = np.asarray(o2, dtype=np.float64)
    e1 = np.exp(np.asarray(lse1, dtype=np.float64))
    e2 = np.exp(np.asarray(lse2, dtype=np.float64))
    tot = e1 + e2
    return (e1[..., None] * o1 + e2[..., None] * o2) / tot[..., None], np.log(tot)


def ring_attention(q: np.ndarray, k_chunks: Sequence[np.ndarray], v_chunks: Sequence[np.ndarray],
                   scale: float, key_masks: Optional[Sequence[np.ndarray]] = None,
                   order: Optional[Sequence[int]] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Algorithm 2 without the transport: attention per KV chunk, folded by lse_merge.

    `order` is the sequence in which chunks are visited (default ring order 0..W-1).
    """
    W = len(k_chunks)
    order = list(range(W)) if order is None else list(order)
    o = lse = None
    for r in order:
        m = None if key_masks is None else key_masks[r]
        o_r, lse_r = attention(q, k_chunks[r], v_chunks[r], scale, m)
        if o is None:
            o, lse = o_r, lse_r
        else:
            o, lse = lse_merge(o, lse, o_r, lse_r)
    return o, lse


# ---------------------------------------------------------------------------
# FP8 E4M3 (fn) codec from the format's definition
# ---------------------------------------------------------------------------
def e4m3fn_decode_table() -> np.ndarray:
    """Value of each of the 256 byte codes: 1 sign, 4 exponent (bias 7), 3 mantissa bits.

    exponent field 0: subnormal, 2^-6 * (m/8); otherwise 2^(e-7) * (1 + m/8);
    the all-ones exponent+mantissa code (0x7F / 0xFF) is NaN; there is no infinity.
    """
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            val = np.nan
        elif e == 0:
            val = sign * (2.0 ** -6) * (m / 8.0)
        else:
            val = sign * (2.0 ** (e - 7)) * (1.0 + m / 8.0)
        t[code] = val
    return t


_DEC = e4m3fn_decode_table()
_MAG = _DEC[:0x7F].copy()          # 127 non-negative finite magnitudes, ascending, code == index


def e4m3fn_decode(codes: np.ndarray) -> np.ndarray:
    return _DEC[np.asarray(codes, dtype=np.uint8)]


def e4m3fn_encode(t: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code of each float32 in t: ties to the even code, saturating at +-448.

    A magnitude above 448 has no finite code above it, so it saturates to 0x7E whether
    it would have rounded down or up.  NaN maps to 0x7F with the input's sign bit.
    """
    t = np.asarray(t, dtype=np.float32)
    mag = np.abs(t.astype(np.float64))
    nan = np.isnan(mag)
    mag = np.where(nan, 0.0, mag)
    hi = np.searchsorted(_MAG, mag, side="left")            # first code with value >= mag
    hi = np.minimum(hi, 0x7E)
    lo = np.maximum(hi - 1, 0)
    d_hi = np.abs(_MAG[hi] - mag)
    d_lo = np.abs(mag - _MAG[lo])
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi)
    code = np.where(mag > FP8_MAX, 0x7E, code)
    code = np.where(nan, 0x7F, code).astype(np.uint8)
    sign = np.signbit(t).astype(np.uint8) << 7
    return (code | sign).astype(np.uint8)


# ---------------------------------------------------------------------------
# per-row FP8 quantise / dequantise, Algorithm 1 lines 1-2 and 4
# ---------------------------------------------------------------------------
def fp8_quant(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """x [rows, cols] float32 (or bf16-exact float32) -> (codes uint8, scales float32 [rows])."""
    x = np.asarray(x, dtype=np.float32)
    assert x.ndim == 2
    if x.shape[1] == 0:
        return np.zeros(x.shape, np.uint8), np.ones(x.shape[0], np.float32)
    a = np.max(np.abs(x), axis=1).astype(np.float32)
    with np.errstate(under="ignore"):
        s = (a / np.float32(FP8_MAX)).astype(np.float32)     # IEEE fp32 division
    s = np.where(s == 0, np.float32(1.0), s).astype(np.float32)
    with np.errstate(over="ignore", invalid="ignore"):
        t = (x / s[:, None]).astype(np.float32)              # IEEE fp32 division
    return e4m3fn_encode(t), s


def fp8_dequant(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """y = float32(decode(code)) * scale, product rounded once in float32."""
    val = e4m3fn_decode(codes).astype(np.float32)            # exact: every code fits fp32
    return (val * np.asarray(scales, dtype=np.float32)[:, None]).astype(np.float32)


def round_to_bf16(y: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), nearest-even on the 16 dropped bits."""
    y = np.ascontiguousarray(y, dtype=np.float32)
    u = y.view(np.uint32).astype(np.uint64)
    keep = u >> 16
    rem = u & 0xFFFF
    up = (rem > 0x8000) | ((rem == 0x8000) & ((keep & 1) == 1))
    isnan = np.isnan(y)
    out = (keep + up.astype(np.uint64)).astype(np.uint16)
    return np.where(isnan, np.uint16(0x7FC0), out).astype(np.uint16)


def fp8_dequant_bf16(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """Dequantise to bf16: the float32 product above, then rounded to bf16 bits."""
    return round_to_bf16(fp8_dequant(codes, scales))


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def dequant_exact_f64(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """decode(code) * scale in fp64 (exact): what an FP8 K/V chunk means as numbers."""
    return e4m3fn_decode(codes) * np.asarray(scales, dtype=np.float64)[..., None]


# ---------------------------------------------------------------------------
# Algorithm 1 around the All-to-All of section 2.2.1: rows visited as a 4-D index
# ---------------------------------------------------------------------------
def row_map_offsets(n: Sequence[int], strides: Sequence[int]) -> np.ndarray:
    """Offset sum_k i_k * strides[k] of every index (i0, i1, i2, i3), i3 fastest."""
    idx = np.indices(tuple(int(x) for x in n), dtype=np.int64).reshape(4, -1)
    return (idx * np.asarray(strides, dtype=np.int64)[:, None]).sum(axis=0)


def fp8_quant_mapped(x_flat: np.ndarray, n: Sequence[int], src_stride: Sequence[int],
                     dst_row_stride: Sequence[int], cols: int) -> Tuple[np.ndarray, np.ndarray]:
    """Row (i0..i3) is x_flat[sum i_k src_stride[k] : +cols]; its codes and scale go to row
    sum i_k dst_row_stride[k] of the dense [rows, cols] / [rows] outputs."""
    src = row_map_offsets(n, src_stride)
    dst = row_map_offsets(n, dst_row_stride)
    rows = np.asarray(x_flat, dtype=np.float32).reshape(-1)[src[:, None] + np.arange(cols)[None, :]]
    q, s = fp8_quant(rows)
    total = int(np.prod(n))
    assert sorted(dst.tolist()) == list(range(total)), "destination rows must be a permutation"
    q_out = np.empty((total, cols), dtype=np.uint8)
    s_out = np.empty((total,), dtype=np.float32)
    q_out[dst] = q
    s_out[dst] = s
    return q_out, s_out


def fp8_dequant_mapped(codes: np.ndarray, scales: np.ndarray, n: Sequence[int],
                       src_row_stride: Sequence[int], dst_stride: Sequence[int], cols: int,
                       out_elems: int, to_bf16: bool) -> np.ndarray:
    """Row (i0..i3) is read at row sum i_k src_row_stride[k] of codes / scales and written to
    y_flat[sum i_k dst_stride[k] : +cols]; elements no row maps to stay 0."""
    src = row_map_offsets(n, src_row_stride)
    dst = row_map_offsets(n, dst_stride)
    y = fp8_dequant(codes[src], scales[src])
    if to_bf16:   # the bf16-rounded values, held as float32
        y = bf16_bits_to_f64(round_to_bf16(y)).astype(np.float32)
    out = np.zeros((out_elems,), dtype=np.float32)
    out[dst[:, None] + np.arange(cols)[None, :]] = y
    return out
