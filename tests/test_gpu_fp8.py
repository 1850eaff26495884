"""FP8 pack/unpack parity: HIP kernels (through the C ABI) vs the oracle, bit-exact."""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from paper_2602_10940_amd import workloads as W
from tests.gpu_util import DEV, dev_bf16, dev_f32, host_bits_bf16

pytestmark = pytest.mark.gpu


def _usp():
    import paper_2602_10940_amd as P
    return P


def _check_quant(x32, dtype):
    P = _usp()
    xd = dev_bf16(x32) if dtype == "bf16" else dev_f32(x32)
    q, s = P.usp_fp8_quant(xd)
    torch.cuda.synchronize()
    eq, es = orc.fp8_quant(x32)
    np.testing.assert_array_equal(s.cpu().numpy().view(np.uint32), es.view(np.uint32))
    gq = q.cpu().numpy()
    bad = np.argwhere(gq != eq)
    assert bad.size == 0, "first mismatches %s got %s exp %s x %s s %s" % (
        bad[:5], gq[tuple(bad[:5].T)], eq[tuple(bad[:5].T)], x32[tuple(bad[:5].T)], es[bad[:5, 0]])
    return q, s, eq, es


@pytest.mark.parametrize("rows,cols,dtype", [
    (256, 128, "f32"),        # tiny config payload
    (256, 128, "bf16"),
    (37, 8, "bf16"), (5, 64, "f32"), (129, 136, "bf16"), (3, 256, "bf16"), (66, 520, "f32"),
    (19, 1000, "bf16"), (7, 2048, "bf16"), (50, 3072, "bf16"), (9, 4096, "f32"),
    (3, 4104, "bf16"), (2, 20000, "bf16"),      # long-row kernel
    (1, 65536, "bf16"),                          # per-tensor scale = one row
    (1001, 128, "bf16"),                         # ring K/V view, ragged row count
    (1, 1 << 22, "bf16"), (3, 500008, "f32"),    # few very long rows: chunked over the whole chip
    (600, 8200, "bf16"), (1030, 4104, "bf16"),   # both sides of the rows threshold of that path
])
def test_quant_bit_exact(rows, cols, dtype):
    x = W.make_matrix(100 + rows + cols, rows, cols, dtype, "wide" if rows % 2 else "normal")
    _check_quant(x, dtype)


def test_quant_tiny_workload_payload():
    x = W.make_payload(W.WORKLOADS["tiny"])
    _check_quant(x, "f32")


def test_quant_zero_rows_negative_zero_and_empty():
    P = _usp()
    x = W.make_matrix(5, 12, 64, "f32", "zero_rows")
    x[0, 5] = -0.0
    q, s, eq, es = _check_quant(x, "f32")
    assert q[0, 5].item() == 0x80
    q0, s0 = P.usp_fp8_quant(torch.empty((0, 64), dtype=torch.bfloat16, device=DEV))
    assert q0.shape == (0, 64)
    q1, s1 = P.usp_fp8_quant(torch.empty((5, 0), dtype=torch.bfloat16, device=DEV))
    torch.cuda.synchronize()
    assert torch.all(s1 == 1.0)


def test_quant_denormal_scales():
    # absmax so small that absmax/448 is a float32 denormal: the division must stay IEEE
    x = W.make_matrix(6, 64, 32, "f32")
    x *= np.float32(1e-37)
    x[::4] *= np.float32(1e-5)
    _check_quant(x, "f32")


def test_converter_every_rounding_boundary():
    """Row absmax exactly 448 makes the scale 1.0, so the cast sees x itself: sweep every
    float32 whose low 16 bits are at / next to a tie, for all high halves with |x| <= 448."""
    hi = np.arange(0, 0x43E0 + 1, dtype=np.uint32)
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=np.uint32)
    bits = ((hi[:, None] << 16) | lows[None, :]).reshape(-1)
    vals = bits.view(np.float32)
    vals = vals[np.abs(vals) <= 448.0]
    vals = np.concatenate([vals, -vals])
    pad = (-len(vals)) % 7
    vals = np.concatenate([vals, np.zeros(pad, np.float32)])
    x = np.empty((len(vals) // 7, 8), np.float32)
    x[:, 0] = 448.0
    x[:, 1:] = vals.reshape(-1, 7)
    q, s, eq, es = _check_quant(x, "f32")
    assert np.all(es == 1.0)


def test_converter_exhaustive_every_float32_up_to_448():
    """Every float32 bit pattern with |x| <= 448, both signs (2.28e9 values), through the row
    kernel with scale 1.0 (each row starts with 448).  The expected code comes from the oracle:
    its encoder is a step function of the magnitude, so the 126 smallest float32 values at which
    it steps (found by bisection on the oracle, and verified on both sides of each step) define
    it everywhere; the device only looks the values up in that table."""
    P = _usp()
    enc = lambda b: int(orc.e4m3fn_encode(np.array([b], np.uint32).view(np.float32))[0])
    top = 0x43E00000                                   # 448.0f
    assert enc(top) == 0x7E and enc(0) == 0
    steps = []
    for c in range(1, 0x7F):
        lo, hi = 0, top                                # smallest bits with code >= c
        while lo < hi:
            mid = (lo + hi) // 2
            if enc(mid) >= c:
                hi = mid
            else:
                lo = mid + 1
        assert enc(lo) == c and enc(lo - 1) == c - 1
        steps.append(lo)
    # the oracle really is monotone between its steps (sampled)
    rng = np.random.Generator(np.random.PCG64(5))
    sample = np.sort(rng.integers(0, top + 1, 200000).astype(np.uint32))
    codes = orc.e4m3fn_encode(sample.view(np.float32)).astype(np.int64)
    assert np.all(np.diff(codes) >= 0)
    np.testing.assert_array_equal(codes, np.searchsorted(np.array(steps, np.uint32), sample, side="right"))

    steps_d = torch.tensor(steps, dtype=torch.int32, device=DEV)
    per_row, rows = 2040, 32768
    lead = torch.zeros((rows, 8), dtype=torch.float32, device=DEV)
    lead[:, 0] = 448.0
    for start in range(0, top + 1, per_row * rows):
        n = min(per_row * rows, top + 1 - start)
        bits = torch.arange(start, start + per_row * rows, dtype=torch.int32, device=DEV)
        bits[n:] = 0                                   # past 448: pad with +0
        want = torch.bucketize(bits, steps_d, right=True).to(torch.uint8).reshape(rows, per_row)
        mag = bits.view(torch.float32).reshape(rows, per_row)
        for sign, neg in ((1.0, 0), (-1.0, 0x80)):
            x = torch.cat([lead, mag * sign], dim=1).contiguous()
            q, sc = P.usp_fp8_quant(x)
            assert bool((sc == 1.0).all())
            bad = (q[:, 8:] != (want | neg)).nonzero()
            assert bad.numel() == 0, (start, sign, bad[:4].tolist())


def test_division_exact_next_to_every_rounding_boundary():
    """Arbitrary scales: for 256 seeded absmax values, every row holds x = fl(mid * s) shifted by
    -2..+2 ulps for each of the 126 midpoints between adjacent E4M3 magnitudes, so x / s lands on
    or next to every rounding boundary and a quotient off by one ulp would flip a code."""
    rng = np.random.Generator(np.random.PCG64(77))
    tab = orc.e4m3fn_decode_table()[:0x7F]
    mids = ((tab[:-1] + tab[1:]) / 2).astype(np.float32)            # 126 boundaries, exact in fp32
    amax = (rng.uniform(1.0, 2.0, 256) * np.exp2(rng.integers(-40, 40, 256))).astype(np.float32)
    s = (amax / np.float32(448)).astype(np.float32)
    base = (mids[None, :] * s[:, None]).astype(np.float32)          # [256, 126]
    cols = [amax[:, None]]
    for k in (-2, -1, 0, 1, 2):
        v = base.copy()
        for _ in range(abs(k)):
            v = np.nextafter(v, np.float32(np.inf) if k > 0 else np.float32(0))
        cols += [v, -v]
    x = np.concatenate(cols, axis=1)
    pad = (-x.shape[1]) % 8
    x = np.concatenate([x, np.zeros((x.shape[0], pad), np.float32)], axis=1).astype(np.float32)
    assert np.all(np.abs(x[:, 1:]) < amax[:, None])
    _check_quant(x, "f32")


def test_dequant_all_codes_and_bit_exact():
    P = _usp()
    codes = np.arange(256, dtype=np.uint8).reshape(1, 256).repeat(4, 0)
    codes[:, 0x7F] = 0x7E     # NaN codes never come out of the quantiser
    codes[:, 0xFF] = 0xFE
    scales = np.array([1.0, 0.37, 3.1e-3, 1.7e4], np.float32)
    qd = torch.from_numpy(codes).to(DEV)
    sd = torch.from_numpy(scales).to(DEV)
    y32 = P.usp_fp8_dequant(qd, sd, torch.float32)
    y16 = P.usp_fp8_dequant(qd, sd, torch.bfloat16)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(y32.cpu().numpy().view(np.uint32), orc.fp8_dequant(codes, scales).view(np.uint32))
    np.testing.assert_array_equal(host_bits_bf16(y16), orc.fp8_dequant_bf16(codes, scales))


@pytest.mark.parametrize("rows,cols", [(256, 128), (33, 8), (17, 24), (64, 3072), (1001, 128), (2, 20000)])
def test_roundtrip_bit_exact(rows, cols):
    P = _usp()
    x = W.make_matrix(7 + rows, rows, cols, "bf16", "wide")
    q, s = P.usp_fp8_quant(dev_bf16(x))
    y16 = P.usp_fp8_dequant(q, s, torch.bfloat16)
    y32 = P.usp_fp8_dequant(q, s, torch.float32)
    torch.cuda.synchronize()
    eq, es = orc.fp8_quant(x)
    np.testing.assert_array_equal(q.cpu().numpy(), eq)
    np.testing.assert_array_equal(host_bits_bf16(y16), orc.fp8_dequant_bf16(eq, es))
    np.testing.assert_array_equal(y32.cpu().numpy().view(np.uint32), orc.fp8_dequant(eq, es).view(np.uint32))


def test_full_size_flux_payload_every_byte():
    """FLUX-1024 All-to-All payload [4608, 3072] bf16 in the launch configuration the bench
    times; every scale, every code and every dequantised bf16 is checked against the oracle."""
    P = _usp()
    wl = W.WORKLOADS["flux1024_u"]
    x = W.make_payload(wl)
    q, s = P.usp_fp8_quant(dev_bf16(x))
    y = P.usp_fp8_dequant(q, s, torch.bfloat16)
    torch.cuda.synchronize()
    eq, es = orc.fp8_quant(x)
    np.testing.assert_array_equal(s.cpu().numpy().view(np.uint32), es.view(np.uint32))
    np.testing.assert_array_equal(q.cpu().numpy(), eq)
    np.testing.assert_array_equal(host_bits_bf16(y), orc.fp8_dequant_bf16(eq, es))
    assert q.numel() * 2 == x.size * 2 and q.element_size() == 1   # half the bf16 volume


# ---------------------------------------------------------------------------
# pack / unpack in the layouts on either side of the All-to-All (section 2.2.1)
# ---------------------------------------------------------------------------
def _a2a_maps(N, B, H, S_loc, D):
    Hn, S = H // N, N * S_loc
    return {"n": (N, B, Hn, S_loc), "dense": (B * Hn * S_loc, Hn * S_loc, S_loc, 1),
            "seq_sharded": (Hn * S_loc * D, H * S_loc * D, S_loc * D, D),    # into [B,H,S_loc,D]
            "head_sharded": (S_loc * D, Hn * S * D, S * D, D)}               # into [B,Hn,S,D]


@pytest.mark.parametrize("N,B,H,S_loc,D,dtype", [
    (4, 2, 8, 37, 128, "bf16"), (2, 1, 6, 100, 64, "bf16"), (8, 1, 24, 9, 128, "f32"), (3, 2, 3, 5, 4096, "bf16"),
])
def test_mapped_pack_and_unpack_bit_exact(N, B, H, S_loc, D, dtype):
    P = _usp()
    m = _a2a_maps(N, B, H, S_loc, D)
    Hn, S = H // N, N * S_loc
    up = dev_bf16 if dtype == "bf16" else dev_f32
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    for side, shape in (("seq_sharded", (B, H, S_loc, D)), ("head_sharded", (B, Hn, S, D))):
        x = W.make_matrix(300 + N + S_loc, int(np.prod(shape[:-1])), D, dtype, "wide").reshape(shape)
        q, s = P.usp_fp8_quant_mapped(up(x), m["n"], m[side], m["dense"], D)
        torch.cuda.synchronize()
        eq, es = orc.fp8_quant_mapped(x, m["n"], m[side], m["dense"], D)
        np.testing.assert_array_equal(q.cpu().numpy(), eq)
        np.testing.assert_array_equal(s.cpu().numpy().view(np.uint32), es.view(np.uint32))
        y = torch.zeros(shape, dtype=tdt, device=DEV)
        P.usp_fp8_dequant_mapped(q, s, m["n"], m["dense"], m[side], y)
        torch.cuda.synchronize()
        ey = orc.fp8_dequant_mapped(eq, es, m["n"], m["dense"], m[side], D, x.size, to_bf16=(dtype == "bf16"))
        got = host_bits_bf16(y).reshape(-1) if dtype == "bf16" else y.cpu().numpy().view(np.uint32).reshape(-1)
        exp = W.f32_to_bf16_bits(ey) if dtype == "bf16" else ey.view(np.uint32)
        np.testing.assert_array_equal(got, exp.reshape(-1))


def test_four_rank_exchange_on_one_gpu():
    """Section 2.2.1's example (4 ranks, 8 heads, 1024 tokens) with the ranks played in turn by one
    GPU and the all_to_all by block slicing: [B,8,256,D] -> [B,2,1024,D], bit-equal to quantising
    and dequantising the whole [B,8,1024,D] tensor row by row."""
    P = _usp()
    N, B, H, S_loc, D = 4, 1, 8, 256, 128
    Hn, S = H // N, N * S_loc
    m = _a2a_maps(N, B, H, S_loc, D)
    full = W.make_matrix(77, B * H * S, D, "bf16").reshape(B, H, S, D)
    xs = [np.ascontiguousarray(full[:, :, r * S_loc:(r + 1) * S_loc]) for r in range(N)]
    send = [P.usp_fp8_quant_mapped(dev_bf16(x), m["n"], m["seq_sharded"], m["dense"], D) for x in xs]
    fq, fs = orc.fp8_quant(full.reshape(-1, D))
    want = orc.fp8_dequant_bf16(fq, fs).reshape(B, H, S, D)      # bf16 bit patterns
    blk = B * Hn * S_loc
    for r in range(N):
        rq = torch.cat([send[src][0][r * blk:(r + 1) * blk] for src in range(N)])
        rs = torch.cat([send[src][1][r * blk:(r + 1) * blk] for src in range(N)])
        y = torch.zeros((B, Hn, S, D), dtype=torch.bfloat16, device=DEV)
        P.usp_fp8_dequant_mapped(rq, rs, m["n"], m["dense"], m["head_sharded"], y)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host_bits_bf16(y), want[:, r * Hn:(r + 1) * Hn])


def test_mapped_arguments_are_checked():
    P = _usp()
    x = torch.zeros((4, 8, 16), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(P.UspError):     # row stride of 4 bf16 = 8 bytes: rows not 16-byte aligned
        P.usp_fp8_quant_mapped(x, (1, 1, 4, 8), (0, 0, 128, 4), (32, 32, 8, 1), 16)
    with pytest.raises(P.UspError):     # cols beyond the single-pass kernel
        P.usp_fp8_quant_mapped(x, (1, 1, 1, 1), (0, 0, 0, 0), (1, 1, 1, 1), 8192)
