"""libusp_diag.so: the diagnostic MFMA-rate kernel runs and computes what it claims to, and the
give-up path of the one-launch ring's bounded arrival wait, driven from the host (a count that is
never reached, a short poll limit; every kernel runs to its end), returns NaN rows."""
import numpy as np
import pytest
import torch

from tests.gpu_util import DEV

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [0, 1])
def test_probe_constant_operands_sum_exactly(shape):
    from paper_2602_10940_amd import diag as P
    wgs, iters = 6, 10
    out = torch.full((wgs * 512,), -1.0, dtype=torch.float32, device=DEV)
    clocks = torch.zeros((2,), dtype=torch.int64, device=DEV)
    P.usp_diag_mfma_rate(wgs, iters, False, out, clocks, shape=shape)
    torch.cuda.synchronize()
    # A = 1, B = 0.5.  32x32x16: one MFMA adds 16 * 0.5 to each of a lane's 16 accumulator elements; an
    # accumulator takes 8 MFMAs per iteration; a thread sums its 4 accumulators.  16x16x32: 32 * 0.5 to each
    # of 4 elements, 8 MFMAs per accumulator and iteration, 8 accumulators: the same total
    want = 4 * 16 * 8 * 8.0 * iters
    assert torch.all(out == want), (out.min().item(), out.max().item(), want)
    cyc, ticks = [int(v) for v in clocks.cpu()]
    assert cyc > 0 and ticks > 0
    assert 200.0 < cyc / ticks * 100.0 < 3000.0   # shader clock in MHz


def test_probe_random_operands_finite():
    from paper_2602_10940_amd import diag as P
    out = torch.empty((4 * 512,), dtype=torch.float32, device=DEV)
    clocks = torch.zeros((2,), dtype=torch.int64, device=DEV)
    P.usp_diag_mfma_rate(4, 50, True, out, clocks)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and out.abs().max() > 0


def test_probe_rejects_bad_arguments():
    import paper_2602_10940_amd as U
    from paper_2602_10940_amd import diag as P
    out = torch.empty((512,), dtype=torch.float32, device=DEV)
    clocks = torch.zeros((2,), dtype=torch.int64, device=DEV)
    with pytest.raises(U.UspError):
        P.usp_diag_mfma_rate(1, 0, True, out, clocks)


def test_short_bf16_division_gives_the_codes_of_the_ieee_division_for_every_pair():
    """Algorithm 1 line 2 with bf16 inputs: the pack's short sequence against the true division, over
    every (row absmax a, element x) pair of bf16 values with |x| <= a (both signs, packed in both byte
    positions of the encoder), on the device.  The reference side of this comparison (the compiler's IEEE
    division and the hardware's E4M3 convert) is what the oracle-against-kernel tests of test_gpu_fp8.py
    pin for every fp32 in range and next to every rounding boundary."""
    from paper_2602_10940_amd import diag
    pairs, bad_codes, bad_quot, slow_rows = diag.usp_diag_check_bf16_division()
    # a = 0x0001 .. 0x7f7f: a values in the fast range contribute 2 * (abits + 1) pairs each
    assert slow_rows > 0 and slow_rows < 0x7f7f // 2 + 2000
    assert pairs > 500_000_000
    assert bad_codes == 0, (pairs, bad_codes, bad_quot)
    assert bad_quot < pairs // 100          # the quotients themselves do differ now and then (last bit)


def test_payload_floor_kernels_run():
    from paper_2602_10940_amd import diag
    x = torch.randn((64, 3072), device=DEV).to(torch.bfloat16)
    q = torch.zeros((64, 3072), dtype=torch.uint8, device=DEV)
    s = torch.zeros((64,), dtype=torch.float32, device=DEV)
    diag.usp_diag_payload_floor(0, x, q, s)
    diag.usp_diag_payload_floor(1, x, q, s)
    torch.cuda.synchronize()
    assert torch.equal(s, x.float().abs().amax(dim=1))
    diag.usp_diag_payload_floor(2, x, q, s)
    torch.cuda.synchronize()
    q32 = q.view(torch.int32)                      # per unit of 8 bytes: (row, lane)
    assert int(q32[0, 1]) == 0 and int(q32[63, 0]) == 63 and int(q32[63, 3]) == 1 and int(q32[5, 2 * 64 * 5 + 2 * 7 + 1]) == 7


FUSED, WIDE, SPLIT = 16, 4, 8


def _ring(kind, seed=91, shape=(2, 3, 128, 300, (128, 192, 64))):
    import paper_2602_10940_amd as U
    from paper_2602_10940_amd import workloads as W
    from tests.gpu_util import dev_bf16
    B, H, d, Sq, lens = shape
    inp = W.make_attention_inputs(W.Workload("late", seed, B, H, d, Sq, lens, "bf16"))
    r = dict(q=dev_bf16(inp.q), softmax_scale=float(inp.softmax_scale))
    if kind == "fp8":
        kq, ksc, vq, vsc = [], [], [], []
        for k, v in zip(inp.k, inp.v):
            b_, h_, L, dd = k.shape
            a, sa = U.usp_fp8_quant(dev_bf16(k).reshape(b_ * h_ * L, dd))
            b2, sb = U.usp_fp8_quant(dev_bf16(v).reshape(b_ * h_ * L, dd))
            kq.append(a.reshape(b_, h_, L, dd)); ksc.append(sa.reshape(b_, h_, L))
            vq.append(b2.reshape(b_, h_, L, dd)); vsc.append(sb.reshape(b_, h_, L))
        r.update(k_chunks=kq, v_chunks=vq, k_scales=ksc, v_scales=vsc)
    else:
        r.update(k_chunks=[dev_bf16(k) for k in inp.k], v_chunks=[dev_bf16(v) for v in inp.v])
    return r


@pytest.mark.parametrize("kind,flags", [("bf16", FUSED | WIDE), ("bf16", FUSED | SPLIT), ("fp8", WIDE), ("fp8", SPLIT)])
def test_arrival_wait_that_gives_up_returns_nan_rows(kind, flags):
    """Algorithm 2 inside one launch: an attention work-group that stops waiting for a chunk must hand
    back rows nobody can mistake for a result.  O = 0 with lse = -inf is a valid result (every key
    masked), so both come back as NaN, for every row of the work-group, in both work decompositions
    (in the key-split one the wave that gave up may belong to the group that does not store)."""
    import paper_2602_10940_amd as U
    from paper_2602_10940_amd import diag
    r = _ring(kind)
    ref_o, ref_l = U.usp_ring_attn_fwd(flags=flags, **r)
    torch.cuda.synchronize()
    assert torch.isfinite(ref_o.float()).all() and torch.isfinite(ref_l).all()
    desc = U.make_attn_desc(r["q"], r["k_chunks"], torch.empty_like(r["q"]), r["softmax_scale"], flags)
    ws = torch.full((U.usp_ring_attn_workspace_bytes(desc),), 0xFF, dtype=torch.uint8, device=DEV)
    # the knobs at their defaults: the library's own call
    o, l = diag.usp_diag_ring_attn_fwd_wait(arrive_need_extra=0, arrive_polls=0, flags=flags, workspace=ws, **r)
    torch.cuda.synchronize()
    assert torch.equal(o, ref_o) and torch.equal(l, ref_l)
    # one more arrival than there are copy work-groups: never reached; 200 polls, then give up
    o, l = diag.usp_diag_ring_attn_fwd_wait(arrive_need_extra=1, arrive_polls=200, flags=flags, workspace=ws, **r)
    torch.cuda.synchronize()
    assert torch.isnan(o.float()).all(), int(torch.isnan(o.float()).sum())
    assert torch.isnan(l).all(), int(torch.isnan(l).sum())
    # the next ordinary call through the same workspace is unaffected
    o, l = U.usp_ring_attn_fwd(flags=flags, workspace=ws, **r)
    torch.cuda.synchronize()
    assert torch.equal(o, ref_o) and torch.equal(l, ref_l)


def test_arrival_wait_knobs_are_ignored_by_other_forms_and_checked():
    import paper_2602_10940_amd as U
    from paper_2602_10940_amd import diag
    r = _ring("bf16")
    ref = U.usp_ring_attn_fwd(flags=64, **r)                       # one launch per chunk: no arrival counters
    o, l = diag.usp_diag_ring_attn_fwd_wait(arrive_need_extra=1, arrive_polls=10, flags=64, **r)
    torch.cuda.synchronize()
    assert torch.equal(o, ref[0]) and torch.equal(l, ref[1])
    with pytest.raises(U.UspError):
        diag.usp_diag_ring_attn_fwd_wait(arrive_need_extra=-1, arrive_polls=0, **r)
