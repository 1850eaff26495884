"""usp_ring_attn_fwd_noalloc: the entry point for callers that cannot allocate (HIP graph capture,
tight serving loops).  Its workspace is the library's own device array, shared by every call on the
GPU and keeping the previous call's contents, so the test makes two calls in a row, the second with
a smaller input, and checks each against usp_ring_attn_fwd (same kernels in the same order: the
bits must be equal) and against the fp64 oracle at the usual bars.

Named to be collected last: a failure here must not hide the tests before it under `pytest -x`."""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from paper_2602_10940_amd import workloads as W
from tests.gpu_util import DEV, dev_bf16, host_f64
from tests.test_gpu_attention import _assert_parity

pytestmark = pytest.mark.gpu

STEPWISE, FUSED = 64, 16


def _inputs(seed, B, H, Sq, lens, masked=(0, 0)):
    wl = W.Workload("noalloc", seed, B, H, 128, Sq, lens, "bf16", masked_keys=masked)
    inp = W.make_attention_inputs(wl)
    km = None if inp.key_mask is None else [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    return inp, dict(q=dev_bf16(inp.q), k_chunks=[dev_bf16(k) for k in inp.k], v_chunks=[dev_bf16(v) for v in inp.v],
                     key_mask=km, softmax_scale=float(inp.softmax_scale))


def _both(P, r, flags):
    """(existing entry point with a workspace of the caller's, new entry point) on the same inputs."""
    ref_o, ref_l = P.usp_ring_attn_fwd(flags=flags, **r)
    out = torch.full_like(r["q"], float("nan"))
    lse = torch.full(r["q"].shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    P.usp_ring_attn_fwd_noalloc(out=out, lse=lse, flags=flags, **r)
    torch.cuda.synchronize()
    return ref_o, ref_l, out, lse


@pytest.mark.parametrize("flags", [STEPWISE, 0, FUSED])
def test_two_calls_in_a_row_the_second_smaller(flags):
    """STEPWISE: fp32 carried O and per-tile records in the scratch; 0: one launch over the ring
    (records of a masked ring); FUSED: staging buffers and arrival counters in the scratch."""
    import paper_2602_10940_amd as P
    big_inp, big = _inputs(71, 2, 4, 600, (256, 192, 320), masked=(700, 760))
    small_inp, small = _inputs(72, 1, 2, 200, (128, 64), masked=(100, 150))
    for inp, r in ((big_inp, big), (small_inp, small)):
        ref_o, ref_l, out, lse = _both(P, r, flags)
        assert torch.equal(out, ref_o) and torch.equal(lse, ref_l)
        ro, rl = orc.ring_attention(inp.q, inp.k, inp.v, float(inp.softmax_scale), inp.key_mask)
        _assert_parity(host_f64(out), host_f64(lse), ro, rl)
    # and the big one again, after the small one has left its state behind
    ref_o, ref_l, out, lse = _both(P, big, flags)
    assert torch.equal(out, ref_o) and torch.equal(lse, ref_l)


def test_fp8_ring_on_the_scratch():
    import paper_2602_10940_amd as P
    from tests.test_gpu_fp8_ring import _fp8_ring
    for seed, shape in ((73, (1, 3, 300, (128, 256, 64))), (74, (1, 2, 130, (64, 64)))):
        wl = W.Workload("noalloc8", seed, shape[0], shape[1], 128, shape[2], shape[3], "bf16")
        inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
        scale = float(inp.softmax_scale)
        for flags in (0, STEPWISE):
            ref_o, ref_l = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, softmax_scale=scale, flags=flags)
            out = torch.full_like(q, float("nan"))
            lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device=DEV)
            P.usp_ring_attn_fwd_noalloc(q, kq, vq, out, lse, k_scales=ksc, v_scales=vsc, softmax_scale=scale, flags=flags)
            torch.cuda.synchronize()
            assert torch.equal(out, ref_o) and torch.equal(lse, ref_l)
        ro, rl = orc.ring_attention(inp.q, kx, vx, scale)
        _assert_parity(host_f64(out), host_f64(lse), ro, rl)


def test_limits_are_errors_with_nothing_enqueued():
    import paper_2602_10940_amd as P
    inp, r = _inputs(75, 1, 2, 128, (64, 64))
    out = torch.zeros_like(r["q"])
    lse = torch.zeros(r["q"].shape[:3], dtype=torch.float32, device=DEV)
    with pytest.raises(P.UspError) as e:                       # side stream + events: not in this entry point
        P.usp_ring_attn_fwd_noalloc(out=out, lse=lse, flags=1, **r)
    assert e.value.status == -2
    # a shard whose workspace exceeds the scratch: descriptor only, the pointers are never followed
    q = torch.empty((1, 24, 4096, 128), dtype=torch.bfloat16, device=DEV)
    kq = [torch.empty((1, 24, 4096, 128), dtype=torch.uint8, device=DEV) for _ in range(2)]
    sc = [torch.empty((1, 24, 4096), dtype=torch.float32, device=DEV) for _ in range(2)]
    desc = P.make_attn_desc(q, kq, q, 0.0, 0)
    assert P.usp_ring_attn_workspace_bytes(desc) > P.USP_NOALLOC_SCRATCH_BYTES
    with pytest.raises(P.UspError) as e:
        P.usp_ring_attn_fwd_noalloc(q, kq, kq, torch.empty_like(q), torch.empty((1, 24, 4096), dtype=torch.float32, device=DEV),
                                    k_scales=sc, v_scales=sc)
    assert e.value.status == -3 and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert float(out.float().abs().sum()) == 0.0 and float(lse.abs().sum()) == 0.0


@pytest.mark.parametrize("flags", [0, FUSED, STEPWISE])
def test_replays_from_a_hip_graph(flags):
    """The caller this entry point names: the call recorded into a HIP graph (nothing may allocate under
    capture).  Replays, with eager calls of another shape on the same scratch in between, must
    reproduce the eager result bit for bit."""
    import paper_2602_10940_amd as P
    _, r = _inputs(76, 1, 3, 260, (192, 128, 64), masked=(300, 340))
    _, other = _inputs(77, 1, 2, 100, (64, 128))
    out = torch.empty_like(r["q"])
    lse = torch.empty(r["q"].shape[:3], dtype=torch.float32, device=DEV)
    o2 = torch.empty_like(other["q"])
    l2 = torch.empty(other["q"].shape[:3], dtype=torch.float32, device=DEV)
    ref_o, ref_l = P.usp_ring_attn_fwd(flags=flags, **r)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            P.usp_ring_attn_fwd_noalloc(out=out, lse=lse, flags=flags, **r)
    torch.cuda.synchronize()
    for _ in range(3):
        out.zero_(); lse.zero_()
        P.usp_ring_attn_fwd_noalloc(out=o2, lse=l2, flags=flags, **other)   # leaves its state in the scratch
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_o) and torch.equal(lse, ref_l)
