"""FP8 K/V rings through usp_ring_attn_fwd in its one-launch form (Algorithm 2 with the payloads of
Algorithm 1): the chunks travel as E4M3 codes + per-(batch, head, token) scales and are decoded by
work-groups of the attention launch itself.  Parity against the fp64 oracle attending over
decode(code) * scale exactly; agreement with the one-launch-per-chunk form of the same call."""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from paper_2602_10940_amd import workloads as W
from tests.gpu_util import DEV, dev_bf16, host_f64
from tests.test_gpu_attention import _assert_parity

pytestmark = pytest.mark.gpu

STEPWISE, FUSED, WIDE, SPLIT = 64, 16, 4, 8


def _P():
    import paper_2602_10940_amd as P
    return P


def _fp8_ring(wl):
    """Inputs of the workload with K/V quantised by the library; the oracle's exact dequantisation."""
    P = _P()
    inp = W.make_attention_inputs(wl)
    q = dev_bf16(inp.q)
    kq, ksc, vq, vsc, kx, vx = [], [], [], [], [], []
    for k, v in zip(inp.k, inp.v):
        B, H, L, d = k.shape
        a, sa = P.usp_fp8_quant(dev_bf16(k).reshape(B * H * L, d))
        b, sb = P.usp_fp8_quant(dev_bf16(v).reshape(B * H * L, d))
        kq.append(a.reshape(B, H, L, d)); ksc.append(sa.reshape(B, H, L))
        vq.append(b.reshape(B, H, L, d)); vsc.append(sb.reshape(B, H, L))
        kx.append(orc.dequant_exact_f64(a.cpu().numpy().reshape(B, H, L, d), sa.cpu().numpy().reshape(B, H, L)))
        vx.append(orc.dequant_exact_f64(b.cpu().numpy().reshape(B, H, L, d), sb.cpu().numpy().reshape(B, H, L)))
    return inp, q, kq, ksc, vq, vsc, kx, vx


def _call(q, kq, ksc, vq, vsc, scale, flags, **kw):
    P = _P()
    o, l = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, softmax_scale=scale, flags=flags, **kw)
    torch.cuda.synchronize()
    return o, l


@pytest.mark.parametrize("B,H,Sq,lens", [
    (1, 3, 160, (192, 64, 128, 128)),          # four chunks, one work-group round
    (2, 2, 300, (128, 256)),                   # a batch of two, a ragged last query block
    (1, 2, 1100, (64, 0, 448, 64, 0, 256)),    # empty chunks in between; enough queries for 256-query work-groups
    (1, 1, 130, (64,) * 16),                   # the most chunks one launch takes
])
def test_fp8_ring_one_launch_against_oracle(B, H, Sq, lens):
    wl = W.Workload("fp8_one", 61, B, H, 128, Sq, tuple(lens), "bf16", outlier_frac=0.01, outlier_mul=20.0)
    inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
    scale = float(inp.softmax_scale)
    ro, rl = orc.ring_attention(inp.q, kx, vx, scale)
    so, sl = _call(q, kq, ksc, vq, vsc, scale, STEPWISE)            # one launch per chunk
    _assert_parity(host_f64(so), host_f64(sl), ro, rl)
    for flags in (0, FUSED, WIDE, SPLIT, FUSED | SPLIT):
        o, l = _call(q, kq, ksc, vq, vsc, scale, flags)
        _assert_parity(host_f64(o), host_f64(l), ro, rl)
        # the two forms differ only in where the running state is rounded
        assert float((o.float() - so.float()).abs().max()) <= 2.0 ** -6 * max(1.0, float(so.float().abs().max()))
        assert float((l - sl).abs().max()) <= 1e-4


def test_fp8_ring_one_launch_poisoned_workspace_and_alternating_inputs():
    """The decoded chunks, their records and the arrival counters live in the workspace: a call must not
    depend on what the previous call (or nobody) left there."""
    P = _P()
    shape = (1, 6, 128, 700, (512, 256, 320))
    runs = []
    for seed in (71, 72):
        inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(W.Workload("fp8_alt", seed, *shape, "bf16"))
        ref = _call(q, kq, ksc, vq, vsc, float(inp.softmax_scale), 0)
        ro, rl = orc.ring_attention(inp.q, kx, vx, float(inp.softmax_scale))
        _assert_parity(host_f64(ref[0]), host_f64(ref[1]), ro, rl)
        runs.append((inp, q, kq, ksc, vq, vsc, ref))
    assert not torch.equal(runs[0][6][0], runs[1][6][0])
    desc = P.make_attn_desc(runs[0][1], runs[0][2], torch.empty_like(runs[0][1]), float(runs[0][0].softmax_scale), FUSED)
    ws = torch.full((P.usp_ring_attn_workspace_bytes(desc),), 0xFF, dtype=torch.uint8, device=DEV)
    for it in range(6):
        inp, q, kq, ksc, vq, vsc, (ref_o, ref_l) = runs[it & 1]
        o, l = _call(q, kq, ksc, vq, vsc, float(inp.softmax_scale), FUSED, workspace=ws)
        assert torch.equal(o, ref_o) and torch.equal(l, ref_l), it
    outs = []                                                       # back to back, no synchronisation between
    for it in range(6):
        inp, q, kq, ksc, vq, vsc, _ = runs[it & 1]
        outs.append(P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, softmax_scale=float(inp.softmax_scale),
                                        flags=FUSED, workspace=ws))
    torch.cuda.synchronize()
    for it, (o, l) in enumerate(outs):
        assert torch.equal(o, runs[it & 1][6][0]) and torch.equal(l, runs[it & 1][6][1]), it


def test_fp8_ring_one_launch_with_key_masks():
    """Key masks in the one-launch form: the copy work-groups write them into the per-tile records
    (factor 0, bias -inf, a flag per tile).  A tail of masked keys; then a batch of three with a mask
    of its own per entry: nothing masked, a hole in the first chunk with the second chunk dead, and
    only the first tile plus one key of the second chunk alive."""
    P = _P()
    wl = W.Workload("fp8_masked", 73, 1, 2, 128, 150, (128, 192), "bf16", masked_keys=(250, 320))
    inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
    km = [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    ro, rl = orc.ring_attention(inp.q, kx, vx, float(inp.softmax_scale), inp.key_mask)
    for flags in (0, FUSED, STEPWISE, WIDE, SPLIT):
        o, l = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, key_mask=km,
                                   softmax_scale=float(inp.softmax_scale), flags=flags)
        torch.cuda.synchronize()
        _assert_parity(host_f64(o), host_f64(l), ro, rl)

    wl = W.Workload("fp8_masked_b3", 74, 3, 2, 128, 300, (192, 128, 64), "bf16", masked_keys=(100, 384))
    inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
    for m in inp.key_mask:
        m[0, :] = 1
    inp.key_mask[0][1, :] = 1; inp.key_mask[0][1, 3:70] = 0; inp.key_mask[1][1, :] = 0; inp.key_mask[2][1, :] = 1
    inp.key_mask[0][2, :] = 0; inp.key_mask[0][2, :64] = 1; inp.key_mask[1][2, :] = 0; inp.key_mask[1][2, 5] = 1
    inp.key_mask[2][2, :] = 0
    km = [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    ro, rl = orc.ring_attention(inp.q, kx, vx, float(inp.softmax_scale), inp.key_mask)
    for flags in (0, STEPWISE, WIDE, SPLIT):
        o, l = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, key_mask=km,
                                   softmax_scale=float(inp.softmax_scale), flags=flags)
        torch.cuda.synchronize()
        _assert_parity(host_f64(o), host_f64(l), ro, rl)
    # a mask for some chunks only
    km2 = [km[0], None, km[2]]
    masks2 = [inp.key_mask[0], np.ones_like(inp.key_mask[1]), inp.key_mask[2]]
    ro2, rl2 = orc.ring_attention(inp.q, kx, vx, float(inp.softmax_scale), masks2)
    o, l = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, key_mask=km2, softmax_scale=float(inp.softmax_scale))
    torch.cuda.synchronize()
    _assert_parity(host_f64(o), host_f64(l), ro2, rl2)


def test_fp8_ring_flux1024_r4_full_size_every_row():
    """The configuration bench.py times for the FP8 ring (flags 0 and FUSED_PREFETCH give the same
    launch): every query row of every head against the oracle, for it and for the per-chunk form."""
    wl = W.WORKLOADS["flux1024_r4"]
    inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
    scale = float(inp.softmax_scale)
    o, l = _call(q, kq, ksc, vq, vsc, scale, FUSED)
    o0, l0 = _call(q, kq, ksc, vq, vsc, scale, 0)
    assert torch.equal(o, o0) and torch.equal(l, l0)
    so, sl = _call(q, kq, ksc, vq, vsc, scale, STEPWISE)
    assert float((o.float() - so.float()).abs().max()) <= 2.0 ** -6
    assert float((l - sl).abs().max()) <= 1e-4
    ro, rl = orc.ring_attention(inp.q, kx, vx, scale)
    for oo, ll in ((o, l), (so, sl)):
        ho, hl = host_f64(oo), host_f64(ll)
        assert ho.shape == ro.shape == (1, 24, 1152, 128)
        _assert_parity(ho, hl, ro, rl)
        for h in range(wl.H):
            _assert_parity(ho[:, h:h + 1], hl[:, h:h + 1], ro[:, h:h + 1], rl[:, h:h + 1])


@pytest.mark.parametrize("flags", [0, STEPWISE])
def test_fp8_ring_call_replays_from_a_hip_graph(flags):
    """The FP8 ring call (one launch, and one launch per chunk) captured into a HIP graph: every replay,
    with the workspace scrubbed and eager calls of the program in between, reproduces the eager result."""
    P = _P()
    wl = W.Workload("fp8_graph", 81, 1, 3, 128, 200, (192, 64, 128, 128), "bf16")
    inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
    scale = float(inp.softmax_scale)
    out = torch.empty_like(q)
    lse = torch.empty((1, 3, 200), dtype=torch.float32, device=DEV)
    desc = P.make_attn_desc(q, kq, out, scale, flags)
    ws = torch.empty((P.usp_ring_attn_workspace_bytes(desc),), dtype=torch.uint8, device=DEV)
    call = lambda: P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, softmax_scale=scale, flags=flags,
                                       out=out, lse=lse, workspace=ws)
    call()
    torch.cuda.synchronize()
    ref_o, ref_l = out.clone(), lse.clone()
    ro, rl = orc.ring_attention(inp.q, kx, vx, scale)
    _assert_parity(host_f64(ref_o), host_f64(ref_l), ro, rl)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            call()
    torch.cuda.synchronize()
    for _ in range(3):
        out.zero_(); lse.zero_(); ws.fill_(0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_o) and torch.equal(lse, ref_l)
        call()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_o) and torch.equal(lse, ref_l)


@pytest.mark.parametrize("fp8", [False, True])
def test_later_chunks_in_pinned_host_memory(fp8):
    """With the double-buffered modes the chunks after the first are only read by the transfers: they may
    sit in pinned host memory (a slow link).  Same result as with every chunk in device memory."""
    P = _P()
    wl = W.Workload("far_chunks", 95, 1, 3, 128, 200, (192, 64, 128, 128), "bf16")
    inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
    scale = float(inp.softmax_scale)
    host = lambda t: torch.empty(t.shape, dtype=t.dtype, pin_memory=True).copy_(t)
    far = lambda ts: [ts[0]] + [host(t) for t in ts[1:]]
    if fp8:
        near = dict(k_chunks=kq, v_chunks=vq, k_scales=ksc, v_scales=vsc)
        away = dict(k_chunks=far(kq), v_chunks=far(vq), k_scales=far(ksc), v_scales=far(vsc))
    else:
        ks = [dev_bf16(k) for k in inp.k]; vs = [dev_bf16(v) for v in inp.v]
        near = dict(k_chunks=ks, v_chunks=vs)
        away = dict(k_chunks=far(ks), v_chunks=far(vs))
    torch.cuda.synchronize()
    for flags, side in ((1, torch.cuda.Stream()), (FUSED, None), (FUSED | STEPWISE, None)):
        ro, rl = P.usp_ring_attn_fwd(q, softmax_scale=scale, flags=flags, copy_stream=side, **near)
        o, l = P.usp_ring_attn_fwd(q, softmax_scale=scale, flags=flags, copy_stream=side, **away)
        torch.cuda.synchronize()
        assert torch.equal(o, ro) and torch.equal(l, rl), flags


def test_two_rings_on_two_streams_at_once():
    """An FP8 ring and a bf16 ring, each as one launch with its transfers inside, issued on two streams
    without synchronising: every launch has its own counters and buffers in its own workspace, and its
    copy work-groups are dispatched ahead of its own attention work-groups whatever else is running."""
    P = _P()
    wl = W.Workload("two_streams", 97, 1, 6, 128, 700, (512, 256, 320), "bf16")
    inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
    ks = [dev_bf16(k) for k in inp.k]; vs = [dev_bf16(v) for v in inp.v]
    scale = float(inp.softmax_scale)
    ref8 = _call(q, kq, ksc, vq, vsc, scale, FUSED)
    refb = P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=scale, flags=FUSED)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for it in range(6):
        with torch.cuda.stream(s1):
            a = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, softmax_scale=scale, flags=FUSED, compute_stream=s1)
        with torch.cuda.stream(s2):
            b = P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=scale, flags=FUSED, compute_stream=s2)
        outs.append((a, b))
    torch.cuda.synchronize()
    for it, (a, b) in enumerate(outs):
        assert torch.equal(a[0], ref8[0]) and torch.equal(a[1], ref8[1]), it
        assert torch.equal(b[0], refb[0]) and torch.equal(b[1], refb[1]), it


def test_fp8_ring_with_scales_and_masks_that_are_not_16_byte_aligned():
    """The one-launch form reads scales 16 bytes and mask bytes 4 at a time; tensors that start at an odd
    offset send the call to the per-chunk form, with the same result."""
    P = _P()
    wl = W.Workload("fp8_unaligned", 98, 2, 2, 128, 150, (128, 192), "bf16", masked_keys=(250, 320))
    inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
    km = [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    scale = float(inp.softmax_scale)
    ref = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, key_mask=km, softmax_scale=scale, flags=STEPWISE)
    def shifted(t, n):                     # the same values, n elements into a larger allocation
        flat = torch.empty((t.numel() + n,), dtype=t.dtype, device=DEV)
        flat[n:].copy_(t.reshape(-1))
        return flat[n:].reshape(t.shape)
    ksc1 = [shifted(t, 1) for t in ksc]
    km1 = [shifted(t, 1) for t in km]
    torch.cuda.synchronize()
    assert ksc1[0].data_ptr() % 16 != 0 and km1[0].data_ptr() % 4 != 0
    for kw in (dict(k_scales=ksc1, key_mask=km), dict(k_scales=ksc, key_mask=km1), dict(k_scales=ksc1, key_mask=km1)):
        o, l = P.usp_ring_attn_fwd(q, kq, vq, v_scales=vsc, softmax_scale=scale, **kw)
        torch.cuda.synchronize()
        assert torch.equal(o, ref[0]) and torch.equal(l, ref[1])


def test_two_host_threads_call_at_once():
    """Two host threads issue rings on streams of their own at the same time (ctypes drops the GIL
    around a call): the library's per-call state (error text, event pool, the d = 64 marker) is
    per thread, and a refused call in one thread leaves the other's results and error text alone."""
    import threading
    P = _P()
    wl = W.Workload("two_threads", 99, 1, 4, 128, 520, (256, 192, 128), "bf16")
    inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
    wl64 = W.Workload("two_threads_d64", 100, 1, 4, 64, 300, (128, 200), "bf16")
    inp64 = W.make_attention_inputs(wl64)
    q64 = dev_bf16(inp64.q); k64 = [dev_bf16(k) for k in inp64.k]; v64 = [dev_bf16(v) for v in inp64.v]
    scale, scale64 = float(inp.softmax_scale), float(inp64.softmax_scale)
    ref8 = _call(q, kq, ksc, vq, vsc, scale, 0)
    ref64 = P.usp_ring_attn_fwd(q64, k64, v64, softmax_scale=scale64)
    torch.cuda.synchronize()
    results, errors = {}, []

    def fp8_rings():
        try:
            st = torch.cuda.Stream()
            outs = []
            with torch.cuda.stream(st):
                for it in range(20):
                    outs.append(P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, softmax_scale=scale,
                                                    flags=(0, STEPWISE, 1)[it % 3], compute_stream=st,
                                                    copy_stream=torch.cuda.Stream() if it % 3 == 2 else None))
            st.synchronize()
            results["fp8"] = outs
        except Exception as e:   # noqa: BLE001 (reported by the main thread)
            errors.append(e)

    def d64_rings_and_refusals():
        try:
            st = torch.cuda.Stream()
            outs = []
            with torch.cuda.stream(st):
                for it in range(20):
                    outs.append(P.usp_ring_attn_fwd(q64, k64, v64, softmax_scale=scale64, compute_stream=st))
                    with pytest.raises(P.UspError, match="exclude"):
                        P.usp_ring_attn_fwd(q64, k64, v64, softmax_scale=scale64, flags=WIDE | SPLIT, compute_stream=st)
            st.synchronize()
            results["d64"] = outs
        except Exception as e:   # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=fp8_rings), threading.Thread(target=d64_rings_and_refusals)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not errors, errors
    assert all(not t.is_alive() for t in threads)
    torch.cuda.synchronize()
    ref_step = _call(q, kq, ksc, vq, vsc, scale, STEPWISE)
    for it, (o, l) in enumerate(results["fp8"]):
        want = ref8 if it % 3 == 0 else ref_step        # (the side-stream form shares the per-chunk kernels)
        assert torch.equal(o, want[0]) and torch.equal(l, want[1]), it
    for it, (o, l) in enumerate(results["d64"]):
        assert torch.equal(o, ref64[0]) and torch.equal(l, ref64[1]), it


def test_masked_fp8_ring_many_calls_through_one_workspace():
    """Three rings of one shape (short chunks, three batch entries, key masks) take turns through one
    workspace, 3000 calls back to back: every result must equal its ring's own reference bit for bit.
    (The copy work-groups' 16-byte device-scope stores are inline asm; without wait states behind them
    the instruction that computed the next store's data could change the one in flight, which showed
    as wrong per-key factors in one call out of a few hundred.)"""
    P = _P()
    rings = []
    for seed in (200, 201, 202):
        wl = W.Workload("fp8_many", seed, 3, 2, 128, 130, (128, 256, 128, 128), "bf16", masked_keys=(441, 583))
        inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
        km = [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
        rings.append(dict(q=q, k_chunks=kq, v_chunks=vq, k_scales=ksc, v_scales=vsc, key_mask=km,
                          softmax_scale=float(inp.softmax_scale)))
    refs = []
    for r in rings:
        a = P.usp_ring_attn_fwd(**r)
        b = P.usp_ring_attn_fwd(flags=STEPWISE, **r)
        torch.cuda.synchronize()
        assert (a[0].float() - b[0].float()).abs().max().item() <= 2.0 ** -5 and (a[1] - b[1]).abs().max().item() <= 1e-4
        refs.append(a)
    desc = P.make_attn_desc(rings[0]["q"], rings[0]["k_chunks"], torch.empty_like(rings[0]["q"]), rings[0]["softmax_scale"], 0)
    ws = torch.full((P.usp_ring_attn_workspace_bytes(desc),), 0xFF, dtype=torch.uint8, device=DEV)
    rng = np.random.Generator(np.random.PCG64(9))
    bad = 0
    for batch in range(60):
        outs = []
        for _ in range(50):
            i = int(rng.integers(0, 3))
            outs.append((i, P.usp_ring_attn_fwd(workspace=ws, **rings[i])))
        torch.cuda.synchronize()
        bad += sum(1 for i, (o, l) in outs if not (torch.equal(o, refs[i][0]) and torch.equal(l, refs[i][1])))
    assert bad == 0, bad


def test_fp8_step_preparation_one_launch_and_three_agree():
    """A chunk of whole tiles with 16-byte aligned scales is prepared by one launch (K widened, V
    dequantised, records, live-tile counts); scales that are only 4-byte aligned, like a ragged chunk,
    take the three launches of the general case.  Same arithmetic: the results must be equal bit for bit,
    with and without a key mask."""
    wl = W.Workload("fp8_step_prep", 91, 2, 3, 128, 200, (128, 192, 64), "bf16", masked_keys=(250, 330))
    inp, q, kq, ksc, vq, vsc, kx, vx = _fp8_ring(wl)
    scale = float(inp.softmax_scale)
    km = [torch.from_numpy(m).to(DEV) for m in inp.key_mask]

    def shifted(t):   # the same values at an address that is 4 bytes past a 16-byte boundary
        buf = torch.empty((t.numel() + 4,), dtype=t.dtype, device=DEV)
        assert buf.data_ptr() % 16 == 0
        v = buf[1:1 + t.numel()].view(t.shape)
        v.copy_(t)
        return v

    for mask in (None, km):
        ref_o, ref_l = _call(q, kq, ksc, vq, vsc, scale, 64, key_mask=mask)                       # one launch per chunk
        o, l = _call(q, kq, [shifted(s) for s in ksc], vq, [shifted(s) for s in vsc], scale, 64, key_mask=mask)
        assert torch.equal(o, ref_o) and torch.equal(l, ref_l)
    ro, rl = orc.ring_attention(inp.q, kx, vx, scale, inp.key_mask)
    _assert_parity(host_f64(o), host_f64(l), ro, rl)
