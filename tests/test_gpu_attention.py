"""usp_ring_attn_fwd parity against the fp64 oracle, through the C ABI.

Bars (bf16 inputs): attention max-abs 2e-2 and relative L2 5e-3, lse 1e-3.
"""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from paper_2602_10940_amd import workloads as W
from tests.gpu_util import (ATTN_MAX_ABS, ATTN_REL_L2, DEV, LSE_ABS, attn_errors, dev_bf16, dev_f32,
                            host_f64)

pytestmark = pytest.mark.gpu


def _P():
    import paper_2602_10940_amd as P
    return P


def _run(inp, flags=0, dtype=None, copy_stream=None, **kw):
    P = _P()
    dtype = dtype or inp.wl.dtype
    up = dev_bf16 if dtype == "bf16" else dev_f32
    q = up(inp.q)
    ks = [up(k) for k in inp.k]
    vs = [up(v) for v in inp.v]
    km = None if inp.key_mask is None else [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    out, lse = P.usp_ring_attn_fwd(q, ks, vs, key_mask=km, softmax_scale=float(inp.softmax_scale),
                                   flags=flags, copy_stream=copy_stream, **kw)
    torch.cuda.synchronize()
    return host_f64(out), host_f64(lse)


def _oracle(inp, rows=None):
    q = inp.q if rows is None else inp.q[:, :, rows, :]
    return orc.ring_attention(q, inp.k, inp.v, float(inp.softmax_scale), inp.key_mask)


def _assert_parity(got_o, got_l, ref_o, ref_l, fp32=False):
    mx, rl = attn_errors(got_o, ref_o)
    fin = np.isfinite(ref_l)
    le = float(np.max(np.abs(got_l[fin] - ref_l[fin]))) if fin.any() else 0.0
    assert np.array_equal(np.isneginf(got_l), np.isneginf(ref_l))
    bar_abs, bar_l2, bar_lse = (2e-5, 5e-6, 2e-5) if fp32 else (ATTN_MAX_ABS, ATTN_REL_L2, LSE_ABS)
    # the absolute bar is stated for N(0,1) values (|O| < 1); with x20 outliers |O| reaches tens and
    # the bf16 output rounding alone is 2^-9 |O|, so the bar scales with the largest output
    bar_abs *= max(1.0, float(np.max(np.abs(ref_o))))
    assert mx <= bar_abs and rl <= bar_l2 and le <= bar_lse, (mx, rl, le)
    return mx, rl, le


# ---------------------------------------------------------------------------------------
def test_tiny_fp32_ring2():
    """Config 1: B=1 H=2 d=64, Q shard 128, two KV chunks of 128, fp32 (fp32 arithmetic path)."""
    inp = W.make_attention_inputs(W.WORKLOADS["tiny"])
    o, l = _run(inp)
    ro, rl = _oracle(inp)
    _assert_parity(o, l, ro, rl, fp32=True)
    o2, l2 = _run(inp, flags=2)          # merge as a separate kernel
    _assert_parity(o2, l2, ro, rl, fp32=True)
    o3, l3 = _run(inp, flags=16)         # chunk 1 staged by work-groups of step 0's launch
    np.testing.assert_array_equal(o3, o)
    np.testing.assert_array_equal(l3, l)


_KERNEL_FLAG = {"auto": 0, "wide": 4, "split": 8, "mixed": 32}   # USP_ATTN_KERNEL_*


def _small_wl(name, H, Sq, lens, **kw):
    base = W.WORKLOADS[name]
    return W.Workload(base.name + "_small", base.seed, 1, H, 128, Sq, tuple(lens), "bf16",
                      k_mul=base.k_mul, head_scale=base.head_scale, outlier_frac=base.outlier_frac,
                      outlier_mul=base.outlier_mul, **kw)


@pytest.mark.parametrize("Sq,lens", [
    (256, (64,)), (256, (128,)), (300, (200,)),          # ragged query and key tails
    (33, (1,)), (1, (70,)), (513, (129, 64, 7)),         # degenerate sizes, several chunks
    (128, (0, 96)), (64, (64, 0, 64)),                   # empty chunks
])
@pytest.mark.parametrize("kernel", ["auto", "wide", "split", "mixed"])
def test_mfma_small_shapes(Sq, lens, kernel):
    inp = W.make_attention_inputs(_small_wl("flux1024_u", 2, Sq, lens))
    o, l = _run(inp, flags=_KERNEL_FLAG[kernel])
    ro, rl = _oracle(inp)
    _assert_parity(o, l, ro, rl)


@pytest.mark.parametrize("variant", ["wide", "split", "mixed"])
@pytest.mark.parametrize("Sq,lens", [
    (128, (64,)), (130, (128,)), (257, (192,)),          # 1, 2, 3 key tiles; ragged query tails
    (384, (448, 64, 512)), (96, (1152,)),                # odd / even tile counts, several chunks
])
def test_mfma_both_work_decompositions(Sq, lens, variant):
    """Unmasked chunks of whole 64-key tiles run on the ping-pong kernels; force each variant."""
    P = _P()
    inp = W.make_attention_inputs(_small_wl("flux1024_u", 3, Sq, lens))
    flag = _KERNEL_FLAG[variant]
    o, l = _run(inp, flags=flag)
    ro, rl = _oracle(inp)
    _assert_parity(o, l, ro, rl)


def test_kernel_variant_flags_exclude_each_other():
    P = _P()
    inp = W.make_attention_inputs(_small_wl("flux1024_u", 1, 64, (64,)))
    with pytest.raises(P.UspError):
        _run(inp, flags=P.USP_ATTN_KERNEL_WIDE | P.USP_ATTN_KERNEL_SPLIT)


def test_mfma_matches_generic_kernel_on_fp32_copy():
    """Same bf16-exact values through the fp32 generic kernel: both must sit on the oracle."""
    inp = W.make_attention_inputs(_small_wl("flux1024_u", 2, 200, (150, 90)))
    ro, rl = _oracle(inp)
    o16, l16 = _run(inp)
    o32, l32 = _run(inp, dtype="f32")
    _assert_parity(o16, l16, ro, rl)
    _assert_parity(o32, l32, ro, rl, fp32=True)


@pytest.mark.parametrize("kernel", ["wide", "split", "mixed"])
def test_key_mask_and_fully_masked_rows(kernel):
    fl = _KERNEL_FLAG[kernel]
    wl = _small_wl("qwen_r2", 2, 192, (128, 128), masked_keys=(90, 256))   # chunk 1 fully masked
    inp = W.make_attention_inputs(wl)
    o, l = _run(inp, flags=fl)
    ro, rl = _oracle(inp)
    _assert_parity(o, l, ro, rl)
    wl2 = _small_wl("qwen_r2", 1, 64, (64, 64), masked_keys=(0, 128))      # nothing left
    inp2 = W.make_attention_inputs(wl2)
    o2, l2 = _run(inp2, flags=fl)
    assert np.all(o2 == 0) and np.all(np.isneginf(l2))
    # dead keys at the front, in the middle of a tile, and whole dead tiles between live ones
    wl3 = _small_wl("qwen_r2", 2, 100, (300, 200), masked_keys=(0, 70))
    inp3 = W.make_attention_inputs(wl3)
    inp3.key_mask[0][:, 130:260] = 0
    inp3.key_mask[1][:, 5:9] = 0
    o3, l3 = _run(inp3, flags=fl)
    ro3, rl3 = _oracle(inp3)
    _assert_parity(o3, l3, ro3, rl3)


@pytest.mark.parametrize("kernel", ["wide", "split", "mixed"])
def test_batch_of_three_with_a_different_mask_per_entry(kernel):
    """B = 3: every batch entry has its own key mask (different live tile counts, one entry with
    trailing dead tiles only, one fully dead second chunk), FP8 K/V with per-(b,h,token) scales on
    one pass and plain bf16 on the other; also a ring of plain chunks in every transfer mode."""
    P = _P()
    wl = W.Workload("b3", 11, 3, 2, 128, 150, (200, 136), "bf16", masked_keys=(100, 336))
    inp = W.make_attention_inputs(wl)
    inp.key_mask[0][0, :] = 1; inp.key_mask[1][0, :] = 1          # entry 0: nothing masked
    inp.key_mask[0][1, :] = 1; inp.key_mask[0][1, 3:70] = 0      # entry 1: a hole in chunk 0, chunk 1 dead
    inp.key_mask[0][2, 64:] = 0; inp.key_mask[1][2, :] = 0        # entry 2: only the first tile lives
    inp.key_mask[1][2, 5] = 1                                     # ... and one key of chunk 1
    fl = _KERNEL_FLAG[kernel]
    o, l = _run(inp, flags=fl)
    ro, rl = _oracle(inp)
    _assert_parity(o, l, ro, rl)
    for extra in (16, 2):                                         # fused prefetch, unfused merge
        o2, l2 = _run(inp, flags=fl | extra)
        _assert_parity(o2, l2, ro, rl)
    # FP8 K/V of the same values
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
    km = [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    fo, fl_ = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, key_mask=km,
                                  softmax_scale=float(inp.softmax_scale), flags=fl | 16)
    torch.cuda.synchronize()
    ro8, rl8 = orc.ring_attention(inp.q, kx, vx, float(inp.softmax_scale), inp.key_mask)
    _assert_parity(host_f64(fo), host_f64(fl_), ro8, rl8)


@pytest.mark.parametrize("kernel,Sc", [("auto", 96), ("wide", 128), ("split", 192), ("mixed", 320)])
def test_strided_layouts(kernel, Sc):
    """[B,S,H,d] storage viewed as [B,H,S,d]: token stride H*d, head stride d; chunk lengths with and
    without a ragged last tile (the kernels with and without per-tile key records)."""
    P = _P()
    inp = W.make_attention_inputs(_small_wl("flux1024_u", 3, 130, (Sc,)))
    def bshd(x):
        t = dev_bf16(np.ascontiguousarray(x.transpose(0, 2, 1, 3)))
        return t.permute(0, 2, 1, 3)
    q, k, v = bshd(inp.q), bshd(inp.k[0]), bshd(inp.v[0])
    out = torch.empty((1, 130, 3, 128), dtype=torch.bfloat16, device=DEV).permute(0, 2, 1, 3)
    o, l = P.usp_ring_attn_fwd(q, [k], [v], softmax_scale=float(inp.softmax_scale), out=out,
                               flags=_KERNEL_FLAG[kernel])
    torch.cuda.synchronize()
    ro, rl = _oracle(inp)
    _assert_parity(host_f64(o), host_f64(l), ro, rl)


def test_ring4_fused_unfused_and_double_buffered_agree():
    wl = W.Workload("r4_small", 2, 1, 4, 128, 288, (288,) * 4, "bf16")
    inp = W.make_attention_inputs(wl)
    ro, rl = _oracle(inp)
    o, l = _run(inp)
    _assert_parity(o, l, ro, rl)
    ou, lu = _run(inp, flags=2)
    _assert_parity(ou, lu, ro, rl)
    side = torch.cuda.Stream()
    od, ld = _run(inp, flags=1, copy_stream=side)
    np.testing.assert_array_equal(od, o)        # same kernels, same order: bit-identical
    np.testing.assert_array_equal(ld, l)
    of, lf = _run(inp, flags=16)                # transfers inside the attention launches
    np.testing.assert_array_equal(of, o)
    np.testing.assert_array_equal(lf, l)
    of2, lf2 = _run(inp, flags=16 | 2)          # ... with the merge as a separate kernel
    np.testing.assert_array_equal(of2, ou)
    np.testing.assert_array_equal(lf2, lu)


@pytest.mark.parametrize("flags,lens,masked", [(0, (192, 64, 100, 128), None), (16, (192, 64, 100, 128), None),
                                               (2, (192, 64, 100, 128), None), (0, (192, 64, 128, 128), None),
                                               (16, (192, 64, 128, 128), None),
                                               (0, (192, 64, 128, 128), (200, 300)), (16, (192, 64, 128, 128), (200, 300))])
def test_ring_call_replays_from_a_hip_graph(flags, lens, masked):
    """The library allocates nothing and clears nothing with memset nodes, so a ring call can be
    captured into a HIP graph.  Every replay (with eager calls and synchronisations of the program
    in between, outputs scrubbed first) must reproduce the eager result bit for bit."""
    P = _P()
    wl = W.Workload("r4_graph", 12, 1, 3, 128, 200, tuple(lens), "bf16", masked_keys=masked or (0, 0))
    inp = W.make_attention_inputs(wl)
    q = dev_bf16(inp.q); ks = [dev_bf16(k) for k in inp.k]; vs = [dev_bf16(v) for v in inp.v]
    km = None if inp.key_mask is None else [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    out = torch.empty_like(q)
    lse = torch.empty((1, 3, 200), dtype=torch.float32, device=DEV)
    desc = P.make_attn_desc(q, ks, out, float(inp.softmax_scale), flags)
    ws = torch.empty((P.usp_ring_attn_workspace_bytes(desc),), dtype=torch.uint8, device=DEV)
    call = lambda: P.usp_ring_attn_fwd(q, ks, vs, key_mask=km, softmax_scale=float(inp.softmax_scale), flags=flags,
                                       out=out, lse=lse, workspace=ws)
    call()
    torch.cuda.synchronize()
    ref_o, ref_l = out.clone(), lse.clone()
    ro, rl = _oracle(inp)
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
        call()                                   # eager work of the program between replays
        torch.cuda.synchronize()
        assert torch.equal(out, ref_o) and torch.equal(lse, ref_l)


@pytest.mark.parametrize("flags", [1, 16])
@pytest.mark.parametrize("lens", [(136,) * 8, (128, 0, 192, 64, 0, 7, 256, 64), (128, 0, 192, 64, 0, 64, 256, 64),
                                  (0, 64, 1152, 64), (64,) * 16])
def test_double_buffer_poisoned_staging(flags, lens):
    """Fill the workspace with NaN bit patterns first: a chunk consumed before its copy landed
    (a missing event, a transfer into the wrong buffer) would put NaN into O.  Both transfer
    modes; equal chunks, and unequal ones with empty chunks, a ragged tail and whole-tile chunks
    (every attention kernel variant carries a transfer at some step).  With lengths that are all
    multiples of 64, flags 16 runs the whole ring as one launch whose first work-groups copy the
    chunks and publish arrival counters; a tile loaded before its chunk's count was reached would
    be the NaN of the poisoned buffer."""
    P = _P()
    wl = W.Workload("r8_small", 5, 1, 2, 128, 200, tuple(lens), "bf16")
    inp = W.make_attention_inputs(wl)
    q = dev_bf16(inp.q); ks = [dev_bf16(k) for k in inp.k]; vs = [dev_bf16(v) for v in inp.v]
    out = torch.empty_like(q)
    desc = P.make_attn_desc(q, ks, out, float(inp.softmax_scale), flags)
    ws = torch.full((P.usp_ring_attn_workspace_bytes(desc),), 0xFF, dtype=torch.uint8, device=DEV)
    side = torch.cuda.Stream() if flags == 1 else None
    for _ in range(3):
        o, l = P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=float(inp.softmax_scale), flags=flags,
                                   out=out, workspace=ws, copy_stream=side)
    torch.cuda.synchronize()
    ro, rl = _oracle(inp)
    _assert_parity(host_f64(o), host_f64(l), ro, rl)


def test_fp8_kv_ring_against_oracle_on_dequantised_values():
    """K/V chunks travel as E4M3 bytes + per-(b,h,token) scales (quantised by the library);
    the oracle attends over decode(code)*scale exactly."""
    P = _P()
    wl = W.Workload("r2_fp8_small", 6, 1, 3, 128, 160, (192, 100), "bf16", outlier_frac=0.01, outlier_mul=20.0)
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
    ro, rl = orc.ring_attention(inp.q, kx, vx, float(inp.softmax_scale))
    for flags, side in ((0, None), (1, torch.cuda.Stream()), (16, None), (4, None), (8, None)):
        o, l = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc,
                                   softmax_scale=float(inp.softmax_scale), flags=flags, copy_stream=side)
        torch.cuda.synchronize()
        _assert_parity(host_f64(o), host_f64(l), ro, rl)


def test_fp8_kv_d64():
    """FP8 K/V with head dimension 64 and bf16 Q: codes widened to bf16 rows of 64, then the matrix-core
    kernels in their head-dimension-64 form."""
    P = _P()
    rng = np.random.Generator(np.random.PCG64(9))
    B, H, Sq, L, d = 1, 2, 50, 70, 64
    bf = lambda x: W.bf16_bits_to_f32(W.f32_to_bf16_bits(x))
    qh = bf(rng.standard_normal((B, H, Sq, d), dtype=np.float32))
    kh = bf(rng.standard_normal((B, H, L, d), dtype=np.float32))
    vh = bf(rng.standard_normal((B, H, L, d), dtype=np.float32))
    a, sa = P.usp_fp8_quant(dev_bf16(kh).reshape(-1, d))
    b, sb = P.usp_fp8_quant(dev_bf16(vh).reshape(-1, d))
    o, l = P.usp_ring_attn_fwd(dev_bf16(qh), [a.reshape(B, H, L, d)], [b.reshape(B, H, L, d)],
                               k_scales=[sa.reshape(B, H, L)], v_scales=[sb.reshape(B, H, L)])
    torch.cuda.synchronize()
    kx = orc.dequant_exact_f64(a.cpu().numpy().reshape(B, H, L, d), sa.cpu().numpy().reshape(B, H, L))
    vx = orc.dequant_exact_f64(b.cpu().numpy().reshape(B, H, L, d), sb.cpu().numpy().reshape(B, H, L))
    ro, rl = orc.attention(qh, kx, vx, 1.0 / np.sqrt(np.float32(d)))
    _assert_parity(host_f64(o), host_f64(l), ro, rl)


def test_flux1024_full_size_every_row():
    """Config 2 at full size (B=1 H=24 d=128 S=4608, one chunk), the plain call bench.py times:
    every query row of every head against the oracle (whole tensors, not a sample)."""
    wl = W.WORKLOADS["flux1024_u"]
    inp = W.make_attention_inputs(wl)
    o, l = _run(inp)
    ro, rl = _oracle(inp)
    assert o.shape == ro.shape == (1, 24, 4608, 128) and l.shape == rl.shape
    _assert_parity(o, l, ro, rl)
    # per head as well: one bad work-group must not hide in the norm of the whole tensor
    for h in range(wl.H):
        _assert_parity(o[:, h:h + 1], l[:, h:h + 1], ro[:, h:h + 1], rl[:, h:h + 1])


def test_flux1024_ring4_full_size_every_row():
    """Config 3 shapes (Q shard 1152, four chunks of 1152), every row of every head against the
    oracle: the plain call (one launch over the ring, what bench.py times as the resident ring),
    the side-stream double buffering of Algorithm 2, and one launch per chunk."""
    wl = W.WORKLOADS["flux1024_r4"]
    inp = W.make_attention_inputs(wl)
    ro, rl = _oracle(inp)
    for flags, side in ((0, None), (1, torch.cuda.Stream()), (64, None), (16, None)):
        o, l = _run(inp, flags=flags, copy_stream=side)
        assert o.shape == ro.shape
        _assert_parity(o, l, ro, rl)
        for h in range(wl.H):
            _assert_parity(o[:, h:h + 1], l[:, h:h + 1], ro[:, h:h + 1], rl[:, h:h + 1])


def test_flux1024_ring4_full_size_every_transfer_mode_bit_identical():
    """Config 3 at full size: the plain call, the side-stream schedule, the transfers inside the
    attention launches and the separate-merge variant of the latter all run the same kernels on the
    same values in the same order."""
    wl = W.WORKLOADS["flux1024_r4"]
    inp = W.make_attention_inputs(wl)
    o0, l0 = _run(inp, flags=64)                 # one launch per chunk, all chunks resident
    o1, l1 = _run(inp, flags=1, copy_stream=torch.cuda.Stream())
    o16, l16 = _run(inp, flags=16)
    np.testing.assert_array_equal(o1, o0); np.testing.assert_array_equal(l1, l0)
    o80, l80 = _run(inp, flags=16 | 64)
    np.testing.assert_array_equal(o80, o0); np.testing.assert_array_equal(l80, l0)
    # the plain call covers the four resident chunks with one launch: same result up to rounding order
    om, lm = _run(inp)
    # ... and so does the fused-prefetch call, whose first work-groups play the ring's transfers
    np.testing.assert_array_equal(o16, om); np.testing.assert_array_equal(l16, lm)
    assert not np.array_equal(om, o0)            # (a different order of operations did run)
    assert np.abs(om - o0).max() <= 2.0 ** -7 and np.abs(lm - l0).max() <= 1e-5
    ro, rl = _oracle(inp)
    _assert_parity(om, lm, ro, rl)


@pytest.mark.parametrize("kernel", ["auto", "wide", "split"])
@pytest.mark.parametrize("Sq,lens", [
    (200, (64, 64)),
    (300, (128, 0, 192, 64, 0, 256)),
    (130, (64,) * 16),
    (257, (640, 64, 1152)),
])
def test_one_launch_over_resident_chunks(Sq, lens, kernel):
    """Chunks that are all resident, unmasked and multiples of 64 keys long are covered by one launch
    (their tiles as one stream); the result must meet the same bars as the launch-per-chunk path."""
    wl = W.Workload("multi_small", 41, 1, 3, 128, Sq, tuple(lens), "bf16")
    inp = W.make_attention_inputs(wl)
    ro, rl = _oracle(inp)
    o, l = _run(inp, flags=_KERNEL_FLAG[kernel])
    _assert_parity(o, l, ro, rl)
    os_, ls_ = _run(inp, flags=_KERNEL_FLAG[kernel] | 64)
    _assert_parity(os_, ls_, ro, rl)
    assert np.abs(o - os_).max() <= 2.0 ** -6 and np.abs(l - ls_).max() <= 1e-5


@pytest.mark.parametrize("kernel", ["wide", "split"])
def test_one_launch_with_transfers_inside_batch_of_two(kernel):
    """The ring as one launch whose first work-groups play the transfers, both work decompositions,
    two batch entries, poisoned workspace: parity, and the same bits as the call on resident chunks."""
    P = _P()
    wl = W.Workload("pipe1_b2", 44, 2, 3, 128, 260, (128, 64, 192), "bf16")
    inp = W.make_attention_inputs(wl)
    q = dev_bf16(inp.q); ks = [dev_bf16(k) for k in inp.k]; vs = [dev_bf16(v) for v in inp.v]
    flags = _KERNEL_FLAG[kernel]
    ref_o, ref_l = P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=float(inp.softmax_scale), flags=flags)
    out = torch.empty_like(q)
    desc = P.make_attn_desc(q, ks, out, float(inp.softmax_scale), flags | 16)
    ws = torch.full((P.usp_ring_attn_workspace_bytes(desc),), 0xFF, dtype=torch.uint8, device=DEV)
    for _ in range(2):
        o, l = P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=float(inp.softmax_scale), flags=flags | 16,
                                   out=out, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(o, ref_o) and torch.equal(l, ref_l)
    ro, rl = _oracle(inp)
    _assert_parity(host_f64(o), host_f64(l), ro, rl)


def test_one_launch_with_transfers_inside_alternating_inputs_share_a_workspace():
    """Two different rings of the same shape take turns through one workspace: a staging line left in
    some cache by the previous call would surface as the other ring's keys."""
    P = _P()
    shape = (1, 6, 128, 700, (512, 256, 320))
    runs = []
    for seed in (45, 46):
        inp = W.make_attention_inputs(W.Workload("pipe1_alt", seed, *shape, "bf16"))
        q = dev_bf16(inp.q); ks = [dev_bf16(k) for k in inp.k]; vs = [dev_bf16(v) for v in inp.v]
        ref = P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=float(inp.softmax_scale))
        runs.append((inp, q, ks, vs, ref))
    torch.cuda.synchronize()
    assert not torch.equal(runs[0][4][0], runs[1][4][0])
    desc = P.make_attn_desc(runs[0][1], runs[0][2], torch.empty_like(runs[0][1]), float(runs[0][0].softmax_scale), 16)
    ws = torch.full((P.usp_ring_attn_workspace_bytes(desc),), 0xFF, dtype=torch.uint8, device=DEV)
    for it in range(6):
        inp, q, ks, vs, (ref_o, ref_l) = runs[it & 1]
        o, l = P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=float(inp.softmax_scale), flags=16, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(o, ref_o) and torch.equal(l, ref_l), it
    # back to back without synchronising in between
    outs = []
    for it in range(6):
        inp, q, ks, vs, _ = runs[it & 1]
        outs.append(P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=float(inp.softmax_scale), flags=16, workspace=ws))
    torch.cuda.synchronize()
    for it, (o, l) in enumerate(outs):
        assert torch.equal(o, runs[it & 1][4][0]) and torch.equal(l, runs[it & 1][4][1]), it


def test_one_launch_falls_back_beyond_sixteen_chunks_and_for_masks():
    wl = W.Workload("multi_17", 42, 1, 2, 128, 150, (64,) * 17, "bf16")
    inp = W.make_attention_inputs(wl)
    ro, rl = _oracle(inp)
    o, l = _run(inp)
    _assert_parity(o, l, ro, rl)
    o2, l2 = _run(inp, flags=64)
    np.testing.assert_array_equal(o, o2)         # 17 chunks: the plain call is the stepwise one
    np.testing.assert_array_equal(l, l2)


def test_one_launch_strided_kv_chunks():
    """Chunks that are slices of one [B, H, S, d] array (a common kv_stride instead of dense chunks)."""
    P = _P()
    wl = W.Workload("multi_strided", 43, 2, 3, 128, 190, (128, 256, 64), "bf16")
    inp = W.make_attention_inputs(wl)
    ro, rl = _oracle(inp)
    q = dev_bf16(inp.q)
    kfull = dev_bf16(np.concatenate(inp.k, axis=2))
    vfull = dev_bf16(np.concatenate(inp.v, axis=2))
    bounds = np.cumsum((0,) + wl.chunk_len)
    ks = [kfull[:, :, a:b] for a, b in zip(bounds[:-1], bounds[1:])]
    vs = [vfull[:, :, a:b] for a, b in zip(bounds[:-1], bounds[1:])]
    assert not ks[1].is_contiguous()
    for flags in (0, 64):
        o, l = P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=float(inp.softmax_scale), flags=flags)
        torch.cuda.synchronize()
        _assert_parity(host_f64(o), host_f64(l), ro, rl)


def test_long_sequence_16k_keys_single_chunk_and_ragged_ring():
    """A 2048 x 2048-image-sized sequence (16 896 tokens + a ragged remainder) on 3 heads: one chunk
    of 16 896 keys (264 tiles per work-group) on the plain kernels, and the same keys plus 40 more
    as three unequal chunks, the last of them ragged (extended kernels, merge, fused prefetch)."""
    wl = W.Workload("long16k", 31, 1, 3, 128, 1000, (16896,), "bf16", k_mul=0.5)
    inp = W.make_attention_inputs(wl)
    rows = W.sample_rows(5, wl.Sq, 40)
    ro, rl = _oracle(inp, rows)
    for kernel in ("auto", "wide"):
        o, l = _run(inp, flags=_KERNEL_FLAG[kernel])
        _assert_parity(o[:, :, rows], l[:, :, rows], ro, rl)
    wl2 = W.Workload("long16k_r3", 32, 1, 3, 128, 1000, (8192, 6400, 2344), "bf16", k_mul=0.5)
    inp2 = W.make_attention_inputs(wl2)
    ro2, rl2 = _oracle(inp2, rows)
    for flags in (0, 16):
        o2, l2 = _run(inp2, flags=flags)
        _assert_parity(o2[:, :, rows], l2[:, :, rows], ro2, rl2)


def test_flux2048_u2r8_full_size_every_row():
    """Config 4 shapes: H=12, Q shard 2112 (8.25 query blocks), eight chunks of 2112 (33 tiles),
    per-head scales U(0.5,2); every row of every head against the oracle, for the double-buffered
    call and for each launch configuration bench.py times on this shard."""
    wl = W.WORKLOADS["flux2048_u2r8"]
    inp = W.make_attention_inputs(wl)
    side = torch.cuda.Stream()
    ro, rl = _oracle(inp)
    o, l = _run(inp, flags=1, copy_stream=side)
    assert o.shape == ro.shape == (1, 12, 2112, 128)
    _assert_parity(o, l, ro, rl)
    for h in range(wl.H):
        _assert_parity(o[:, h:h + 1], l[:, h:h + 1], ro[:, h:h + 1], rl[:, h:h + 1])
    os_, ls_ = _run(inp, flags=64)               # resident chunks, one launch per chunk
    np.testing.assert_array_equal(os_, o); np.testing.assert_array_equal(ls_, l)
    of, lf = _run(inp, flags=16 | 64)            # ... each carrying the next transfer
    np.testing.assert_array_equal(of, o); np.testing.assert_array_equal(lf, l)
    o1, l1 = _run(inp)                           # the eight resident chunks in one launch
    _assert_parity(o1, l1, ro, rl)
    for h in range(wl.H):
        _assert_parity(o1[:, h:h + 1], l1[:, h:h + 1], ro[:, h:h + 1], rl[:, h:h + 1])
    op, lp = _run(inp, flags=16)                 # one launch with the seven transfers inside
    np.testing.assert_array_equal(op, o1); np.testing.assert_array_equal(lp, l1)


def test_qwen_r2_full_size_fp8_kv_masked_every_row():
    """Config 5 shapes: H=24, Q shard 4096, two chunks of 4096, 1 % x20 outliers, keys 7802..8191
    masked, K/V quantised per (head, token) by the library and consumed as codes + scales.
    Gate: every row of every head against the oracle attending over the exactly dequantised values,
    for the plain call (what bench.py times) and the side-stream double buffering.
    Reported (not gated): the error against the oracle on the unquantised inputs."""
    P = _P()
    wl = W.WORKLOADS["qwen_r2"]
    inp = W.make_attention_inputs(wl)
    q = dev_bf16(inp.q)
    kq, ksc, vq, vsc = [], [], [], []
    for k, v in zip(inp.k, inp.v):
        B, H, L, d = k.shape
        a, sa = P.usp_fp8_quant(dev_bf16(k).reshape(B * H * L, d))
        b, sb = P.usp_fp8_quant(dev_bf16(v).reshape(B * H * L, d))
        kq.append(a.reshape(B, H, L, d)); ksc.append(sa.reshape(B, H, L))
        vq.append(b.reshape(B, H, L, d)); vsc.append(sb.reshape(B, H, L))
    km = [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    kx = [orc.dequant_exact_f64(a.cpu().numpy(), s_.cpu().numpy()) for a, s_ in zip(kq, ksc)]
    vx = [orc.dequant_exact_f64(a.cpu().numpy(), s_.cpu().numpy()) for a, s_ in zip(vq, vsc)]
    ro, rl = orc.ring_attention(inp.q, kx, vx, float(inp.softmax_scale), inp.key_mask)
    del kx, vx
    side = torch.cuda.Stream()
    for flags, cs in ((0, None), (1, side)):
        o, l = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, key_mask=km,
                                   softmax_scale=float(inp.softmax_scale), flags=flags, copy_stream=cs)
        torch.cuda.synchronize()
        o, l = host_f64(o), host_f64(l)
        assert o.shape == ro.shape == (1, 24, 4096, 128)
        _assert_parity(o, l, ro, rl)
        for h in range(wl.H):
            _assert_parity(o[:, h:h + 1], l[:, h:h + 1], ro[:, h:h + 1], rl[:, h:h + 1])
    # accuracy of FP8 K/V against unquantised inputs (report only)
    uo, ul = orc.ring_attention(inp.q, inp.k, inp.v, float(inp.softmax_scale), inp.key_mask)
    mx, rel = attn_errors(o, uo)
    print("qwen_r2 FP8 K/V vs unquantised oracle: max-abs %.3g rel-L2 %.3g lse max-abs %.3g"
          % (mx, rel, np.abs(l - ul).max()))


def test_invalid_arguments_are_rejected():
    P = _P()
    q = torch.zeros((1, 1, 16, 128), dtype=torch.bfloat16, device=DEV)
    k = torch.zeros((1, 1, 16, 128), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(P.UspError) as e:
        P.usp_ring_attn_fwd(q, [k, k], [k, k], flags=1, copy_stream=None,
                            workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    assert e.value.status == -3
    with pytest.raises(P.UspError) as e:
        P.usp_ring_attn_fwd(q[..., 1:], [k], [k])      # misaligned, d = 127
    assert e.value.status == -1
    with pytest.raises(P.UspError):
        P.usp_fp8_quant(torch.zeros((4, 12), dtype=torch.bfloat16, device=DEV))


@pytest.mark.parametrize("flags", [0, 64, 16])
def test_long_sequence_65536_keys_sampled_rows(flags):
    """A 64K-key ring (4 chunks of 16384) against the oracle on sampled query rows: tile counts, byte
    offsets and the running sums far beyond the benchmark shapes."""
    wl = W.Workload("long", 77, 1, 2, 128, 512, (16384,) * 4, "bf16")
    inp = W.make_attention_inputs(wl)
    o, l = _run(inp, flags=flags)
    rows = np.array([0, 1, 31, 32, 127, 128, 255, 256, 300, 511])
    ro, rl = _oracle(inp, rows)
    _assert_parity(o[:, :, rows, :], l[:, :, rows], ro, rl)


@pytest.mark.parametrize("masked", [False, True])
def test_largest_batch_times_heads_sampled_pairs(masked):
    """65532 (batch, head) pairs, next to the most the launch grids take (65535): short shards, two
    chunks, inputs drawn on the device from a seeded generator; sampled pairs against the oracle.  With
    key masks the per-tile records are prepared by a launch whose second grid dimension is the pairs."""
    P = _P()
    B, H, Sq, lens, d = 3, 21844, 40, (128, 64), 128
    gen = torch.Generator(device=DEV)
    gen.manual_seed(4242)

    def draw(*shape):
        return torch.randn(shape, generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)

    q = draw(B, H, Sq, d)
    ks = [draw(B, H, L, d) for L in lens]
    vs = [draw(B, H, L, d) for L in lens]
    km = None
    if masked:
        km = [torch.ones((B, L), dtype=torch.uint8, device=DEV) for L in lens]
        km[0][1, 100:] = 0; km[1][1, :22] = 0        # entry 1: keys 100..149 of the ring are dead
        km[1][2, :] = 0                              # entry 2: the whole second chunk
    scale = 1.0 / np.sqrt(d)
    o, l = P.usp_ring_attn_fwd(q, ks, vs, key_mask=km, softmax_scale=float(np.float32(scale)))
    torch.cuda.synchronize()
    rng = np.random.Generator(np.random.PCG64(4243))
    pairs = [(0, 0), (0, 1), (1, 7), (1, H - 1), (2, 0), (2, H - 1)] + \
            [(int(rng.integers(0, B)), int(rng.integers(0, H))) for _ in range(10)]
    for b, h in pairs:
        sl = lambda t: host_f64(t[b:b + 1, h:h + 1])
        mk = None if km is None else [m[b:b + 1].cpu().numpy() for m in km]
        ro, rl = orc.ring_attention(sl(q), [sl(k) for k in ks], [sl(v) for v in vs], float(np.float32(scale)), mk)
        _assert_parity(sl(o), host_f64(l[b:b + 1, h:h + 1]), ro, rl)


@pytest.mark.parametrize("kernel", ["auto", "wide", "split"])
@pytest.mark.parametrize("B,Sq,lens,masked", [
    (1, 200, (128, 64, 192), (100, 250)),          # dead keys across a chunk boundary
    (2, 300, (64, 128, 64, 64), (64, 192)),        # one chunk entirely dead
    (3, 130, (256, 128), (0, 70)),                 # the ring starts with dead keys
    (1, 257, (128, 0, 192, 64), (383, 384)),       # a single dead key, the last one; an empty chunk
])
def test_one_launch_over_bf16_chunks_with_key_masks(B, Sq, lens, masked, kernel):
    """bf16 chunks of whole tiles with key masks are covered by one launch too, through per-tile records
    written just before it: parity, agreement with the launch-per-chunk form, and the same with the
    transfers inside the launch (poisoned workspace)."""
    P = _P()
    wl = W.Workload("multi_masked", 47, B, 3, 128, Sq, tuple(lens), "bf16", masked_keys=masked)
    inp = W.make_attention_inputs(wl)
    if B == 3:                                     # a different mask per batch entry
        for m in inp.key_mask:
            m[0, :] = 1
        inp.key_mask[0][2, ::3] = 0
    ro, rl = _oracle(inp)
    flags = _KERNEL_FLAG[kernel]
    o, l = _run(inp, flags=flags)
    _assert_parity(o, l, ro, rl)
    os_, ls_ = _run(inp, flags=flags | 64)
    _assert_parity(os_, ls_, ro, rl)
    assert np.abs(o - os_).max() <= 2.0 ** -6 and np.abs(l - ls_).max() <= 1e-5
    q = dev_bf16(inp.q); ks = [dev_bf16(k) for k in inp.k]; vs = [dev_bf16(v) for v in inp.v]
    km = [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    out = torch.empty_like(q)
    desc = P.make_attn_desc(q, ks, out, float(inp.softmax_scale), flags | 16)
    ws = torch.full((P.usp_ring_attn_workspace_bytes(desc),), 0xFF, dtype=torch.uint8, device=DEV)
    for _ in range(2):
        of, lf = P.usp_ring_attn_fwd(q, ks, vs, key_mask=km, softmax_scale=float(inp.softmax_scale), flags=flags | 16,
                                     out=out, workspace=ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host_f64(of), o)
    np.testing.assert_array_equal(host_f64(lf), l)


def test_one_launch_masked_ring_with_every_key_of_an_entry_dead():
    """A batch entry whose keys are all dead: lse = -inf and O = 0 for its rows, the other entry unaffected."""
    wl = W.Workload("multi_masked_all", 48, 2, 2, 128, 140, (128, 64), "bf16", masked_keys=(0, 0))
    inp = W.make_attention_inputs(wl)
    inp.key_mask = [np.ones((2, L), dtype=np.uint8) for L in wl.chunk_len]
    for m in inp.key_mask:
        m[1, :] = 0
    ro, rl = _oracle(inp)
    o, l = _run(inp)
    _assert_parity(o, l, ro, rl)
    assert np.all(np.isneginf(l[1])) and np.all(o[1] == 0.0) and np.all(np.isfinite(l[0]))
