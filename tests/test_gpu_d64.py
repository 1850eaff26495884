"""bf16 attention with head dimension 64: the call runs on the matrix-core kernels in their
head-dimension-64 form (128-byte rows of Q, K, V and O read and written in place).  Parity against the
fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from paper_2602_10940_amd import workloads as W
from tests.gpu_util import DEV, dev_bf16, host_f64
from tests.test_gpu_attention import _assert_parity, _oracle, _run

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,H,Sq,lens,flags", [
    (1, 3, 200, (192, 100), 0),            # a ragged chunk: one launch per chunk with key records
    (2, 2, 300, (128, 256, 64), 0),        # whole tiles: one launch over the ring
    (1, 2, 130, (128, 256, 64), 16),       # ... with the transfers inside
    (1, 2, 130, (136,) * 3, 1),            # side-stream double buffering
    (1, 4, 520, (320,), 4),                # one chunk, 256-query work-groups
    (1, 2, 150, (200, 136), 2),            # merge as a separate kernel
    (1, 36, 2048, (128,), 0),              # 288 query blocks: d = 128 would take the mixed launch here
    (1, 3, 300, (128, 64), 32),            # the mixed launch asked for by flag
])
def test_bf16_d64_against_oracle(B, H, Sq, lens, flags):
    wl = W.Workload("d64", 91, B, H, 64, Sq, tuple(lens), "bf16")
    inp = W.make_attention_inputs(wl)
    side = torch.cuda.Stream() if flags == 1 else None
    o, l = _run(inp, flags=flags, copy_stream=side)
    assert o.shape == (B, H, Sq, 64)
    ro, rl = _oracle(inp)
    _assert_parity(o, l, ro, rl)


def test_bf16_d64_with_key_mask_and_strided_layout():
    """[B,S,H,d] storage viewed as [B,H,S,d] for Q, K, V and O, and a key mask over the second chunk."""
    import paper_2602_10940_amd as P
    wl = W.Workload("d64_masked", 92, 2, 3, 64, 140, (200, 136), "bf16", masked_keys=(300, 336))
    inp = W.make_attention_inputs(wl)
    ro, rl = _oracle(inp)
    o, l = _run(inp)
    _assert_parity(o, l, ro, rl)
    whole_k = np.concatenate(inp.k, axis=2); whole_v = np.concatenate(inp.v, axis=2)
    def bshd(x):
        return dev_bf16(np.ascontiguousarray(x.transpose(0, 2, 1, 3))).permute(0, 2, 1, 3)
    q, kk, vv = bshd(inp.q), bshd(whole_k), bshd(whole_v)
    ks = [kk[:, :, :200], kk[:, :, 200:]]; vs = [vv[:, :, :200], vv[:, :, 200:]]
    out = torch.empty((2, 140, 3, 64), dtype=torch.bfloat16, device=DEV).permute(0, 2, 1, 3)
    km = [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    o2, l2 = P.usp_ring_attn_fwd(q, ks, vs, key_mask=km, softmax_scale=float(inp.softmax_scale), out=out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host_f64(o2), o)
    np.testing.assert_array_equal(host_f64(l2), l)


def test_bf16_d64_default_scale_is_that_of_the_original_head_dimension():
    import paper_2602_10940_amd as P
    wl = W.Workload("d64_scale", 93, 1, 2, 64, 100, (128,), "bf16")
    inp = W.make_attention_inputs(wl)
    q = dev_bf16(inp.q); k = dev_bf16(inp.k[0]); v = dev_bf16(inp.v[0])
    o0, l0 = P.usp_ring_attn_fwd(q, [k], [v], softmax_scale=0.0)       # 0: the library's 1 / sqrt(d)
    o1, l1 = P.usp_ring_attn_fwd(q, [k], [v], softmax_scale=0.125)
    torch.cuda.synchronize()
    assert torch.equal(o0, o1) and torch.equal(l0, l1)
    ro, rl = orc.ring_attention(inp.q, inp.k, inp.v, 0.125)
    _assert_parity(host_f64(o0), host_f64(l0), ro, rl)


@pytest.mark.parametrize("lens,flags", [((192, 100), 0), ((128, 256, 64), 0), ((128, 256, 64), 64), ((128, 192), 16),
                                        ((256, 0), 0), ((256, 64, 0), 1), ((0, 128, 0, 64), 16)])   # empty chunks, also last
def test_fp8_kv_d64_ring_against_oracle(lens, flags):
    """FP8 K/V chunks with d = 64 (ragged chunks: one launch per chunk; whole tiles: the one-launch
    form with the decode inside), a key mask over the tail."""
    import paper_2602_10940_amd as P
    S = sum(lens)
    wl = W.Workload("d64_fp8", 94, 2, 3, 64, 150, tuple(lens), "bf16", masked_keys=(S - 40, S))
    inp = W.make_attention_inputs(wl)
    q = dev_bf16(inp.q)
    kq, ksc, vq, vsc, kx, vx = [], [], [], [], [], []
    for k, v in zip(inp.k, inp.v):
        B, H, L, d = k.shape
        if L == 0:
            kq.append(torch.empty((B, H, 0, d), dtype=torch.uint8, device=DEV)); vq.append(kq[-1])
            ksc.append(torch.empty((B, H, 0), dtype=torch.float32, device=DEV)); vsc.append(ksc[-1])
            kx.append(k.astype(np.float64)); vx.append(v.astype(np.float64))
            continue
        a, sa = P.usp_fp8_quant(dev_bf16(k).reshape(B * H * L, d))
        b, sb = P.usp_fp8_quant(dev_bf16(v).reshape(B * H * L, d))
        kq.append(a.reshape(B, H, L, d)); ksc.append(sa.reshape(B, H, L))
        vq.append(b.reshape(B, H, L, d)); vsc.append(sb.reshape(B, H, L))
        kx.append(orc.dequant_exact_f64(a.cpu().numpy().reshape(B, H, L, d), sa.cpu().numpy().reshape(B, H, L)))
        vx.append(orc.dequant_exact_f64(b.cpu().numpy().reshape(B, H, L, d), sb.cpu().numpy().reshape(B, H, L)))
    km = [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    o, l = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, key_mask=km, softmax_scale=float(inp.softmax_scale),
                               flags=flags, copy_stream=torch.cuda.Stream() if flags & 1 else None)
    torch.cuda.synchronize()
    ro, rl = orc.ring_attention(inp.q, kx, vx, float(inp.softmax_scale), inp.key_mask)
    _assert_parity(host_f64(o), host_f64(l), ro, rl)
