"""Seeded random sweep of usp_ring_attn_fwd against the fp64 oracle: head dimension 64 / 128, batch,
heads, Q shard length, 1-5 chunks (whole tiles or ragged, empty chunks included), bf16 or FP8 K/V,
key masks (shared or per batch entry), x20 outliers, every schedule / kernel flag, and (one seed) the
softmax scale at 0.25 to 6 times 1/sqrt(d).  Small shapes; each case is printed before it runs."""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from paper_2602_10940_amd import workloads as W
from tests.gpu_util import DEV, dev_bf16, host_f64
from tests.test_gpu_attention import _assert_parity

pytestmark = pytest.mark.gpu

FLAGS = [0, 64, 16, 16 | 64, 1, 2, 4, 8, 32, 16 | 8, 16 | 4, 2 | 16, 64 | 8, 64 | 4]


def _case(rng, case, vary_scale=False):
    d = int(rng.choice([128, 128, 64]))
    B = int(rng.choice([1, 1, 2, 3])); H = int(rng.integers(1, 5))
    Sq = int(rng.choice([1, 31, 64, 100, 128, 130, 200, 256, 300, 520, 700]))
    n = int(rng.integers(1, 6))
    whole = rng.random() < 0.6
    lens = tuple(int(64 * rng.integers(0 if n > 1 else 1, 5)) if whole else int(rng.integers(0 if n > 1 else 1, 300))
                 for _ in range(n))
    if sum(lens) == 0:
        lens = lens[:-1] + (64,)
    fp8 = bool(rng.random() < 0.45)
    masked = bool(rng.random() < 0.4)
    flags = int(rng.choice(FLAGS))
    S = sum(lens)
    lo = int(rng.integers(0, S)); hi = int(rng.integers(lo, S + 1))
    outliers = bool(rng.random() < 0.3)
    own_masks = bool(rng.random() < 0.5)
    wl = W.Workload("sweep", 1000 + case, B, H, d, Sq, lens, "bf16", masked_keys=(lo, hi) if masked else (0, 0),
                    outlier_frac=0.01 if outliers else 0.0, outlier_mul=20.0)
    scale_mul = float(rng.choice([0.25, 1.0, 2.5, 6.0])) if vary_scale else 1.0
    return wl, fp8, flags, own_masks, scale_mul


@pytest.mark.parametrize("seed,vary_scale", [(7, False), (10, False), (13, False), (17, True)])
def test_random_sweep(seed, vary_scale):
    import paper_2602_10940_amd as P
    rng = np.random.Generator(np.random.PCG64(seed))
    for case in range(40):
        wl, fp8, flags, own_masks, scale_mul = _case(rng, case, vary_scale)
        print("case", seed, case, dict(d=wl.d, B=wl.B, H=wl.H, Sq=wl.Sq, lens=wl.chunk_len, fp8=fp8, masked=wl.masked_keys,
                                       flags=flags, scale_mul=scale_mul), flush=True)
        inp = W.make_attention_inputs(wl)
        if inp.key_mask is not None and own_masks and wl.B > 1:     # entry 0 keeps every key
            for m in inp.key_mask:
                m[0, :] = 1
        q = dev_bf16(inp.q)
        km = None if inp.key_mask is None else [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
        side = torch.cuda.Stream() if flags & 1 else None
        scale = float(np.float32(float(inp.softmax_scale) * scale_mul))
        if fp8:
            kq, ksc, vq, vsc, kx, vx = [], [], [], [], [], []
            for k, v in zip(inp.k, inp.v):
                b_, h_, L, dd = k.shape
                if L == 0:
                    kq.append(torch.empty((b_, h_, 0, dd), dtype=torch.uint8, device=DEV)); vq.append(kq[-1])
                    ksc.append(torch.empty((b_, h_, 0), dtype=torch.float32, device=DEV)); vsc.append(ksc[-1])
                    kx.append(k.astype(np.float64)); vx.append(v.astype(np.float64))
                    continue
                a, sa = P.usp_fp8_quant(dev_bf16(k).reshape(b_ * h_ * L, dd))
                b2, sb = P.usp_fp8_quant(dev_bf16(v).reshape(b_ * h_ * L, dd))
                kq.append(a.reshape(b_, h_, L, dd)); ksc.append(sa.reshape(b_, h_, L))
                vq.append(b2.reshape(b_, h_, L, dd)); vsc.append(sb.reshape(b_, h_, L))
                kx.append(orc.dequant_exact_f64(a.cpu().numpy().reshape(b_, h_, L, dd), sa.cpu().numpy().reshape(b_, h_, L)))
                vx.append(orc.dequant_exact_f64(b2.cpu().numpy().reshape(b_, h_, L, dd), sb.cpu().numpy().reshape(b_, h_, L)))
            o, l = P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, key_mask=km, softmax_scale=scale, flags=flags,
                                       copy_stream=side)
            torch.cuda.synchronize()
            ro, rl = orc.ring_attention(inp.q, kx, vx, scale, inp.key_mask)
        else:
            ks = [dev_bf16(k) for k in inp.k]; vs = [dev_bf16(v) for v in inp.v]
            o, l = P.usp_ring_attn_fwd(q, ks, vs, key_mask=km, softmax_scale=scale, flags=flags, copy_stream=side)
            torch.cuda.synchronize()
            ro, rl = orc.ring_attention(inp.q, inp.k, inp.v, scale, inp.key_mask)
        _assert_parity(host_f64(o), host_f64(l), ro, rl)
