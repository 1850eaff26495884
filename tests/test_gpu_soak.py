"""Many calls of one form through one workspace, a few inputs of the same shape taking turns: every
result must equal the bits of its input's own reference.  Catches what single calls do not: state
left in the workspace or in a cache by the previous call, and rare timing-dependent faults of the
launches that exchange data between work-groups while they run."""
import numpy as np
import pytest
import torch

from paper_2602_10940_amd import workloads as W
from tests.gpu_util import DEV, dev_bf16

pytestmark = pytest.mark.gpu

STEPWISE, FUSED, DBUF, UNFUSED, WIDE, SPLIT, MIXED = 64, 16, 1, 2, 4, 8, 32


def _inputs(kind, seed, B, H, d, Sq, lens, masked):
    import paper_2602_10940_amd as P
    wl = W.Workload("soak", seed, B, H, d, Sq, lens, "bf16", masked_keys=masked)
    inp = W.make_attention_inputs(wl)
    km = None if inp.key_mask is None else [torch.from_numpy(m).to(DEV) for m in inp.key_mask]
    r = dict(q=dev_bf16(inp.q), key_mask=km, softmax_scale=float(inp.softmax_scale))
    if kind == "fp8":
        kq, ksc, vq, vsc = [], [], [], []
        for k, v in zip(inp.k, inp.v):
            b_, h_, L, dd = k.shape
            a, sa = P.usp_fp8_quant(dev_bf16(k).reshape(b_ * h_ * L, dd))
            b2, sb = P.usp_fp8_quant(dev_bf16(v).reshape(b_ * h_ * L, dd))
            kq.append(a.reshape(b_, h_, L, dd)); ksc.append(sa.reshape(b_, h_, L))
            vq.append(b2.reshape(b_, h_, L, dd)); vsc.append(sb.reshape(b_, h_, L))
        r.update(k_chunks=kq, v_chunks=vq, k_scales=ksc, v_scales=vsc)
    else:
        r.update(k_chunks=[dev_bf16(k) for k in inp.k], v_chunks=[dev_bf16(v) for v in inp.v])
    return r


_SHORT = (3, 2, 128, 130, (128, 256, 128, 128))          # short chunks: the work-groups wait at every chunk boundary
_RAGGED = (2, 3, 128, 200, (100, 64, 37, 200))
CASES = [
    ("bf16", _SHORT, (0, 0), (0, FUSED, FUSED | STEPWISE, DBUF, SPLIT | STEPWISE)),
    ("bf16", _SHORT, (441, 583), (0, FUSED, STEPWISE)),
    ("fp8", _SHORT, (0, 0), (0, STEPWISE, FUSED | STEPWISE)),
    ("fp8", _SHORT, (441, 583), (0, WIDE, STEPWISE)),
    ("fp8", _RAGGED, (90, 260), (0, FUSED, DBUF)),
    ("bf16", (3, 2, 64, 130, (128, 256, 128, 128)), (441, 583), (0, FUSED)),
    ("bf16", (1, 8, 128, 1500, (1024,)), (0, 0), (0, SPLIT, MIXED)),
]


@pytest.mark.parametrize("kind,shape,masked,flag_list", CASES)
def test_many_calls_through_one_workspace(kind, shape, masked, flag_list):
    import paper_2602_10940_amd as P
    rings = [_inputs(kind, 400 + i, *shape, masked) for i in range(3)]
    for flags in flag_list:
        kw = dict(copy_stream=torch.cuda.Stream()) if flags & DBUF else {}
        refs = []
        for r in rings:
            refs.append(P.usp_ring_attn_fwd(flags=flags, **kw, **r))
        torch.cuda.synchronize()
        desc = P.make_attn_desc(rings[0]["q"], rings[0]["k_chunks"], torch.empty_like(rings[0]["q"]), rings[0]["softmax_scale"], flags)
        need = P.usp_ring_attn_workspace_bytes(desc)
        ws = torch.full((max(need, 256),), 0xFF, dtype=torch.uint8, device=DEV)
        rng = np.random.Generator(np.random.PCG64(11))
        for batch in range(12):
            outs = []
            for _ in range(50):
                i = int(rng.integers(0, 3))
                outs.append((i, P.usp_ring_attn_fwd(flags=flags, workspace=ws if need else None, **kw, **rings[i])))
            torch.cuda.synchronize()
            bad = sum(1 for i, (o, l) in outs if not (torch.equal(o, refs[i][0]) and torch.equal(l, refs[i][1])))
            assert bad == 0, (flags, batch, bad)        # stop at the first batch with a mismatch
