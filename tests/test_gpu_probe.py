"""usp_probe_mfma_rate: the diagnostic MFMA-rate kernel runs and computes what it claims to."""
import pytest
import torch

from tests.gpu_util import DEV

pytestmark = pytest.mark.gpu


def test_probe_constant_operands_sum_exactly():
    import paper_2602_10940_amd as P
    wgs, iters = 6, 10
    out = torch.full((wgs * 512,), -1.0, dtype=torch.float32, device=DEV)
    clocks = torch.zeros((2,), dtype=torch.int64, device=DEV)
    P.usp_probe_mfma_rate(wgs, iters, False, out, clocks)
    torch.cuda.synchronize()
    # A = 1, B = 0.5: one MFMA adds 16 * 0.5 to each of a lane's 16 accumulator elements; an accumulator
    # takes 8 MFMAs per iteration; a thread sums its 4 accumulators
    want = 4 * 16 * 8 * 8.0 * iters
    assert torch.all(out == want), (out.min().item(), out.max().item(), want)
    cyc, ticks = [int(v) for v in clocks.cpu()]
    assert cyc > 0 and ticks > 0
    assert 200.0 < cyc / ticks * 100.0 < 3000.0   # shader clock in MHz


def test_probe_random_operands_finite():
    import paper_2602_10940_amd as P
    out = torch.empty((4 * 512,), dtype=torch.float32, device=DEV)
    clocks = torch.zeros((2,), dtype=torch.int64, device=DEV)
    P.usp_probe_mfma_rate(4, 50, True, out, clocks)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and out.abs().max() > 0


def test_probe_rejects_bad_arguments():
    import paper_2602_10940_amd as P
    out = torch.empty((512,), dtype=torch.float32, device=DEV)
    clocks = torch.zeros((2,), dtype=torch.int64, device=DEV)
    with pytest.raises(P.UspError):
        P.usp_probe_mfma_rate(1, 0, True, out, clocks)
