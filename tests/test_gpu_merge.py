"""usp_lse_merge parity against the oracle's merge (section 3.4 equations)."""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from tests.gpu_util import DEV, dev_bf16, dev_f32, host_f64

pytestmark = pytest.mark.gpu


def _inputs(seed, rows, d, bf16):
    rng = np.random.Generator(np.random.PCG64(seed))
    o1 = rng.standard_normal((rows, d), dtype=np.float32)
    o2 = rng.standard_normal((rows, d), dtype=np.float32)
    l1 = (rng.standard_normal(rows, dtype=np.float32) * 4).astype(np.float32)
    l2 = (rng.standard_normal(rows, dtype=np.float32) * 4).astype(np.float32)
    if bf16:
        from paper_2602_10940_amd import workloads as W
        o1 = W.bf16_bits_to_f32(W.f32_to_bf16_bits(o1))
        o2 = W.bf16_bits_to_f32(W.f32_to_bf16_bits(o2))
    return o1, l1, o2, l2


@pytest.mark.parametrize("rows,d,bf16", [(256, 64, False), (1000, 128, True), (77, 128, False),
                                         (5, 8, True), (130, 24, False), (9, 200, True),
                                         (3, 512, False), (27648, 128, True)])
def test_merge_matches_oracle(rows, d, bf16):
    import paper_2602_10940_amd as P
    o1, l1, o2, l2 = _inputs(rows + d, rows, d, bf16)
    up = dev_bf16 if bf16 else dev_f32
    o, l = P.usp_lse_merge(up(o1), dev_f32(l1), up(o2), dev_f32(l2))
    torch.cuda.synchronize()
    eo, el = orc.lse_merge(o1, l1, o2, l2)
    np.testing.assert_allclose(host_f64(l), el, rtol=0, atol=2e-6 * max(1.0, np.abs(el).max()))
    tol = (2.0 ** -8) if bf16 else 4e-6
    assert np.all(np.abs(host_f64(o) - eo) <= tol * np.abs(eo) + 1e-6)


def test_merge_in_place_and_special_values():
    import paper_2602_10940_amd as P
    rows, d = 64, 128
    o1, l1, o2, l2 = _inputs(1, rows, d, False)
    l1[0] = -np.inf; l2[1] = -np.inf; l1[2] = l2[2] = -np.inf
    l1[3], l2[3] = 80.0, 79.0
    l1[4], l2[4] = -80.0, -85.0
    l1[5], l2[5] = 30.0, -60.0
    eo, el = orc.lse_merge(o1, l1, o2, l2)
    a, la = dev_f32(o1), dev_f32(l1)
    o, l = P.usp_lse_merge(a, la, dev_f32(o2), dev_f32(l2), o_out=a, lse_out=la)   # alias first input
    torch.cuda.synchronize()
    got_l, got_o = host_f64(l), host_f64(o)
    assert np.isneginf(got_l[2]) and np.all(got_o[2] == 0)
    np.testing.assert_array_equal(got_o[0], o2[0].astype(np.float64)); assert got_l[0] == l2[0]
    np.testing.assert_array_equal(got_o[1], o1[1].astype(np.float64)); assert got_l[1] == l1[1]
    fin = np.isfinite(el)
    np.testing.assert_allclose(got_l[fin], el[fin], rtol=0, atol=1e-5)
    np.testing.assert_allclose(got_o, eo, rtol=0, atol=1e-5)
    # aliasing the second input gives the same numbers
    b, lb = dev_f32(o2), dev_f32(l2)
    o2_, l2_ = P.usp_lse_merge(dev_f32(o1), dev_f32(l1), b, lb, o_out=b, lse_out=lb)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host_f64(o2_), got_o)


def test_merge_commutes_on_device():
    import paper_2602_10940_amd as P
    o1, l1, o2, l2 = _inputs(2, 500, 128, True)
    a = P.usp_lse_merge(dev_bf16(o1), dev_f32(l1), dev_bf16(o2), dev_f32(l2))
    b = P.usp_lse_merge(dev_bf16(o2), dev_f32(l2), dev_bf16(o1), dev_f32(l1))
    torch.cuda.synchronize()
    np.testing.assert_allclose(host_f64(a[1]), host_f64(b[1]), rtol=0, atol=1e-6)
    np.testing.assert_allclose(host_f64(a[0]), host_f64(b[0]), rtol=2.0 ** -7, atol=1e-6)
