"""Pins for the attention / merge part of the fp64 oracle (CPU only).

None of these re-type the oracle's formulas with numpy: they use 50-digit mpmath
loops, closed forms, torch's fp64 library routines, and invariants the paper
states (section 2.2.2: the merged result equals full attention whatever the
chunk order).
"""
import itertools
import math

import mpmath as mp
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc


def _rand(seed, *shape):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


# ---------------------------------------------------------------------------
# brute force, 50 digits
# ---------------------------------------------------------------------------
def _mp_attention_row(qrow, K, V, scale, keep=None):
    mp.mp.dps = 50
    S, d = len(K), len(qrow)
    scores = []
    for j in range(S):
        if keep is not None and not keep[j]:
            scores.append(None)
            continue
        acc = mp.mpf(0)
        for t in range(d):
            acc += mp.mpf(float(qrow[t])) * mp.mpf(float(K[j][t]))
        scores.append(acc * mp.mpf(float(scale)))
    live = [s for s in scores if s is not None]
    Z = sum(mp.e ** s for s in live)
    lse = mp.log(Z)
    out = []
    for t in range(len(V[0])):
        num = mp.mpf(0)
        for j in range(S):
            if scores[j] is not None:
                num += mp.e ** scores[j] * mp.mpf(float(V[j][t]))
        out.append(num / Z)
    return [float(x) for x in out], float(lse)


@pytest.mark.parametrize("Sq,S,d", [(3, 5, 2), (2, 7, 4), (4, 9, 3)])
def test_bruteforce_tiny(Sq, S, d):
    q = _rand(1, 1, 2, Sq, d) * 2.0
    k = _rand(2, 1, 2, S, d) * 2.0
    v = _rand(3, 1, 2, S, d)
    scale = 1.0 / math.sqrt(d)
    o, lse = orc.attention(q, k, v, scale)
    for h in range(2):
        for i in range(Sq):
            eo, el = _mp_attention_row(q[0, h, i], k[0, h], v[0, h], scale)
            np.testing.assert_allclose(o[0, h, i], eo, rtol=0, atol=1e-14)
            assert abs(lse[0, h, i] - el) < 1e-14


def test_bruteforce_masked():
    Sq, S, d = 3, 8, 2
    q, k, v = _rand(4, 1, 1, Sq, d), _rand(5, 1, 1, S, d), _rand(6, 1, 1, S, d)
    keep = np.array([[1, 1, 0, 1, 0, 0, 1, 0]], dtype=np.uint8)
    o, lse = orc.attention(q, k, v, 0.7, keep)
    for i in range(Sq):
        eo, el = _mp_attention_row(q[0, 0, i], k[0, 0], v[0, 0], 0.7, keep[0])
        np.testing.assert_allclose(o[0, 0, i], eo, rtol=0, atol=1e-14)
        assert abs(lse[0, 0, i] - el) < 1e-14


def test_transposed_operand_would_fail():
    # q.k must contract over d: a non-square case where Sq != S != d with asymmetric data
    q = np.zeros((1, 1, 2, 3)); k = np.zeros((1, 1, 4, 3)); v = np.zeros((1, 1, 4, 5))
    q[0, 0, 0] = [1, 0, 0]; q[0, 0, 1] = [0, 2, 0]
    k[0, 0, :, 0] = [0, 1, 2, 3]          # query 0 sees scores 0,1,2,3
    k[0, 0, :, 1] = [3, 2, 1, 0]          # query 1 sees scores 6,4,2,0
    v[0, 0, :, :] = np.arange(20).reshape(4, 5)
    o, lse = orc.attention(q, k, v, 1.0)
    w0 = np.exp([0, 1, 2, 3]); w0 /= w0.sum()
    w1 = np.exp([6, 4, 2, 0]); w1 /= w1.sum()
    np.testing.assert_allclose(o[0, 0, 0], w0 @ v[0, 0], atol=1e-13)
    np.testing.assert_allclose(o[0, 0, 1], w1 @ v[0, 0], atol=1e-13)
    assert abs(lse[0, 0, 0] - math.log(sum(math.exp(x) for x in [0, 1, 2, 3]))) < 1e-13
    assert abs(lse[0, 0, 1] - math.log(sum(math.exp(x) for x in [6, 4, 2, 0]))) < 1e-13


# ---------------------------------------------------------------------------
# closed forms
# ---------------------------------------------------------------------------
def test_equal_keys_gives_mean_of_v():
    S, d = 37, 8
    q = _rand(7, 1, 1, 5, d)
    k = np.broadcast_to(_rand(8, 1, 1, 1, d), (1, 1, S, d)).copy()
    v = _rand(9, 1, 1, S, d)
    o, lse = orc.attention(q, k, v, 0.25)
    np.testing.assert_allclose(o[0, 0], np.broadcast_to(v[0, 0].mean(0), (5, d)), atol=1e-14)
    s = (q[0, 0] * k[0, 0, 0]).sum(-1) * 0.25
    np.testing.assert_allclose(lse[0, 0], s + math.log(S), atol=1e-13)


def test_zero_q_uniform():
    S, d = 19, 4
    q = np.zeros((1, 2, 3, d))
    k, v = _rand(10, 1, 2, S, d), _rand(11, 1, 2, S, d)
    o, lse = orc.attention(q, k, v, 0.5)
    np.testing.assert_allclose(lse, math.log(S), atol=1e-14)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(2, keepdims=True), o.shape), atol=1e-14)


def test_constant_v_and_shift_invariance():
    S, d = 23, 6
    q, k = _rand(12, 1, 1, 4, d), _rand(13, 1, 1, S, d)
    v = np.full((1, 1, S, d), 3.25)
    o, lse = orc.attention(q, k, v, 0.3)
    np.testing.assert_allclose(o, 3.25, atol=1e-13)
    # adding a constant c to every score of a row (k -> k + c*q/(|q|^2*scale)) is awkward;
    # instead append a coordinate: q' = [q, 1], k' = [k, c/scale] => scores + c
    c = 2.5
    q2 = np.concatenate([q, np.ones((1, 1, 4, 1))], -1)
    k2 = np.concatenate([k, np.full((1, 1, S, 1), c / 0.3)], -1)
    v2 = _rand(14, 1, 1, S, d)
    oa, la = orc.attention(q, k, v2, 0.3)
    ob, lb = orc.attention(q2, k2, v2, 0.3)
    np.testing.assert_allclose(ob, oa, atol=1e-13)
    np.testing.assert_allclose(lb, la + c, atol=1e-13)


def test_dominant_key_selects_its_value():
    S, d = 16, 4
    q = np.zeros((1, 1, 1, d)); q[..., 0] = 1.0
    k = np.zeros((1, 1, S, d)); k[0, 0, 11, 0] = 200.0
    v = _rand(15, 1, 1, S, d)
    o, lse = orc.attention(q, k, v, 1.0)
    np.testing.assert_allclose(o[0, 0, 0], v[0, 0, 11], atol=1e-13)
    assert abs(lse[0, 0, 0] - 200.0) < 1e-13


def test_scale_is_applied_once():
    # doubling scale == doubling q
    q, k, v = _rand(16, 1, 1, 3, 4), _rand(17, 1, 1, 6, 4), _rand(18, 1, 1, 6, 4)
    o1, l1 = orc.attention(q, k, v, 0.8)
    o2, l2 = orc.attention(2 * q, k, v, 0.4)
    np.testing.assert_allclose(o1, o2, atol=1e-14)
    np.testing.assert_allclose(l1, l2, atol=1e-14)


def test_all_keys_masked_row():
    q, k, v = _rand(19, 1, 1, 2, 4), _rand(20, 1, 1, 5, 4), _rand(21, 1, 1, 5, 4)
    o, lse = orc.attention(q, k, v, 1.0, np.zeros((1, 5), np.uint8))
    assert np.all(o == 0) and np.all(np.isneginf(lse))


# ---------------------------------------------------------------------------
# library cross-checks (independent implementation, fp64)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("B,H,Sq,S,d", [(1, 2, 128, 256, 64), (2, 3, 33, 77, 128)])
def test_against_torch_sdpa_and_logsumexp(B, H, Sq, S, d):
    q, k, v = _rand(22, B, H, Sq, d), _rand(23, B, H, S, d), _rand(24, B, H, S, d)
    scale = 1.0 / math.sqrt(d)
    o, lse = orc.attention(q, k, v, scale)
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    to = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale)
    np.testing.assert_allclose(o, to.numpy(), atol=1e-12)
    tl = torch.logsumexp(torch.einsum("bhqd,bhkd->bhqk", tq, tk) * scale, dim=-1)
    np.testing.assert_allclose(lse, tl.numpy(), atol=1e-12)


def test_against_torch_sdpa_masked():
    B, H, Sq, S, d = 1, 2, 17, 40, 16
    q, k, v = _rand(25, B, H, Sq, d), _rand(26, B, H, S, d), _rand(27, B, H, S, d)
    keep = np.ones((B, S), np.uint8); keep[:, 29:] = 0
    o, _ = orc.attention(q, k, v, 0.25, keep)
    m = torch.from_numpy(keep.astype(bool))[:, None, None, :]
    to = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q), torch.from_numpy(k), torch.from_numpy(v), attn_mask=m, scale=0.25)
    np.testing.assert_allclose(o, to.numpy(), atol=1e-12)


# ---------------------------------------------------------------------------
# chunking + merge == one shot, any order (section 2.2.2)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("lens", [(64,), (40, 24), (16, 16, 16, 16), (5, 30, 1, 28),
                                  (8,) * 8])
def test_ring_equals_one_shot_every_order(lens):
    B, H, Sq, d = 1, 2, 9, 8
    S = sum(lens)
    q, k, v = _rand(28, B, H, Sq, d) * 3, _rand(29, B, H, S, d), _rand(30, B, H, S, d)
    full_o, full_l = orc.attention(q, k, v, 0.35)
    offs = np.cumsum((0,) + tuple(lens))
    kc = [k[:, :, offs[i]:offs[i + 1]] for i in range(len(lens))]
    vc = [v[:, :, offs[i]:offs[i + 1]] for i in range(len(lens))]
    perms = list(itertools.permutations(range(len(lens))))
    if len(perms) > 24:
        rng = np.random.default_rng(0)
        perms = [tuple(rng.permutation(len(lens))) for _ in range(24)]
    for p in perms:
        o, l = orc.ring_attention(q, kc, vc, 0.35, order=p)
        np.testing.assert_allclose(o, full_o, atol=1e-12)
        np.testing.assert_allclose(l, full_l, atol=1e-12)


def test_ring_with_masked_tail_chunk_and_fully_masked_chunk():
    B, H, Sq, d = 1, 1, 4, 4
    q, k, v = _rand(31, B, H, Sq, d), _rand(32, B, H, 24, d), _rand(33, B, H, 24, d)
    keep = np.ones((B, 24), np.uint8); keep[:, 13:] = 0          # chunk 2 fully masked
    full_o, full_l = orc.attention(q, k, v, 0.5, keep)
    kc = [k[:, :, i * 8:(i + 1) * 8] for i in range(3)]
    vc = [v[:, :, i * 8:(i + 1) * 8] for i in range(3)]
    mc = [keep[:, i * 8:(i + 1) * 8] for i in range(3)]
    for p in itertools.permutations(range(3)):
        o, l = orc.ring_attention(q, kc, vc, 0.5, mc, order=p)
        np.testing.assert_allclose(o, full_o, atol=1e-13)
        np.testing.assert_allclose(l, full_l, atol=1e-13)


def test_merge_tree_associativity():
    rng = np.random.default_rng(3)
    n, rows, d = 6, 11, 5
    os_ = [rng.standard_normal((rows, d)) for _ in range(n)]
    ls_ = [rng.standard_normal(rows) * 4 for _ in range(n)]

    def fold(idx):
        if len(idx) == 1:
            return os_[idx[0]], ls_[idx[0]]
        cut = rng.integers(1, len(idx))
        a, b = fold(idx[:cut]), fold(idx[cut:])
        return orc.lse_merge(a[0], a[1], b[0], b[1])

    ref = fold(list(range(n)))
    for _ in range(10):
        got = fold(list(rng.permutation(n)))
        np.testing.assert_allclose(got[0], ref[0], atol=1e-13)
        np.testing.assert_allclose(got[1], ref[1], atol=1e-13)


def test_merge_two_forms_agree_and_match_mpmath():
    rng = np.random.default_rng(4)
    o1, o2 = rng.standard_normal((7, 3)), rng.standard_normal((7, 3))
    l1, l2 = rng.standard_normal(7) * 5, rng.standard_normal(7) * 5
    a = orc.lse_merge(o1, l1, o2, l2)
    b = orc.lse_merge_raw(o1, l1, o2, l2)
    np.testing.assert_allclose(a[0], b[0], atol=1e-13)
    np.testing.assert_allclose(a[1], b[1], atol=1e-13)
    mp.mp.dps = 50
    for r in range(7):
        e1, e2 = mp.e ** mp.mpf(float(l1[r])), mp.e ** mp.mpf(float(l2[r]))
        assert abs(a[1][r] - float(mp.log(e1 + e2))) < 1e-13
        for t in range(3):
            ex = (e1 * mp.mpf(float(o1[r, t])) + e2 * mp.mpf(float(o2[r, t]))) / (e1 + e2)
            assert abs(a[0][r, t] - float(ex)) < 1e-13


def test_merge_is_commutative_and_weights_sum_to_one():
    rng = np.random.default_rng(5)
    o1, o2 = rng.standard_normal((9, 4)), rng.standard_normal((9, 4))
    l1, l2 = rng.standard_normal(9) * 3, rng.standard_normal(9) * 3
    a = orc.lse_merge(o1, l1, o2, l2)
    b = orc.lse_merge(o2, l2, o1, l1)
    np.testing.assert_array_equal(a[1], b[1])
    np.testing.assert_allclose(a[0], b[0], atol=1e-15)
    ones = np.ones((9, 4))
    c = orc.lse_merge(ones, l1, ones, l2)                       # convex combination
    np.testing.assert_allclose(c[0], 1.0, atol=1e-15)
    # wrong sign in the exponent would give weights > 1 here:
    assert np.all(a[1] >= np.maximum(l1, l2))
    assert np.all(a[1] <= np.maximum(l1, l2) + math.log(2) + 1e-15)


def test_merge_infinities_and_large_lse():
    o1 = np.array([[1.0, 2.0]] * 4); o2 = np.array([[5.0, -1.0]] * 4)
    l1 = np.array([-np.inf, 0.3, -np.inf, 700.0])
    l2 = np.array([0.5, -np.inf, -np.inf, 699.0])
    o, l = orc.lse_merge(o1, l1, o2, l2)
    np.testing.assert_array_equal(o[0], o2[0]); assert l[0] == 0.5
    np.testing.assert_array_equal(o[1], o1[1]); assert l[1] == 0.3
    assert np.all(o[2] == 0) and np.isneginf(l[2])
    assert abs(l[3] - (700.0 + math.log1p(math.exp(-1.0)))) < 1e-12
    w = 1.0 / (1.0 + math.exp(-1.0))
    np.testing.assert_allclose(o[3], w * o1[3] + (1 - w) * o2[3], atol=1e-13)
