"""Pins for the oracle's attention (the standard transformer attention the paper
broadcasts, Sec. 2.1) against things other than itself: hand-worked values,
closed forms, invariants, and library routines."""
import math

import numpy as np
import pytest
import torch

from oracle import pab_oracle as orc


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def att1(q, k, v):
    """single problem helper: q [Sq,D], k,v [Sk,D]"""
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    return orc.attention(q[None, :, None, :], k[None, :, None, :], v[None, :, None, :])[0, :, 0, :]


# ---- hand-worked fixtures ------------------------------------------------------
def test_worked_examples(golden_attention):
    ln = math.log
    o = att1([[1.0]], [[0.0], [ln(2)]], [[3.0], [6.0]])
    np.testing.assert_allclose(o[0], golden_attention["A_out"], rtol=0, atol=1e-14)

    o = att1([[2, 0, 0, 0]],
             [[ln(3), 0, 0, 0], [0, 7, 0, 0], [ln(4), 0, 0, 0]],
             [[8, 0, 0, 1], [0, 8, 0, 1], [16, 8, -8, 1]])
    np.testing.assert_allclose(o[0], golden_attention["B_out"], rtol=0, atol=1e-13)

    r2 = math.sqrt(2)
    o = att1([[1, 0], [0, 1]], [[r2 * ln(2), 0], [0, r2 * ln(5)]], [[3, 0], [0, 6]])
    np.testing.assert_allclose(o[0], golden_attention["C_out1"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(o[1], golden_attention["C_out2"], rtol=0, atol=1e-13)


# ---- closed forms --------------------------------------------------------------
def test_single_key_returns_its_value():
    q, k, v = rnd((5, 8), 1), rnd((1, 8), 2), rnd((1, 8), 3)
    np.testing.assert_allclose(att1(q, k, v), np.repeat(v, 5, 0), atol=1e-15)


def test_two_keys_sigmoid():
    D = 6
    q, k, v = rnd((4, D), 4), rnd((2, D), 5), rnd((2, D), 6)
    o = att1(q, k, v)
    for i in range(4):
        delta = (q[i] @ k[0] - q[i] @ k[1]) / math.sqrt(D)
        w = 1.0 / (1.0 + math.exp(-delta))
        np.testing.assert_allclose(o[i], w * v[0] + (1 - w) * v[1], atol=1e-14)


def test_identical_keys_give_mean_of_values():
    q, v = rnd((7, 16), 7), rnd((9, 16), 8)
    k = np.repeat(rnd((1, 16), 9), 9, 0)
    np.testing.assert_allclose(att1(q, k, v), np.repeat(v.mean(0, keepdims=True), 7, 0), atol=1e-14)


def test_rows_of_softmax_sum_to_one_and_are_positive():
    # V = identity exposes the probability rows themselves
    Sk = 11
    q, k = rnd((6, 5), 10), rnd((Sk, 5), 11)
    k = np.concatenate([k, np.zeros((Sk, Sk - 5))], 1)
    q = np.concatenate([q, np.zeros((6, Sk - 5))], 1)
    p = att1(q, k, np.eye(Sk))
    assert (p > 0).all()
    np.testing.assert_allclose(p.sum(1), 1.0, atol=1e-14)


def test_constant_values_and_convex_hull():
    q, k, v = rnd((8, 4), 12), rnd((10, 4), 13), rnd((10, 4), 14)
    o = att1(q, k, np.full((10, 4), 2.5))
    np.testing.assert_allclose(o, 2.5, atol=1e-14)
    o = att1(q, k, v)
    assert (o <= v.max(0) + 1e-14).all() and (o >= v.min(0) - 1e-14).all()


def test_sharp_queries_pick_argmax_value():
    q, k, v = rnd((5, 8), 15), rnd((12, 8), 16), rnd((12, 8), 17)
    o = att1(q * 1e4, k, v)
    np.testing.assert_allclose(o, v[(q @ k.T).argmax(1)], atol=1e-9)


def test_large_logits_do_not_overflow():
    q = np.full((1, 4), 300.0)
    k = np.array([[300.0] * 4, [299.0] * 4])
    o = att1(q, k, np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]]))
    assert np.isfinite(o).all() and o[0, 0] > 0.999999


# ---- invariants ------------------------------------------------------------------
def test_key_shift_and_joint_permutation_and_linearity():
    q, k, v, v2 = rnd((6, 8), 18), rnd((13, 8), 19), rnd((13, 8), 20), rnd((13, 8), 21)
    o = att1(q, k, v)
    # adding one vector to every key shifts each row's logits by a constant
    np.testing.assert_allclose(att1(q, k + rnd((1, 8), 22), v), o, atol=1e-12)
    perm = np.random.default_rng(23).permutation(13)
    np.testing.assert_allclose(att1(q, k[perm], v[perm]), o, atol=1e-13)
    np.testing.assert_allclose(att1(q, k, 2 * v - 3 * v2), 2 * o - 3 * att1(q, k, v2), atol=1e-12)
    # permuting queries permutes outputs
    qp = np.random.default_rng(24).permutation(6)
    np.testing.assert_allclose(att1(q[qp], k, v), o[qp], atol=1e-15)


def test_scale_is_one_over_sqrt_d():
    # doubling D by zero-padding changes only the scale: sqrt(2) on q undoes it
    q, k, v = rnd((4, 8), 25), rnd((9, 8), 26), rnd((9, 8), 27)
    z = np.zeros_like
    o = att1(q, k, v)
    qpad, kpad = np.concatenate([q * math.sqrt(2), z(q)], 1), np.concatenate([k, z(k)], 1)
    vpad = np.concatenate([v, z(v)], 1)
    np.testing.assert_allclose(att1(qpad, kpad, vpad)[:, :8], o, atol=1e-13)


# ---- library second opinions -----------------------------------------------------
@pytest.mark.parametrize("B,H,Sq,Sk,D", [(2, 3, 5, 7, 4), (1, 2, 33, 17, 72), (3, 1, 1, 9, 32)])
def test_against_torch_sdpa_fp64(B, H, Sq, Sk, D):
    q, k, v = rnd((B, Sq, H, D), 30), rnd((B, Sk, H, D), 31), rnd((B, Sk, H, D), 32)
    tq, tk, tv = (torch.from_numpy(a).permute(0, 2, 1, 3) for a in (q, k, v))
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(orc.attention(q, k, v), want, atol=1e-12)


def test_against_scipy_softmax():
    from scipy.special import softmax
    q, k, v = rnd((6, 10), 33), rnd((8, 10), 34), rnd((8, 10), 35)
    want = softmax(q @ k.T / math.sqrt(10), axis=1) @ v
    np.testing.assert_allclose(att1(q, k, v), want, atol=1e-13)


# ---- the three views of [T, S, H, D] ------------------------------------------------
def test_views_spatial_temporal_cross():
    T, S, H, D, L = 3, 5, 2, 4, 6
    q, k, v = rnd((T, S, H, D), 40), rnd((T, S, H, D), 41), rnd((T, S, H, D), 42)
    sp = orc.spatial(q, k, v)
    tm = orc.temporal(q, k, v)
    for h in range(H):
        for t in range(T):   # spatial: tokens of frame t among themselves
            np.testing.assert_allclose(sp[t, :, h], att1(q[t, :, h], k[t, :, h], v[t, :, h]), atol=1e-14)
        for s in range(S):   # temporal: frames at position s among themselves
            np.testing.assert_allclose(tm[:, s, h], att1(q[:, s, h], k[:, s, h], v[:, s, h]), atol=1e-14)
    # temporal equals the generic routine on an explicitly transposed copy
    qt, kt, vt = (np.ascontiguousarray(a.transpose(1, 0, 2, 3)) for a in (q, k, v))
    np.testing.assert_allclose(tm, orc.attention(qt, kt, vt).transpose(1, 0, 2, 3), atol=1e-15)
    # one frame: temporal attention is the identity on V
    np.testing.assert_allclose(orc.temporal(q[:1], k[:1], v[:1]), v[:1], atol=1e-15)
    kc, vc = rnd((L, H, D), 43), rnd((L, H, D), 44)
    cr = orc.cross(q, kc, vc)
    assert cr.shape == (T, S, H, D)
    for h in range(H):
        np.testing.assert_allclose(cr[:, :, h].reshape(T * S, D),
                                   att1(q[:, :, h].reshape(T * S, D), kc[:, h], vc[:, h]), atol=1e-14)


def test_attention_rows_matches_full():
    T, S, H, D, L = 3, 6, 2, 8, 5
    q, k, v = rnd((T, S, H, D), 50), rnd((T, S, H, D), 51), rnd((T, S, H, D), 52)
    kc, vc = rnd((L, H, D), 53), rnd((L, H, D), 54)
    rows = np.array([[0, 0, 0], [2, 5, 1], [1, 3, 0]])
    full = [orc.spatial(q, k, v), orc.temporal(q, k, v), orc.cross(q, kc, vc)]
    for kind in range(3):
        kk, vv = (kc, vc) if kind == 2 else (k, v)
        got = orc.attention_rows(kind, q, kk, vv, rows)
        for i, (t, s, h) in enumerate(rows):
            np.testing.assert_allclose(got[i], full[kind][t, s, h], atol=1e-15)


def test_threads_do_not_change_result():
    q, k, v = rnd((2, 9, 3, 8), 60), rnd((2, 9, 3, 8), 61), rnd((2, 9, 3, 8), 62)
    a, used = orc.attention(q, k, v, n_threads=1, return_threads=True)
    assert used == 1
    b = orc.attention(q, k, v, n_threads=4)
    assert np.array_equal(a, b)


def test_bf16_widening_is_exact():
    x = torch.randn(64, generator=torch.Generator().manual_seed(1)).to(torch.bfloat16)
    w = orc.to_f64(x)
    assert w.dtype == np.float64
    assert np.array_equal(w.astype(np.float32), x.float().numpy())


def test_video_oracle_reuses_last_computed_output():
    calls = []
    vo = orc.VideoOracle((2, 4, 6), lo=2, hi=8)
    outs = []
    for step in range(10):
        def fn(step=step):
            calls.append(step)
            g = np.random.default_rng(step)
            return (g.standard_normal((2, 3, 1, 4)),) * 3
        dec, out = vo.step(0, orc.TEMPORAL, step, fn)
        outs.append(out)
    assert calls == [0, 1, 2, 6, 9]            # tiny_temporal row of the golden table
    assert outs[3] is outs[2] and outs[5] is outs[2] and outs[8] is outs[6]
    assert vo.computes == 5
