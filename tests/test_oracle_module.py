"""Pins for the fp64 oracle of the attention module (paper App. B.5 / B.6): each part against a
library routine, closed forms and invariants; the composition against special cases that reduce
to parts already pinned, and against an assembly of library routines."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import pab_module_oracle as mo

RNG = np.random.default_rng(20240812)


def t64(a):
    return torch.from_numpy(np.ascontiguousarray(a)).double()


# ---- layernorm1 -----------------------------------------------------------------------------
def test_layer_norm_matches_library_and_moments():
    x = RNG.standard_normal((5, 7, 48)) * 3.0 + 1.5
    got = mo.layer_norm(x)
    want = F.layer_norm(t64(x), (48,), eps=mo.EPS).numpy()
    assert np.abs(got - want).max() < 1e-12
    assert np.abs(got.mean(-1)).max() < 1e-12
    var = x.var(-1)   # biased
    assert np.allclose((got ** 2).mean(-1), var / (var + mo.EPS), rtol=0, atol=1e-12)


def test_layer_norm_closed_forms():
    # a row of equal values has nothing to normalise
    assert np.all(mo.layer_norm(np.full((2, 6), 3.25)) == 0.0)
    # two values a, b: mean (a+b)/2, deviation +-(a-b)/2 -> +-1 up to eps
    got = mo.layer_norm(np.array([[1.0, 5.0]]))
    assert np.allclose(got, [[-2.0 / math.sqrt(4.0 + mo.EPS), 2.0 / math.sqrt(4.0 + mo.EPS)]], atol=1e-15)
    # adding a constant changes nothing; a positive factor changes only the eps term
    x = RNG.standard_normal((3, 20))
    assert np.abs(mo.layer_norm(x + 7.0) - mo.layer_norm(x)).max() < 1e-12
    assert np.abs(mo.layer_norm(1000.0 * x) - mo.layer_norm(x)).max() < 1e-5
    # the unbiased variance would be off by a factor n/(n-1) = 2 for two values: detectably different
    assert abs(got[0, 1] - 2.0 / math.sqrt(8.0)) > 0.2


def test_modulate():
    x = np.array([[1.0, -2.0, 0.5]])
    assert np.array_equal(mo.modulate(x, np.array([0.5, 0.5, 0.5]), np.array([1.0, 0.0, -1.0])), [[2.5, -1.5, 0.5]])
    assert np.array_equal(mo.modulate(x, np.zeros(3), np.zeros(3)), x)
    # scale multiplies before the shift is added (the other order would give (x + shift)(1 + scale))
    assert mo.modulate(np.array([2.0]), np.array([3.0]), np.array([1.0]))[0] == 7.0


# ---- projections ----------------------------------------------------------------------------
def test_linear_matches_library_and_hand_example():
    x = RNG.standard_normal((4, 3, 10))
    w = RNG.standard_normal((6, 10))
    b = RNG.standard_normal(6)
    assert np.abs(mo.linear(x, w, b) - F.linear(t64(x), t64(w), t64(b)).numpy()).max() < 1e-12
    assert np.abs(mo.linear(x, w, None) - F.linear(t64(x), t64(w)).numpy()).max() < 1e-12
    # W is [out, in]: row o of W gives output o
    w2 = np.array([[1.0, 2.0], [0.0, -1.0], [3.0, 0.0]])
    assert np.array_equal(mo.linear(np.array([1.0, 10.0]), w2, np.array([0.5, 0.0, 0.0])), [21.5, -10.0, 3.0])


# ---- layernorm2 -----------------------------------------------------------------------------
def test_head_layer_norm_matches_library():
    x = RNG.standard_normal((3, 5, 4, 24))
    g, b = RNG.standard_normal(24), RNG.standard_normal(24)
    want = F.layer_norm(t64(x), (24,), t64(g), t64(b), eps=mo.EPS).numpy()
    assert np.abs(mo.head_layer_norm(x, g, b) - want).max() < 1e-12
    # zero input: the normalised part vanishes, the learned shift remains
    assert np.array_equal(mo.head_layer_norm(np.zeros((2, 24)), g, b), np.broadcast_to(b, (2, 24)))


# ---- pos emb --------------------------------------------------------------------------------
def test_rotary_hand_example_and_identity():
    # D = 4: pair 0 turns by pos * 1, pair 1 by pos * 10000^(-1/2) = pos / 100
    x = np.zeros((1, 3, 1, 4))
    x[0, :, 0] = [[1.0, 0.0, 0.0, 2.0]] * 3
    got = mo.rotary(x, np.array([0, 1, 2]))
    assert np.array_equal(got[0, 0, 0], [1.0, 0.0, 0.0, 2.0])            # position 0: nothing turns
    for p in (1, 2):
        want = [math.cos(p), math.sin(p), -2.0 * math.sin(p / 100.0), 2.0 * math.cos(p / 100.0)]
        assert np.allclose(got[0, p, 0], want, atol=1e-15)


def test_rotary_is_a_rotation_and_relative():
    D, P = 24, 9
    q = RNG.standard_normal((2, P, 3, D))
    k = RNG.standard_normal((2, P, 3, D))
    pos = np.arange(P)
    rq, rk = mo.rotary(q, pos), mo.rotary(k, pos)
    # lengths of every pair are kept
    assert np.allclose(rq[..., 0::2] ** 2 + rq[..., 1::2] ** 2, q[..., 0::2] ** 2 + q[..., 1::2] ** 2, atol=1e-12)
    # scores depend on the distance of the positions only: shifting all positions changes nothing
    s0 = np.einsum("bphd,brhd->bhpr", rq, rk)
    s5 = np.einsum("bphd,brhd->bhpr", mo.rotary(q, pos + 5), mo.rotary(k, pos + 5))
    assert np.abs(s0 - s5).max() < 1e-10
    # ... and they do depend on it
    assert np.abs(s0 - np.einsum("bphd,brhd->bhpr", q, k)).max() > 0.1
    # complex-number form of the same definition: (x_2i + i x_2i+1) * exp(i pos theta_i)
    theta = 10000.0 ** (-np.arange(0, D, 2) / D)
    z = (q[..., 0::2] + 1j * q[..., 1::2]) * np.exp(1j * pos[None, :, None, None] * theta)
    assert np.abs(rq[..., 0::2] - z.real).max() < 1e-12 and np.abs(rq[..., 1::2] - z.imag).max() < 1e-12


# ---- composition ----------------------------------------------------------------------------
def make_self_weights(C, heads, rng, zero_qk=False):
    D = C // heads
    w_qkv = rng.standard_normal((3 * C, C)) / math.sqrt(C)
    b_qkv = 0.1 * rng.standard_normal(3 * C)
    if zero_qk:
        w_qkv[: 2 * C] = 0.0
        b_qkv[: 2 * C] = 0.0
    return dict(shift=0.3 * rng.standard_normal(C), scale=0.3 * rng.standard_normal(C), w_qkv=w_qkv, b_qkv=b_qkv,
                gq=1.0 + 0.2 * rng.standard_normal(D), bq=0.2 * rng.standard_normal(D),
                gk=1.0 + 0.2 * rng.standard_normal(D), bk=0.2 * rng.standard_normal(D),
                w_o=rng.standard_normal((C, C)) / math.sqrt(C), b_o=0.1 * rng.standard_normal(C))


def run_self(kind, x, w, heads):
    return mo.self_attention_module(kind, x, w["shift"], w["scale"], w["w_qkv"], w["b_qkv"], w["gq"], w["bq"],
                                    w["gk"], w["bk"], w["w_o"], w["b_o"], heads)


@pytest.mark.parametrize("kind", [0, 1])
def test_zero_queries_and_keys_average_the_values(kind):
    # q = k = learned shift only -> all scores equal -> the attention output is the mean of the
    # values over the sequence axis of that kind; what is left are parts pinned above
    T, S, heads, D = 3, 5, 2, 8
    C = heads * D
    rng = np.random.default_rng(11 + kind)
    x = rng.standard_normal((T, S, C))
    w = make_self_weights(C, heads, rng, zero_qk=True)
    if kind == 1:   # a constant q = k would still be turned by the frame index: make them vanish
        w["bq"][:] = 0.0
        w["bk"][:] = 0.0
    h = mo.modulate(mo.layer_norm(x), w["shift"], w["scale"])
    v = mo.linear(h, w["w_qkv"][2 * C:], w["b_qkv"][2 * C:])
    mean_v = v.mean(axis=1 if kind == 0 else 0, keepdims=True) * np.ones_like(v)
    want = mo.linear(mean_v, w["w_o"], w["b_o"])
    assert np.abs(run_self(kind, x, w, heads) - want).max() < 1e-10
    # the two kinds average over different axes: the test can tell them apart
    other = v.mean(axis=0 if kind == 0 else 1, keepdims=True) * np.ones_like(v)
    assert np.abs(mean_v - other).max() > 0.05


def test_one_frame_temporal_is_projection_of_values():
    # one key per query: softmax weight 1, whatever q and k (and their rotation) are
    S, heads, D = 6, 3, 8
    C = heads * D
    rng = np.random.default_rng(5)
    x = rng.standard_normal((1, S, C))
    w = make_self_weights(C, heads, rng)
    h = mo.modulate(mo.layer_norm(x), w["shift"], w["scale"])
    want = mo.linear(mo.linear(h, w["w_qkv"][2 * C:], w["b_qkv"][2 * C:]), w["w_o"], w["b_o"])
    assert np.abs(run_self(1, x, w, heads) - want).max() < 1e-10


def library_self_module(kind, x, w, heads):
    """The same workflow assembled from library routines (fp64 torch); rotary from its
    complex-number form."""
    T, S, C = x.shape
    D = C // heads
    h = F.layer_norm(t64(x), (C,), eps=mo.EPS) * (1.0 + t64(w["scale"])) + t64(w["shift"])
    qkv = F.linear(h, t64(w["w_qkv"]), t64(w["b_qkv"])).reshape(T, S, 3, heads, D)
    q = F.layer_norm(qkv[:, :, 0], (D,), t64(w["gq"]), t64(w["bq"]), eps=mo.EPS)
    k = F.layer_norm(qkv[:, :, 1], (D,), t64(w["gk"]), t64(w["bk"]), eps=mo.EPS)
    v = qkv[:, :, 2]
    if kind == 1:
        theta = 10000.0 ** (-torch.arange(0, D, 2, dtype=torch.float64) / D)
        rot = torch.polar(torch.ones(T, D // 2, dtype=torch.float64), torch.arange(T, dtype=torch.float64)[:, None] * theta)

        def turn(a):   # [T, S, H, D]
            z = torch.view_as_complex(a.reshape(T, S, heads, D // 2, 2).contiguous()) * rot[:, None, None, :]
            return torch.view_as_real(z).reshape(T, S, heads, D)
        q, k = turn(q), turn(k)
        q, k, v = (a.permute(1, 2, 0, 3) for a in (q, k, v))        # [S, H, T, D]
        o = F.scaled_dot_product_attention(q, k, v).permute(2, 0, 1, 3)
    else:
        q, k, v = (a.permute(0, 2, 1, 3) for a in (q, k, v))        # [T, H, S, D]
        o = F.scaled_dot_product_attention(q, k, v).permute(0, 2, 1, 3)
    return F.linear(o.reshape(T, S, C), t64(w["w_o"]), t64(w["b_o"])).numpy()


@pytest.mark.parametrize("kind", [0, 1])
def test_self_module_against_library_assembly(kind):
    T, S, heads, D = 5, 7, 3, 8
    C = heads * D
    rng = np.random.default_rng(100 + kind)
    x = rng.standard_normal((T, S, C))
    w = make_self_weights(C, heads, rng)
    assert np.abs(run_self(kind, x, w, heads) - library_self_module(kind, x, w, heads)).max() < 1e-10


def test_cross_module_against_library_and_special_case():
    T, S, L, heads, D = 2, 5, 4, 2, 8
    C = heads * D
    rng = np.random.default_rng(77)
    x, y = rng.standard_normal((T, S, C)), rng.standard_normal((L, C))
    w_q, b_q = rng.standard_normal((C, C)) / 4, 0.1 * rng.standard_normal(C)
    w_kv, b_kv = rng.standard_normal((2 * C, C)) / 4, 0.1 * rng.standard_normal(2 * C)
    w_o, b_o = rng.standard_normal((C, C)) / 4, 0.1 * rng.standard_normal(C)
    got = mo.cross_attention_module(x, y, w_q, b_q, w_kv, b_kv, w_o, b_o, heads)
    q = F.linear(t64(x), t64(w_q), t64(b_q)).reshape(1, T * S, heads, D).permute(0, 2, 1, 3)
    kv = F.linear(t64(y), t64(w_kv), t64(b_kv)).reshape(L, 2, heads, D)
    k, v = kv[:, 0].permute(1, 0, 2)[None], kv[:, 1].permute(1, 0, 2)[None]
    o = F.scaled_dot_product_attention(q, k, v).permute(0, 2, 1, 3).reshape(T, S, C)
    assert np.abs(got - F.linear(o, t64(w_o), t64(b_o)).numpy()).max() < 1e-10
    # no query signal: every token gets the mean of the text values
    got0 = mo.cross_attention_module(x, y, np.zeros((C, C)), np.zeros(C), w_kv, b_kv, w_o, b_o, heads)
    v_all = mo.linear(y, w_kv[C:], b_kv[C:])
    want0 = mo.linear(np.broadcast_to(v_all.mean(0), (T, S, C)), w_o, b_o)
    assert np.abs(got0 - want0).max() < 1e-10


# ---- MLP module (Sec. 2.3 last sentence; App. A.2.2 MLP table) --------------------------------
def test_gelu_tanh_matches_library_and_closed_forms():
    x = np.linspace(-6.0, 6.0, 241)
    assert np.abs(mo.gelu_tanh(x) - F.gelu(t64(x), approximate="tanh").numpy()).max() < 1e-14
    assert mo.gelu_tanh(np.array([0.0]))[0] == 0.0
    assert np.abs(mo.gelu_tanh(x) - mo.gelu_tanh(-x) - x).max() < 1e-12      # the even part cancels: g(x) - g(-x) = x
    assert abs(mo.gelu_tanh(np.array([10.0]))[0] - 10.0) < 1e-12
    assert abs(mo.gelu_tanh(np.array([1.0]))[0] - 0.5 * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * 1.044715))) < 1e-15
    # the exact (erf) form differs visibly: the reading is the tanh form
    assert abs(mo.gelu_tanh(np.array([2.0]))[0] - F.gelu(torch.tensor([2.0], dtype=torch.float64)).item()) > 5e-5


def test_mlp_module_against_library_and_special_case():
    C, Fw = 24, 96
    rng = np.random.default_rng(3)
    x = rng.standard_normal((3, 5, C))
    shift, scale = 0.3 * rng.standard_normal(C), 0.3 * rng.standard_normal(C)
    w1, b1 = rng.standard_normal((Fw, C)) / math.sqrt(C), 0.1 * rng.standard_normal(Fw)
    w2, b2 = rng.standard_normal((C, Fw)) / math.sqrt(Fw), 0.1 * rng.standard_normal(C)
    got = mo.mlp_module(x, shift, scale, w1, b1, w2, b2)
    h = F.layer_norm(t64(x), (C,), eps=mo.EPS) * (1.0 + t64(scale)) + t64(shift)
    want = F.linear(F.gelu(F.linear(h, t64(w1), t64(b1)), approximate="tanh"), t64(w2), t64(b2)).numpy()
    assert np.abs(got - want).max() < 1e-12
    # no signal through the first projection: every token gets W2 gelu(b1) + b2
    got0 = mo.mlp_module(x, shift, scale, np.zeros_like(w1), b1, w2, b2)
    assert np.abs(got0 - (w2 @ mo.gelu_tanh(b1) + b2)).max() < 1e-12


def test_mlp_schedule_golden_and_invariants():
    from oracle import pab_oracle as orc
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "timestep_windows.txt")) as f:
        for line in f:
            if line.startswith("mlp "):
                head, steps, pattern = line[4:].split("|")
                h = head.split()
                rows.append((h[0], int(h[1]), int(h[2]), int(h[3]), int(h[4]), int(h[5]), int(h[6]),
                             [int(v) for v in h[7:]], [int(v) for v in steps.split()], pattern.strip()))
    assert len(rows) == 2
    for name, first, stride, n_steps, n, blo, bhi, t_starts, want_steps, pattern in rows:
        ts = [first - s * stride for s in range(n_steps)]
        starts = orc.start_steps_from_timesteps(ts, t_starts)
        assert starts == want_steps, name
        assert len(pattern) == n_steps, name
        got = "".join("CR"[orc.mlp_schedule(s, blo, starts, n, blo, bhi)[0]] for s in range(n_steps))
        assert got == pattern, name
        assert all(orc.mlp_schedule(s, bhi + 1, starts, n, blo, bhi) == (0, s) for s in range(n_steps)), name
        for s in range(n_steps):
            dec, src = orc.mlp_schedule(s, bhi, starts, n, blo, bhi)
            if dec == 1:   # the source is a listed start, computed itself, at most n-1 steps back
                assert src in starts and 0 < s - src <= n - 1
                assert orc.mlp_schedule(src, bhi, starts, n, blo, bhi) == (0, src)
    # range 1 never reuses; range 3 reuses two steps; text construction for a single start
    for n in (1, 2, 3, 5):
        row = "".join("CR"[orc.mlp_schedule(s, 0, [4], n, 0, 0)[0]] for s in range(12))
        assert row == "CCCCC" + "R" * (n - 1) + "C" * (12 - 5 - (n - 1))
    assert orc.start_steps_from_timesteps([900, 800, 700], [950, 800, 750, 10]) == [0, 1, 2, None]
