"""GPU parity of the attention-module kernels (paper App. B.5 / B.6), called through the C ABI,
against the fp64 module oracle on the same seeded inputs."""
import math

import numpy as np
import pytest
import torch

from oracle import pab_module_oracle as mo

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pab():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2408_12588_amd import pab as mod
    return mod


def bf16_randn(shape, seed, scale=1.0):
    g = np.random.Generator(np.random.Philox(key=seed))
    return torch.from_numpy(g.standard_normal(shape).astype(np.float32) * scale).to(torch.bfloat16)


def f64(t):
    return t.detach().cpu().double().numpy()


# Projection: bf16 operands are exact in fp64, products accumulate in fp32 (relative error of the
# sum far below 2^-9 for K <= a few thousand), the result is rounded once to bf16: half an ulp,
# 2^-9 relative.  Bound: 2^-8 |y| + 2^-8 * (typical |y|), the second term for results near zero.
LINEAR_SHAPES = [
    # M, N, K, bias
    (128, 256, 32, True),        # one tile, one K slice
    (1, 4, 32, True),            # smallest legal problem
    (300, 1152, 1152, True),     # ragged token tail, N = 4.5 feature tiles (the output projection)
    (257, 3456, 1152, True),     # the qkv projection: 13.5 feature tiles
    (1000, 520, 64, False),      # no bias, two K slices (ring not yet full), ragged N
    (2049, 260, 96, True),       # 17 token tiles: more than two per XCD, three K slices
    (64, 72, 2304, True),        # long K, narrow N
]


@pytest.mark.parametrize("M,N,K,bias", LINEAR_SHAPES)
def test_linear_matches_oracle(pab, M, N, K, bias):
    print("linear case", M, N, K, bias, flush=True)
    a = bf16_randn((M, K), 10 + M)
    w = bf16_randn((N, K), 20 + N, 1.0 / math.sqrt(K))
    b = bf16_randn((N,), 30 + K, 0.5) if bias else None
    out = pab.pab_linear(a.to(DEV), w.to(DEV), None if b is None else b.to(DEV))
    torch.cuda.synchronize()
    want = mo.linear(f64(a), f64(w), None if b is None else f64(b))
    got = f64(out)
    assert got.shape == want.shape and np.isfinite(got).all()
    err = np.abs(got - want)
    bound = 2.0 ** -8 * np.abs(want) + 2.0 ** -8 * np.abs(want).mean()
    assert (err <= bound).all(), "max excess %.3e at %s" % ((err - bound).max(), np.unravel_index((err - bound).argmax(), err.shape))


def test_linear_side_by_side_outputs(pab):
    # two projections into one buffer through the row pitch: neither may touch the other's columns
    M, K = 200, 64
    a = bf16_randn((M, K), 1).to(DEV)
    w1, w2 = bf16_randn((96, K), 2, 0.125).to(DEV), bf16_randn((160, K), 3, 0.125).to(DEV)
    buf = torch.full((M, 256), 7.0, device=DEV, dtype=torch.bfloat16)
    pab.pab_linear(a, w1, None, out=buf[:, :96])
    pab.pab_linear(a, w2, None, out=buf[:, 96:])
    torch.cuda.synchronize()
    assert torch.equal(buf[:, :96], pab.pab_linear(a, w1))
    assert torch.equal(buf[:, 96:], pab.pab_linear(a, w2))


def test_linear_argument_errors(pab):
    a = torch.zeros((8, 64), device=DEV, dtype=torch.bfloat16)
    w = torch.zeros((8, 64), device=DEV, dtype=torch.bfloat16)
    c = torch.zeros((8, 8), device=DEV, dtype=torch.bfloat16)
    f = pab.lib.pab_linear
    assert f(8, 8, 64, None, w.data_ptr(), None, c.data_ptr(), 8, None) == pab.EINVAL
    assert f(8, 8, 48, a.data_ptr(), w.data_ptr(), None, c.data_ptr(), 8, None) == pab.EINVAL      # K % 32
    assert f(8, 6, 64, a.data_ptr(), w.data_ptr(), None, c.data_ptr(), 8, None) == pab.EINVAL      # N % 4
    assert f(8, 8, 64, a.data_ptr(), w.data_ptr(), None, c.data_ptr(), 4, None) == pab.EINVAL      # ldc < N
    assert f(8, 8, 64, a.data_ptr() + 2, w.data_ptr(), None, c.data_ptr(), 8, None) == pab.EINVAL  # alignment
    assert f(0, 8, 64, a.data_ptr(), w.data_ptr(), None, c.data_ptr(), 8, None) == pab.EINVAL


# ---- the whole module -----------------------------------------------------------------------
# Bound: the attention operation is held to 1e-2 * max|V|; around it sit projections whose inputs
# and outputs are stored in bf16 (2^-9 relative each, averaging out over the K = C terms of a
# product) and whose weights have rows of about unit norm, so the module output carries an
# error of the size of the attention error and is held to the same bar, 1e-2 * max|y|
# (observed: 4-5e-3).
TOL_MODULE = 1e-2


def self_weights(C, heads, seed):
    D = C // heads
    return dict(shift=bf16_randn((C,), seed + 1, 0.3), scale=bf16_randn((C,), seed + 2, 0.3),
                w_qkv=bf16_randn((3 * C, C), seed + 3, 1.0 / math.sqrt(C)), b_qkv=bf16_randn((3 * C,), seed + 4, 0.1),
                gamma_q=(1.0 + 0.2 * bf16_randn((D,), seed + 5).float()).to(torch.bfloat16), beta_q=bf16_randn((D,), seed + 6, 0.2),
                gamma_k=(1.0 + 0.2 * bf16_randn((D,), seed + 7).float()).to(torch.bfloat16), beta_k=bf16_randn((D,), seed + 8, 0.2),
                w_o=bf16_randn((C, C), seed + 9, 1.0 / math.sqrt(C)), b_o=bf16_randn((C,), seed + 10, 0.1))


def oracle_self(kind, x, w, heads):
    return mo.self_attention_module(kind, f64(x), f64(w["shift"]), f64(w["scale"]), f64(w["w_qkv"]), f64(w["b_qkv"]),
                                    f64(w["gamma_q"]), f64(w["beta_q"]), f64(w["gamma_k"]), f64(w["beta_k"]),
                                    f64(w["w_o"]), f64(w["b_o"]), heads)


def check_module(got, want, what):
    got = f64(got)
    assert got.shape == want.shape and np.isfinite(got).all(), what
    err = np.abs(got - want).max()
    bound = TOL_MODULE * np.abs(want).max()
    assert err <= bound, "%s: max abs err %.3e > %.3e" % (what, err, bound)
    return err / np.abs(want).max()


MODULE_SHAPES = [
    # kind, T, S, heads, D
    (0, 2, 150, 4, 72),     # spatial: ragged token tail for every kernel of the chain
    (0, 3, 64, 4, 32),      # head dim 32, hidden size 128
    (1, 16, 21, 4, 72),     # temporal with rotary embedding, 16 frames
    (1, 17, 9, 8, 32),      # 17 frames (32-row temporal kernel), hidden size 256
    (1, 1, 40, 4, 72),      # one frame: attention is the identity on v, frame index 0 turns nothing
]


@pytest.mark.parametrize("kind,T,S,heads,D", MODULE_SHAPES)
def test_self_module_matches_oracle(pab, kind, T, S, heads, D):
    print("module case", kind, T, S, heads, D, flush=True)
    C = heads * D
    x = bf16_randn((T, S, C), 500 + T + S)
    w = self_weights(C, heads, 600 + 10 * kind)
    wd = pab.module_weights(**{k: v.to(DEV) for k, v in w.items()})
    out = pab.pab_module_compute(kind, x.to(DEV), None, wd, heads)
    torch.cuda.synchronize()
    rel = check_module(out, oracle_self(kind, x, w, heads), "self module kind %d" % kind)
    print("   relative max error %.2e" % rel, flush=True)


@pytest.mark.parametrize("T,S,L,heads,D", [(2, 100, 120, 4, 72), (1, 33, 300, 4, 72), (2, 50, 16, 4, 32)])
def test_cross_module_matches_oracle(pab, T, S, L, heads, D):
    print("cross module case", T, S, L, heads, D, flush=True)
    C = heads * D
    x, text = bf16_randn((T, S, C), 700 + S), bf16_randn((L, C), 701 + L)
    w = dict(w_qkv=bf16_randn((C, C), 710, 1.0 / math.sqrt(C)), b_qkv=bf16_randn((C,), 711, 0.1),
             w_kv=bf16_randn((2 * C, C), 712, 1.0 / math.sqrt(C)), b_kv=bf16_randn((2 * C,), 713, 0.1),
             w_o=bf16_randn((C, C), 714, 1.0 / math.sqrt(C)), b_o=bf16_randn((C,), 715, 0.1))
    wd = pab.module_weights(**{k: v.to(DEV) for k, v in w.items()})
    out = pab.pab_module_compute(2, x.to(DEV), text.to(DEV), wd, heads)
    torch.cuda.synchronize()
    want = mo.cross_attention_module(f64(x), f64(text), f64(w["w_qkv"]), f64(w["b_qkv"]), f64(w["w_kv"]), f64(w["b_kv"]),
                                     f64(w["w_o"]), f64(w["b_o"]), heads)
    check_module(out, want, "cross module")


def test_module_broadcast_schedule_and_reuse(pab):
    """Module-level PAB on a small video: computed steps match the oracle run on that step's
    input, reused steps launch nothing and hand back the very bytes of the last computed step."""
    from oracle import pab_oracle as orc
    T, S, heads, D, n_steps, lo, hi = 4, 40, 4, 32, 8, 1, 6
    C = heads * D
    cfg = pab.make_config(2, T, S, 8, heads, D, pab.BF16, n_steps, (2, 3, 0), lo, hi)
    ctx = pab.PabContext(cfg, DEV)
    ctx.workspace.fill_(0xFF)
    scratch = pab.module_scratch(T, S, 8, heads, D, DEV)
    ws = [[self_weights(C, heads, 900 + 37 * (2 * b + k)) for k in range(2)] for b in range(2)]
    wds = [[pab.module_weights(**{n: v.to(DEV) for n, v in w.items()}) for w in row] for row in ws]
    last = {}
    launches = 0
    for step in range(n_steps):
        for block in range(2):
            for kind in range(2):
                x = bf16_randn((T, S, C), 10000 + 100 * step + 10 * block + kind)
                want_dec = orc.schedule(step, lo, hi, cfg.interval[kind])
                if want_dec == 0:
                    dec, ptr = ctx.pab_module_attention(block, kind, step, x.to(DEV), None, wds[block][kind], scratch)
                    launches += 1
                else:   # nothing may be read on a reused step: hand in nothing at all
                    dec, ptr = ctx.pab_module_attention(block, kind, step, None, None, None, None)
                torch.cuda.synchronize()
                assert dec == want_dec, (step, block, kind)
                assert ptr == ctx.pab_slot_ptr(block, kind)
                got = ctx.slot_tensor(block, kind).reshape(T, S, C)
                if dec == 0:
                    check_module(got, oracle_self(kind, x, ws[block][kind], heads), "video step %d" % step)
                    last[(block, kind)] = got.clone()
                else:
                    assert torch.equal(got, last[(block, kind)]), (step, block, kind)
    assert ctx.pab_launch_count() == launches
    ctx.pab_destroy()


def test_module_argument_errors(pab):
    T, S, heads, D = 2, 16, 4, 32
    C = heads * D
    x = torch.zeros((T, S, C), device=DEV, dtype=torch.bfloat16)
    w = self_weights(C, heads, 1)
    wd = pab.module_weights(**{k: v.to(DEV) for k, v in w.items()})
    scratch = pab.module_scratch(T, S, 0, heads, D, DEV)
    out = torch.empty_like(x)
    import ctypes
    f = pab.lib.pab_module_compute
    ok = (0, T, S, 0, heads, D, x.data_ptr(), None, ctypes.byref(wd), scratch.data_ptr(), scratch.numel(), out.data_ptr(), None)
    assert f(*ok) == pab.OK
    bad = list(ok); bad[10] = scratch.numel() // 2
    assert f(*bad) == pab.ENOMEM
    bad = list(ok); bad[6] = None
    assert f(*bad) == pab.EINVAL
    bad = list(ok); bad[0] = 2            # cross without text
    assert f(*bad) == pab.EINVAL
    bad = list(ok); bad[4], bad[5] = 3, 72   # hidden size 216: not a multiple of 32
    assert f(*bad) == pab.EINVAL
    wd2 = pab.module_weights(**{k: v.to(DEV) for k, v in w.items() if k != "gamma_k"})
    bad = list(ok); bad[8] = ctypes.byref(wd2)
    assert f(*bad) == pab.EINVAL
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["opensora_480p", "osp_512_long"])
def test_module_full_size_sampled(pab, name):
    """The benchmark's shapes and launch configuration.  The modules are independent per frame
    (spatial), per position (temporal) and per token (cross), so the oracle can be run on a few
    frames / positions / tokens of the full-size input and compared with those outputs."""
    from paper_2408_12588_amd import workloads as W
    wl = W.BY_NAME[name]
    T, S, H = wl.T, wl.S, wl.heads
    text = W.make_text(wl)
    scratch = pab.module_scratch(T, S, wl.L, H, wl.head_dim, DEV)
    for kind in range(3):
        print("full-size module", name, W.KIND_NAMES[kind], flush=True)
        x = W.make_module_input(wl, 1, kind, 2)
        w = W.make_module_weights(wl, 1, kind)
        wd = pab.module_weights(**{n: t.to(DEV) for n, t in w.items()})
        out = pab.pab_module_compute(kind, x.to(DEV), text.to(DEV) if kind == 2 else None, wd, H, scratch=scratch)
        torch.cuda.synchronize()
        out = out.cpu()
        assert torch.isfinite(out.float()).all()
        if kind == 0:
            for t in (0, T - 1):
                check_module(out[t:t + 1], oracle_self(0, x[t:t + 1], w, H), "%s spatial frame %d" % (name, t))
        elif kind == 1:
            for s in (0, S // 3, S - 1):
                check_module(out[:, s:s + 1], oracle_self(1, x[:, s:s + 1], w, H), "%s temporal position %d" % (name, s))
        else:
            for t, s0 in ((0, 0), (T - 1, S - 8), (T // 2, S // 2)):
                want = mo.cross_attention_module(f64(x[t:t + 1, s0:s0 + 8]), f64(text), f64(w["w_qkv"]), f64(w["b_qkv"]),
                                                 f64(w["w_kv"]), f64(w["b_kv"]), f64(w["w_o"]), f64(w["b_o"]), H)
                check_module(out[t:t + 1, s0:s0 + 8], want, "%s cross tokens (%d, %d..)" % (name, t, s0))


# ---- MLP module and MLP broadcast --------------------------------------------------------------
def mlp_weights_cpu(C, Fw, seed):
    return dict(shift=bf16_randn((C,), seed + 1, 0.3), scale=bf16_randn((C,), seed + 2, 0.3),
                w1=bf16_randn((Fw, C), seed + 3, 1.0 / math.sqrt(C)), b1=bf16_randn((Fw,), seed + 4, 0.1),
                w2=bf16_randn((C, Fw), seed + 5, 1.0 / math.sqrt(Fw)), b2=bf16_randn((C,), seed + 6, 0.1))


def oracle_mlp(x, w):
    return mo.mlp_module(f64(x), f64(w["shift"]), f64(w["scale"]), f64(w["w1"]), f64(w["b1"]), f64(w["w2"]), f64(w["b2"]))


@pytest.mark.parametrize("n_tok,C,Fw", [(300, 288, 1152), (70, 128, 512), (1, 32, 32), (515, 1152, 4608)])
def test_mlp_module_matches_oracle(pab, n_tok, C, Fw):
    print("mlp case", n_tok, C, Fw, flush=True)
    x = bf16_randn((n_tok, C), 40 + n_tok)
    w = mlp_weights_cpu(C, Fw, 50 + C)
    wd = pab.mlp_weights(**{k: v.to(DEV) for k, v in w.items()})
    out = pab.pab_mlp_compute(x.to(DEV), wd, Fw)
    torch.cuda.synchronize()
    check_module(out, oracle_mlp(x, w), "mlp module")


def test_mlp_full_size_sampled(pab):
    # config 2: 25440 tokens, hidden 1152, inner 4608; tokens are independent, so the oracle takes a sample of them
    n_tok, C, Fw = 25440, 1152, 4608
    x = bf16_randn((n_tok, C), 4242)
    w = mlp_weights_cpu(C, Fw, 4300)
    wd = pab.mlp_weights(**{k: v.to(DEV) for k, v in w.items()})
    out = pab.pab_mlp_compute(x.to(DEV), wd, Fw).cpu()
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    rows = np.array([0, 1, 127, 128, 12719, 25312, 25439] + list(np.random.default_rng(1).integers(0, n_tok, 40)))
    check_module(out[rows], oracle_mlp(x[rows], w), "mlp sampled tokens")


def test_mlp_broadcast_video(pab):
    """Small run with MLP broadcasting: blocks 0-1 of 3 take part, starts at steps 2 and 5, range 3."""
    from oracle import pab_oracle as orc
    n_blocks, n_steps, n_tok, C, Fw = 3, 9, 100, 128, 512
    starts, rng_n, blo, bhi = [2, 5], 3, 0, 1
    ctx = pab.MlpContext(n_blocks, n_steps, n_tok, C, Fw, starts, rng_n, blo, bhi, DEV)
    ctx.workspace.fill_(0xFF)
    scratch = pab.mlp_scratch(n_tok, C, Fw, DEV)
    ws = [mlp_weights_cpu(C, Fw, 7000 + 100 * b) for b in range(n_blocks)]
    wds = [pab.mlp_weights(**{k: v.to(DEV) for k, v in w.items()}) for w in ws]
    y = torch.empty((n_tok, C), device=DEV, dtype=torch.bfloat16)
    last, launches = {}, 0
    for step in range(n_steps):
        for block in range(n_blocks):
            x = bf16_randn((n_tok, C), 8000 + 10 * step + block)
            want_dec, want_src = orc.mlp_schedule(step, block, starts, rng_n, blo, bhi)
            if want_dec == 0:
                dec, ptr = ctx.pab_mlp(block, step, x.to(DEV), wds[block], scratch, y=y if block > bhi else None)
                launches += 1
            else:
                dec, ptr = ctx.pab_mlp(block, step, None, None, None)
            torch.cuda.synchronize()
            assert dec == want_dec, (step, block)
            got = ctx.slot_tensor(block) if block <= bhi else y
            assert ptr == got.data_ptr()
            if dec == 0:
                check_module(got, oracle_mlp(x, ws[block]), "mlp video step %d block %d" % (step, block))
                last[block] = (step, got.clone())
            else:
                assert last[block][0] == want_src and torch.equal(got, last[block][1]), (step, block)
    assert ctx.pab_mlp_launch_count() == launches == n_steps * n_blocks - 2 * 2 * 2
    ctx.pab_mlp_destroy()
