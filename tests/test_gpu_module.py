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
