"""The module entry point that allocates nothing (scratch inside the library) against the entry point that takes
the caller's scratch: same kernels, so the outputs must agree bit for bit, on calls that follow each other and
shrink, and the built-in scratch must refuse shapes it cannot hold."""
import ctypes
import math

import numpy as np
import pytest
import torch

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


def weights(pab, C, heads, seed, cross):
    D = C // heads
    if cross:
        w = dict(w_qkv=bf16_randn((C, C), seed, 1.0 / math.sqrt(C)), b_qkv=bf16_randn((C,), seed + 1, 0.1),
                 w_kv=bf16_randn((2 * C, C), seed + 2, 1.0 / math.sqrt(C)), b_kv=bf16_randn((2 * C,), seed + 3, 0.1),
                 w_o=bf16_randn((C, C), seed + 4, 1.0 / math.sqrt(C)), b_o=bf16_randn((C,), seed + 5, 0.1))
    else:
        w = dict(shift=bf16_randn((C,), seed + 1, 0.3), scale=bf16_randn((C,), seed + 2, 0.3),
                 w_qkv=bf16_randn((3 * C, C), seed + 3, 1.0 / math.sqrt(C)), b_qkv=bf16_randn((3 * C,), seed + 4, 0.1),
                 gamma_q=(1.0 + 0.2 * bf16_randn((D,), seed + 5).float()).to(torch.bfloat16), beta_q=bf16_randn((D,), seed + 6, 0.2),
                 gamma_k=(1.0 + 0.2 * bf16_randn((D,), seed + 7).float()).to(torch.bfloat16), beta_k=bf16_randn((D,), seed + 8, 0.2),
                 w_o=bf16_randn((C, C), seed + 9, 1.0 / math.sqrt(C)), b_o=bf16_randn((C,), seed + 10, 0.1))
    return pab.module_weights(**{k: v.to(DEV) for k, v in w.items()})


# kind, T, S, L, heads, D: each call smaller than the one before it, so stale contents of the shared scratch
# (longer rows of the previous call) would show; the first is close to the limit of the built-in scratch
CALLS = [
    (0, 4, 444, 0, 16, 72),     # 1776 tokens x 1152: four planes of 4.09 MB, 16.37 of the 16.78 MB
    (1, 16, 60, 0, 16, 72),     # temporal, 960 tokens
    (2, 2, 100, 120, 4, 72),    # cross, 200 tokens against 120 text rows
    (2, 1, 33, 300, 4, 72),     # cross with more text rows than tokens: the planes are sized by L
    (0, 2, 37, 0, 4, 32),       # small, head dim 32
]


def test_static_scratch_matches_caller_scratch(pab):
    for n, (kind, T, S, L, heads, D) in enumerate(CALLS):
        print("no-alloc case", kind, T, S, L, heads, D, flush=True)
        C = heads * D
        x = bf16_randn((T, S, C), 4000 + n).to(DEV)
        text = bf16_randn((L, C), 4100 + n).to(DEV) if kind == 2 else None
        w = weights(pab, C, heads, 4200 + 20 * n, kind == 2)
        want = pab.pab_module_compute(kind, x, text, w, heads)          # caller-provided scratch (torch allocates it)
        out = torch.full_like(x, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        pab.pab_module_compute_static(kind, x, text, w, heads, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.isfinite(out.float()).all()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16)), (kind, T, S, L)


def test_static_scratch_limits(pab):
    limit = pab.pab_module_static_scratch_bytes()
    assert limit == 16 << 20
    heads, D = 16, 72
    C = heads * D
    T, S = 4, 460                               # 1840 tokens x 1152 x 2 B = 4.24 MB per plane: four planes do not fit
    assert 4 * T * S * C * 2 > limit
    x = torch.zeros((T, S, C), device=DEV, dtype=torch.bfloat16)
    w = weights(pab, C, heads, 5000, False)
    out = torch.empty_like(x)
    with pytest.raises(pab.PabError) as e:
        pab.pab_module_compute_static(0, x, None, w, heads, out)
    assert e.value.status == pab.ENOMEM and "pab_module_compute" in str(e.value)
    # the text decides the plane size when it is longer than the video
    xs = torch.zeros((1, 8, C), device=DEV, dtype=torch.bfloat16)
    with pytest.raises(pab.PabError) as e:
        pab.pab_module_compute_static(2, xs, torch.zeros((2000, C), device=DEV, dtype=torch.bfloat16),
                                      weights(pab, C, heads, 5100, True), heads, torch.empty_like(xs))
    assert e.value.status == pab.ENOMEM
    # argument errors come before any launch
    f = pab.lib.pab_module_compute_static
    assert f(0, 1, 8, 0, heads, D, xs.data_ptr(), None, ctypes.byref(w), None, None) == pab.EINVAL
    assert f(5, 1, 8, 0, heads, D, xs.data_ptr(), None, ctypes.byref(w), xs.data_ptr(), None) == pab.EINVAL
    assert f(0, 1, 8, 0, heads, D, None, None, ctypes.byref(w), xs.data_ptr(), None) == pab.EINVAL
