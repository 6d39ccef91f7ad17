"""The synthetic workloads: shapes of the five configurations and determinism of
the seeded generators."""
import numpy as np
import torch

from paper_2408_12588_amd import workloads as W


def test_shapes_and_counts():
    assert [w.name for w in W.CONFIGS] == ["tiny", "opensora_480p", "latte_512", "osp_512_long", "stress_720p"]
    assert W.OPENSORA_480P.S == 1590 and W.STRESS_720P.S == 3600 and W.OSP_512_LONG.T == 17
    assert len(W.OPENSORA_480P.calls_per_step()) == 84
    assert len(W.LATTE_512.calls_per_step()) == 28
    assert all(k != W.CROSS for _, k in W.LATTE_512.calls_per_step())
    assert W.LATTE_512.kinds_of_block(0) == (W.SPATIAL,) and W.LATTE_512.kinds_of_block(1) == (W.TEMPORAL,)
    # 4 B H Sq Sk D
    assert abs(W.OPENSORA_480P.flops(W.SPATIAL) / 1e12 - 0.1864) < 1e-3
    assert abs(W.OPENSORA_480P.bytes(W.TEMPORAL) / 1e6 - 234.4) < 0.1
    assert abs(W.OPENSORA_480P.bytes(W.CROSS) / 1e6 - 117.8) < 0.1


def test_generators_are_deterministic_and_distinct():
    wl = W.TINY
    a = W.make_qkv(wl, 1, W.SPATIAL, 3)
    b = W.make_qkv(wl, 1, W.SPATIAL, 3)
    c = W.make_qkv(wl, 1, W.SPATIAL, 4)
    for x, y in zip(a, b):
        assert torch.equal(x, y) and x.dtype == torch.float32
    assert not torch.equal(a[0], c[0]) and not torch.equal(a[0], a[1])
    q, k, v = W.make_qkv(wl, 0, W.CROSS, 0)
    assert q.shape == (4, 64, 4, 32) and k.shape == (16, 4, 32) and v.shape == k.shape
    assert abs(float(q.mean())) < 0.05 and abs(float(q.std()) - 1) < 0.05


def test_peaked_rows():
    wl = W.Workload("p", 1, 2, 50, 4, 2, 8, "bf16", 1, (1, 1, 1), 0, 0, peaked_frac=0.05, seed=5)
    rows = W.peaked_rows(wl)
    assert len(rows) == 5 and len(set(rows.tolist())) == 5
    plain = W.Workload("p", 1, 2, 50, 4, 2, 8, "bf16", 1, (1, 1, 1), 0, 0, seed=5)
    q = W.make_qkv(wl, 0, 0, 0)[0].float().reshape(100, -1)
    q0 = W.make_qkv(plain, 0, 0, 0)[0].float().reshape(100, -1)
    ratio = (q.abs().sum(1) / q0.abs().sum(1)).numpy()
    assert np.allclose(ratio[rows], 8.0, rtol=2e-2)
    mask = np.ones(100, bool); mask[rows] = False
    assert np.allclose(ratio[mask], 1.0)
    assert q.dtype == torch.float32 and W.make_qkv(wl, 0, 0, 0)[0].dtype == torch.bfloat16
