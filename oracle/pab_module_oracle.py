"""fp64 oracle of the attention MODULE whose output PAB broadcasts.  TEST INFRASTRUCTURE ONLY.

The paper broadcasts the output of the whole attention module, so that a reused step skips
everything inside it (the workflow of App. B.6: project the hidden states to queries, keys and
values, normalise queries and keys and apply the position embedding, run the attention operation,
project its result); App. B.5 lists the parts it timed: layernorm1, mask, modulate,
qkv proj, layernorm2, pos emb (temporal only), attn, o proj, reshape (self attention) and
qkv proj, attn, o proj, reshape (cross attention).  The paper names these parts and gives no
formulas; each function below states the reading it takes.  Everything is written as the plain
definition in NumPy fp64, one step per part, in the order of the workflow.  Only tests, smoke()
and bench.py's cpu_baseline leg may import this file; it shares nothing with the HIP path.

parity unpinned: which normalisation "layernorm2" is, the rotary pairing and base of "pos emb",
the absence of a norm in the cross module and the activation of the MLP are readings; the
arithmetic of every part is pinned by tests/test_oracle_module.py.
"""
from __future__ import annotations

import numpy as np

from . import pab_oracle as _attn

EPS = 1e-6


def layer_norm(x: np.ndarray, eps: float = EPS) -> np.ndarray:
    """"layernorm1": over the last axis, no learned scale or shift (they come from `modulate`),
    biased variance, eps inside the square root."""
    x = np.asarray(x, dtype=np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def modulate(x: np.ndarray, shift: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """"modulate": x * (1 + scale) + shift with one shift / scale vector of the hidden size for
    the whole video (adaptive layer norm conditioning on the diffusion step)."""
    return np.asarray(x, np.float64) * (1.0 + np.asarray(scale, np.float64)) + np.asarray(shift, np.float64)


def linear(x: np.ndarray, w: np.ndarray, b: np.ndarray | None) -> np.ndarray:
    """"qkv proj" / "o proj": y = x W^T + b with W stored [out, in]."""
    y = np.asarray(x, np.float64) @ np.asarray(w, np.float64).T
    return y if b is None else y + np.asarray(b, np.float64)


def head_layer_norm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float = EPS) -> np.ndarray:
    """"layernorm2": LayerNorm over the head dimension (last axis) of q or k with a learned
    scale and shift of that size."""
    return layer_norm(x, eps) * np.asarray(gamma, np.float64) + np.asarray(beta, np.float64)


def rotary(x: np.ndarray, positions: np.ndarray, base: float = 10000.0) -> np.ndarray:
    """"pos emb" (temporal attention only): rotary embedding.  x: [..., P, H, D] with the position
    axis third from last; positions: [P].  Feature pair (2i, 2i+1) is rotated by the angle
    position * base^(-2i/D)."""
    x = np.asarray(x, np.float64)
    D = x.shape[-1]
    assert D % 2 == 0
    theta = base ** (-np.arange(0, D, 2, dtype=np.float64) / D)          # [D/2]
    ang = np.asarray(positions, np.float64)[:, None] * theta[None, :]    # [P, D/2]
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]           # [P, 1, D/2]
    even, odd = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = even * cos - odd * sin
    out[..., 1::2] = even * sin + odd * cos
    return out


def self_attention_module(kind: int, x, shift, scale, w_qkv, b_qkv, gq, bq, gk, bk, w_o, b_o, heads: int,
                          n_threads: int = 0) -> np.ndarray:
    """Spatial (kind 0) or temporal (kind 1) attention module on x: [T, S, C], C = heads * D.
    Returns [T, S, C] in fp64.  The 3C outputs of the qkv projection are [q | k | v], each laid
    out head-major ([heads, D])."""
    x = np.asarray(x, np.float64)
    T, S, C = x.shape
    D = C // heads
    h = modulate(layer_norm(x), shift, scale)
    qkv = linear(h, w_qkv, b_qkv).reshape(T, S, 3, heads, D)
    q = head_layer_norm(qkv[:, :, 0], gq, bq)
    k = head_layer_norm(qkv[:, :, 1], gk, bk)
    v = qkv[:, :, 2]
    if kind == 1:   # frames are the sequence: rotate by the frame index
        pos = np.arange(T)
        q = np.moveaxis(rotary(np.moveaxis(q, 0, 1), pos), 1, 0)   # rotary wants [.., P, H, D]: put T third from last
        k = np.moveaxis(rotary(np.moveaxis(k, 0, 1), pos), 1, 0)
    o = _attn.kind_attention(kind, np.ascontiguousarray(q), np.ascontiguousarray(k), np.ascontiguousarray(v),
                             n_threads=n_threads)
    return linear(np.asarray(o, np.float64).reshape(T, S, C), w_o, b_o)


def cross_attention_module(x, y, w_q, b_q, w_kv, b_kv, w_o, b_o, heads: int, n_threads: int = 0) -> np.ndarray:
    """Cross attention module: queries from the video tokens x [T, S, C], keys and values from
    the text tokens y [L, C] through one projection to [k | v]; no normalisation, no position."""
    x = np.asarray(x, np.float64)
    T, S, C = x.shape
    D = C // heads
    L = np.asarray(y).shape[0]
    q = linear(x, w_q, b_q).reshape(T, S, heads, D)
    kv = linear(y, w_kv, b_kv).reshape(L, 2, heads, D)
    o = _attn.kind_attention(2, np.ascontiguousarray(q), np.ascontiguousarray(kv[:, 0]),
                             np.ascontiguousarray(kv[:, 1]), n_threads=n_threads)
    return linear(np.asarray(o, np.float64).reshape(T, S, C), w_o, b_o)


def gelu_tanh(x: np.ndarray) -> np.ndarray:
    """Activation of the MLP: GELU in its tanh form, 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))."""
    x = np.asarray(x, np.float64)
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def mlp_module(x, shift, scale, w1, b1, w2, b2) -> np.ndarray:
    """The MLP module of a transformer block, the other object the paper broadcasts (Sec. 2.3 last
    sentence, App. A.2.2 MLP table): layernorm + modulate as in the attention modules, a projection
    to the inner width, the activation, a projection back.  x: [..., C]; w1: [F, C]; w2: [C, F]."""
    h = modulate(layer_norm(x), shift, scale)
    return linear(gelu_tanh(linear(h, w1, b1)), w2, b2)
