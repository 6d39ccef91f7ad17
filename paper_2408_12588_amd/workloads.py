"""Synthetic video-DiT attention workloads and their seeded input generators.

This module holds NO attention or schedule arithmetic: it only names shapes and
draws random tensors, so that the GPU path and the CPU oracle used by the tests
can be fed the very same values.  It does not load the HIP library.

The five workloads stand in for the paper's measured settings (Sec. 3.1 and
App. A.1: Open-Sora 2 s 480p at 30 steps, Latte 2 s 512x512 at 50 steps,
Open-Sora-Plan 512x512 at many steps, plus larger videos as in Sec. 3.4), whose
real activations would need trained weights and prompts.  Values are i.i.d.
N(0,1) drawn from a counter-based generator keyed by
(workload seed, block, kind, step, tensor), then rounded to the storage dtype.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Tuple

import numpy as np
import torch

SPATIAL, TEMPORAL, CROSS = 0, 1, 2
KIND_NAMES = ("spatial", "temporal", "cross")


@dataclass(frozen=True)
class Workload:
    name: str
    n_blocks: int
    T: int                 # latent frames
    S: int                 # tokens per frame (H*W of the latent grid)
    L: int                 # text keys for cross attention (0: no cross attention)
    heads: int
    head_dim: int
    dtype: str             # "bf16" or "f32": storage type of q, k, v and of the output
    n_steps: int
    intervals: Tuple[int, int, int]   # broadcast range per kind (paper App. A.2.1); 0 = kind absent
    lo: int                # first step (0-based, inclusive) of the broadcast segment
    hi: int                # last step (inclusive) of the broadcast segment
    alternating: bool = False   # Latte-like: even blocks spatial only, odd blocks temporal only
    peaked_frac: float = 0.0    # fraction of query token rows scaled by peaked_scale
    peaked_scale: float = 8.0
    seed: int = 0x50414200

    # ---- structure --------------------------------------------------------
    def kinds_of_block(self, block: int) -> Tuple[int, ...]:
        if self.alternating:
            return (SPATIAL,) if block % 2 == 0 else (TEMPORAL,)
        ks = [k for k in (SPATIAL, TEMPORAL, CROSS) if self.intervals[k] > 0]
        return tuple(ks)

    def calls_per_step(self):
        """(block, kind) pairs in execution order for one denoising step."""
        return [(b, k) for b in range(self.n_blocks) for k in self.kinds_of_block(b)]

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    @property
    def elem_size(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def tokens(self) -> int:
        return self.T * self.S

    # ---- bookkeeping used by the benchmark (counts, not method arithmetic) --
    def flops(self, kind: int) -> float:
        """Unpadded multiply-add work of one computed call: 4 * B * H * Sq * Sk * D."""
        H, D = self.heads, self.head_dim
        if kind == SPATIAL:
            return 4.0 * self.T * H * self.S * self.S * D
        if kind == TEMPORAL:
            return 4.0 * self.S * H * self.T * self.T * D
        return 4.0 * H * self.tokens * self.L * D

    def bytes(self, kind: int) -> float:
        """Algorithmic bytes of one computed call: q, k, v read once, o written once."""
        row = self.heads * self.head_dim * self.elem_size
        if kind == CROSS:
            return (2.0 * self.tokens + 2.0 * self.L) * row
        return 4.0 * self.tokens * row

    def qkv_shapes(self, kind: int):
        full = (self.T, self.S, self.heads, self.head_dim)
        if kind == CROSS:
            kv = (self.L, self.heads, self.head_dim)
            return full, kv, kv
        return full, full, full


TINY = Workload("tiny", n_blocks=2, T=4, S=64, L=16, heads=4, head_dim=32, dtype="f32",
                n_steps=10, intervals=(2, 4, 6), lo=2, hi=8, seed=0x50414201)
OPENSORA_480P = Workload("opensora_480p", n_blocks=28, T=16, S=30 * 53, L=120, heads=16,
                         head_dim=72, dtype="bf16", n_steps=30, intervals=(2, 4, 6), lo=3, hi=27,
                         seed=0x50414202)
LATTE_512 = Workload("latte_512", n_blocks=28, T=16, S=32 * 32, L=0, heads=16, head_dim=72,
                     dtype="bf16", n_steps=50, intervals=(2, 3, 0), lo=5, hi=45, alternating=True,
                     seed=0x50414203)
OSP_512_LONG = Workload("osp_512_long", n_blocks=28, T=17, S=1024, L=300, heads=16, head_dim=72,
                        dtype="bf16", n_steps=100, intervals=(2, 4, 6), lo=10, hi=90,
                        seed=0x50414204)
STRESS_720P = Workload("stress_720p", n_blocks=28, T=16, S=45 * 80, L=120, heads=16, head_dim=72,
                       dtype="bf16", n_steps=30, intervals=(2, 4, 6), lo=3, hi=27,
                       peaked_frac=0.05, seed=0x50414205)

CONFIGS = (TINY, OPENSORA_480P, LATTE_512, OSP_512_LONG, STRESS_720P)
BY_NAME = {w.name: w for w in CONFIGS}

_TENSOR_ID = {"q": 0, "k": 1, "v": 2}


def _philox(seed: int, block: int, kind: int, step: int, tensor: int) -> np.random.Generator:
    # Philox takes a 128-bit key; the fields are packed side by side (no hashing needed,
    # each field has its own bit range).
    key = (int(seed) & 0xFFFFFFFF) | (int(block) & 0xFFFF) << 32 | (int(kind) & 0xFF) << 48 \
        | (int(tensor) & 0xFF) << 56 | (int(step) & 0xFFFFFFFF) << 64
    return np.random.Generator(np.random.Philox(key=key))


def normal(shape, seed: int, block: int = 0, kind: int = 0, step: int = 0, tensor: int = 0) -> np.ndarray:
    """fp32 N(0,1) array from the counter-based stream named by the arguments."""
    return _philox(seed, block, kind, step, tensor).standard_normal(shape, dtype=np.float32)


def peaked_rows(wl: Workload) -> np.ndarray:
    """Token rows (indices into T*S) whose queries are scaled: exactly
    floor(frac * tokens) rows from a seeded permutation, the same for every call."""
    n = int(wl.peaked_frac * wl.tokens)
    if n == 0:
        return np.empty(0, dtype=np.int64)
    perm = _philox(wl.seed, 0xFFFF, 0xFF, 0, 0xFF).permutation(wl.tokens)
    return np.sort(perm[:n])


def make_qkv(wl: Workload, block: int, kind: int, step: int):
    """CPU tensors (q, k, v) for one attention call, in the storage dtype and in
    the layouts the library takes: ``[T, S, H, D]`` (spatial, temporal, cross
    queries) and ``[L, H, D]`` (cross keys / values)."""
    shapes = wl.qkv_shapes(kind)
    out = []
    for name, shape in zip("qkv", shapes):
        a = normal(shape, wl.seed, block, kind, step, _TENSOR_ID[name])
        if name == "q" and wl.peaked_frac > 0.0:
            rows = peaked_rows(wl)
            a.reshape(wl.tokens, wl.heads, wl.head_dim)[rows] *= np.float32(wl.peaked_scale)
        out.append(torch.from_numpy(a).to(wl.torch_dtype))
    return tuple(out)


def sample_rows(wl: Workload, n: int, seed: int) -> np.ndarray:
    """n seeded (t, s, h) query-row triples, always including the corner rows
    (first / last frame, token and head) so tile tails are covered."""
    g = _philox(wl.seed, 0xFFFE, 0xFE, seed, 0xFE)
    rows = np.stack([g.integers(0, wl.T, n), g.integers(0, wl.S, n), g.integers(0, wl.heads, n)], 1)
    corners = np.array([[0, 0, 0], [wl.T - 1, wl.S - 1, wl.heads - 1],
                        [0, wl.S - 1, 0], [wl.T - 1, 0, wl.heads - 1]])
    return np.concatenate([corners, rows])[:max(n, 4)].astype(np.int64)


# ---- module-level inputs (paper App. B.5 / B.6: the attention module around the operation) ----
# Random-init stand-ins for trained weights: projection rows of about unit norm, modulation and
# learned norm parameters small around their identity values.  Tensor ids 16.. keep these streams
# apart from the q / k / v ones.
_MODULE_TENSORS = ("shift", "scale", "w_qkv", "b_qkv", "gamma_q", "beta_q", "gamma_k", "beta_k", "w_kv", "b_kv",
                   "w_o", "b_o")


def make_module_weights(wl: Workload, block: int, kind: int) -> dict:
    """bf16 CPU tensors of one attention module's weights, named as the library's weight struct.
    Self attention (spatial, temporal): shift, scale, w_qkv [3C, C], b_qkv, gamma/beta of q and k, w_o, b_o.
    Cross attention: w_qkv [C, C] (queries), b_qkv, w_kv [2C, C], b_kv, w_o, b_o."""
    C, D = wl.heads * wl.head_dim, wl.head_dim
    inv = 1.0 / np.sqrt(C)

    def draw(name, shape, scale, offset=0.0):
        a = normal(shape, wl.seed, block, kind, 0, 16 + _MODULE_TENSORS.index(name)) * np.float32(scale) + np.float32(offset)
        return torch.from_numpy(a).to(torch.bfloat16)

    w = {"w_o": draw("w_o", (C, C), inv), "b_o": draw("b_o", (C,), 0.1)}
    if kind == CROSS:
        w.update(w_qkv=draw("w_qkv", (C, C), inv), b_qkv=draw("b_qkv", (C,), 0.1),
                 w_kv=draw("w_kv", (2 * C, C), inv), b_kv=draw("b_kv", (2 * C,), 0.1))
    else:
        w.update(shift=draw("shift", (C,), 0.3), scale=draw("scale", (C,), 0.3),
                 w_qkv=draw("w_qkv", (3 * C, C), inv), b_qkv=draw("b_qkv", (3 * C,), 0.1),
                 gamma_q=draw("gamma_q", (D,), 0.2, 1.0), beta_q=draw("beta_q", (D,), 0.2),
                 gamma_k=draw("gamma_k", (D,), 0.2, 1.0), beta_k=draw("beta_k", (D,), 0.2))
    return w


def make_module_input(wl: Workload, block: int, kind: int, step: int) -> torch.Tensor:
    """Hidden states x ``[T, S, C]`` (bf16, N(0,1)) entering the module of (block, kind) at a step."""
    C = wl.heads * wl.head_dim
    return torch.from_numpy(normal((wl.T, wl.S, C), wl.seed, block, kind, step, 8)).to(torch.bfloat16)


def make_text(wl: Workload) -> torch.Tensor:
    """Text tokens ``[L, C]`` (bf16, N(0,1)) the cross-attention modules attend to; one per workload."""
    C = wl.heads * wl.head_dim
    return torch.from_numpy(normal((max(wl.L, 1), C), wl.seed, 0xFFFD, 0xFD, 0, 9)).to(torch.bfloat16)
