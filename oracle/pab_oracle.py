"""ctypes front end of the fp64 CPU oracle (``pab_oracle.c``).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module; the product package never does.
It shares nothing with the HIP library.

What it states (paper Sec. 2.1 for the three attention kinds, Sec. 2.3 Eq. 1 for
the broadcast schedule, App. A.2.1 for the per-kind broadcast ranges and the
segment of steps in which broadcasting is active):

* ``schedule`` / ``source_step`` / ``schedule_row``: compute-or-reuse per step.
* ``attention``: softmax(Q K^T / sqrt(D)) V on strided fp64 views.
* ``spatial`` / ``temporal`` / ``cross``: the three views of the activation
  tensor ``[T, S, H, D]`` (frames, tokens per frame, heads, head dim).
* ``VideoOracle``: plays the schedule over a whole video and keeps, per
  (block, kind), the fp64 output of the last computed step (the broadcast
  output Y* of Eq. 1).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pab_oracle.c")
_LIB = os.path.join(_HERE, "libpab_oracle.so")

COMPUTE = 0
REUSE = 1

SPATIAL = 0
TEMPORAL = 1
CROSS = 2


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, OpenMP over batch x head x row)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
             "-fno-fast-math", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.pab_oracle_schedule.restype = ctypes.c_int
        lib.pab_oracle_schedule.argtypes = [ctypes.c_long] * 4
        lib.pab_oracle_source_step.restype = ctypes.c_long
        lib.pab_oracle_source_step.argtypes = [ctypes.c_long] * 4
        lib.pab_oracle_mlp_schedule.restype = ctypes.c_int
        lib.pab_oracle_mlp_schedule.argtypes = [ctypes.c_long, ctypes.c_long, ctypes.POINTER(ctypes.c_long), ctypes.c_long,
                                                ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.POINTER(ctypes.c_long)]
        lib.pab_oracle_window.restype = ctypes.c_long
        lib.pab_oracle_window.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_long, ctypes.c_double,
                                          ctypes.c_double, ctypes.POINTER(ctypes.c_long), ctypes.POINTER(ctypes.c_long)]
        lib.pab_oracle_attention.restype = ctypes.c_int
        dp = ctypes.POINTER(ctypes.c_double)
        lp = ctypes.POINTER(ctypes.c_long)
        lib.pab_oracle_attention.argtypes = (
            [dp, dp, dp, dp] + [ctypes.c_long] * 5 + [lp, lp, lp, lp] + [ctypes.c_int])
        _lib = lib
    return _lib


# --------------------------------------------------------------------------
# schedule (Eq. 1)
# --------------------------------------------------------------------------
def schedule(step: int, lo: int, hi: int, n: int) -> int:
    """COMPUTE or REUSE for one step; ValueError on meaningless arguments."""
    r = _load().pab_oracle_schedule(step, lo, hi, n)
    if r < 0:
        raise ValueError("bad schedule arguments step=%d lo=%d hi=%d n=%d" % (step, lo, hi, n))
    return r


def source_step(step: int, lo: int, hi: int, n: int) -> int:
    """Step whose computed output is delivered at ``step``."""
    r = _load().pab_oracle_source_step(step, lo, hi, n)
    if r < 0:
        raise ValueError("bad schedule arguments")
    return r


def schedule_row(n_steps: int, lo: int, hi: int, n: int) -> str:
    """One character per step: 'C' computed, 'R' reused."""
    return "".join("CR"[schedule(s, lo, hi, n)] for s in range(n_steps))


def mlp_schedule(step: int, block: int, starts, n: int, block_lo: int, block_hi: int):
    """(decision, source step) of the MLP broadcast (paper App. A.2.2, MLP table): 0 computed, 1 reused."""
    arr = (ctypes.c_long * max(len(starts), 1))(*starts)
    src = ctypes.c_long(-1)
    r = _load().pab_oracle_mlp_schedule(step, block, arr, len(starts), n, block_lo, block_hi, ctypes.byref(src))
    if r < 0:
        raise ValueError("bad MLP schedule arguments")
    return r, src.value


def start_steps_from_timesteps(timesteps, start_timesteps):
    """Step index of each starting timestep of the MLP table on a sampler's timestep list (never
    increasing): the first step whose timestep is not above it.  None for a start below every timestep."""
    out = []
    for t0 in start_timesteps:
        hit = None
        for s, t in enumerate(timesteps):
            if t <= t0:
                hit = s
                break
        out.append(hit)
    return out


def window_from_timesteps(timesteps, t_start: float, t_end: float):
    """(lo, hi) step indices of the timestep window [t_start - t_end] (paper App. A.2.1:
    1000 = start of denoising, 0 = end), or None if no step of the sampler falls inside."""
    ts = np.ascontiguousarray(np.asarray(timesteps, dtype=np.float64))
    lo, hi = ctypes.c_long(-1), ctypes.c_long(-1)
    r = _load().pab_oracle_window(ts.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), len(ts),
                                  float(t_start), float(t_end), ctypes.byref(lo), ctypes.byref(hi))
    if r < 0:
        raise ValueError("bad window arguments")
    return None if r == 0 else (lo.value, hi.value)


# --------------------------------------------------------------------------
# attention
# --------------------------------------------------------------------------
def to_f64(x) -> np.ndarray:
    """Exact widening of an fp32 / bf16 / fp64 array or torch tensor to fp64."""
    if isinstance(x, np.ndarray):
        return x.astype(np.float64, copy=False)
    # torch tensor (bf16 has no numpy dtype: widen inside torch, which is exact)
    return x.detach().cpu().double().numpy()


def _strides3(a: np.ndarray):
    if a.strides[3] != a.itemsize:
        raise ValueError("last axis must be contiguous")
    st = (ctypes.c_long * 3)(*(s // a.itemsize for s in a.strides[:3]))
    return st


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, n_threads: int = 0,
              out: np.ndarray | None = None, return_threads: bool = False):
    """q ``[B, Sq, H, D]``, k and v ``[B, Sk, H, D]`` fp64 (any strides on the
    first three axes) -> o ``[B, Sq, H, D]`` fp64."""
    for a in (q, k, v):
        if a.dtype != np.float64 or a.ndim != 4:
            raise ValueError("oracle attention wants 4-d float64 arrays")
    B, Sq, H, D = q.shape
    Bk, Sk, Hk, Dk = k.shape
    if (Bk, Hk, Dk) != (B, H, D) or v.shape != k.shape:
        raise ValueError("shape mismatch q%s k%s v%s" % (q.shape, k.shape, v.shape))
    if out is None:
        out = np.empty((B, Sq, H, D), dtype=np.float64)
    elif out.shape != (B, Sq, H, D) or out.dtype != np.float64:
        raise ValueError("bad out")
    dp = ctypes.POINTER(ctypes.c_double)

    def ptr(a):
        return ctypes.cast(ctypes.c_void_p(a.__array_interface__["data"][0]), dp)

    used = _load().pab_oracle_attention(
        ptr(q), ptr(k), ptr(v), ptr(out), B, H, Sq, Sk, D,
        _strides3(q), _strides3(k), _strides3(v), _strides3(out), int(n_threads))
    if used < 0:
        raise MemoryError("oracle scratch allocation failed")
    if return_threads:
        return out, used
    return out


def spatial(q, k, v, **kw):
    """Sec. 2.1 spatial attention: tokens of one frame attend to each other.
    q, k, v ``[T, S, H, D]``; batch = T frames, sequence = S tokens."""
    return attention(to_f64(q), to_f64(k), to_f64(v), **kw)


def temporal(q, k, v, **kw):
    """Sec. 2.1 temporal attention: the T frames at one spatial position attend
    to each other.  Same ``[T, S, H, D]`` buffers; batch = S, sequence = T.
    The result is returned in ``[T, S, H, D]`` order again."""
    q, k, v = (np.swapaxes(to_f64(a), 0, 1) for a in (q, k, v))   # views [S,T,H,D]
    S, T, H, D = q.shape
    out = np.empty((T, S, H, D), dtype=np.float64)
    res = attention(q, k, v, out=np.swapaxes(out, 0, 1), **kw)
    if isinstance(res, tuple):
        return out, res[1]
    return out


def cross(q, k, v, **kw):
    """Sec. 2.1 cross attention: every video token attends to the L text tokens.
    q ``[tok, H, D]`` (or ``[T, S, H, D]``), k and v ``[L, H, D]``."""
    q = to_f64(q)
    shape = q.shape
    q = q.reshape(1, -1, shape[-2], shape[-1])
    k = to_f64(k)[None]
    v = to_f64(v)[None]
    res = attention(q, k, v, **kw)
    if isinstance(res, tuple):
        return res[0].reshape(shape), res[1]
    return res.reshape(shape)


def kind_attention(kind: int, q, k, v, **kw):
    return (spatial, temporal, cross)[kind](q, k, v, **kw)


def attention_rows(kind: int, q, k, v, rows, **kw):
    """Exact outputs for a sample of query rows (rows of attention are
    independent).  ``rows`` is an integer array ``[n, 3]`` of (t, s, h) triples
    into the ``[T, S, H, D]`` query tensor; returns ``[n, D]`` fp64.
    k and v are ``[T, S, H, D]`` (spatial, temporal) or ``[L, H, D]`` (cross)."""
    rows = np.asarray(rows, dtype=np.int64).reshape(-1, 3)
    D = q.shape[-1]
    out = np.empty((len(rows), D), dtype=np.float64)
    for i, (t, s, h) in enumerate(rows):
        qi = to_f64(q[t, s, h]).reshape(1, 1, 1, D)
        if kind == SPATIAL:
            kk, vv = k[t, :, h], v[t, :, h]
        elif kind == TEMPORAL:
            kk, vv = k[:, s, h], v[:, s, h]
        else:
            kk, vv = k[:, h], v[:, h]
        kk = np.ascontiguousarray(to_f64(kk)).reshape(1, -1, 1, D)
        vv = np.ascontiguousarray(to_f64(vv)).reshape(1, -1, 1, D)
        out[i] = attention(qi, kk, vv, **kw).reshape(D)
    return out


class VideoOracle:
    """Eq. 1 played over a whole sampling run: per (block, kind) the output of
    the last computed step is kept and handed back unchanged on reuse steps."""

    def __init__(self, intervals, lo: int, hi: int):
        self.intervals = tuple(intervals)
        self.lo, self.hi = lo, hi
        self.cache = {}
        self.computes = 0

    def step(self, block: int, kind: int, step: int, qkv_fn):
        """``qkv_fn()`` -> (q, k, v) is only called when the step computes.
        Returns (decision, fp64 output in the layout of q)."""
        dec = schedule(step, self.lo, self.hi, self.intervals[kind])
        if dec == COMPUTE:
            q, k, v = qkv_fn()
            self.cache[(block, kind)] = (step, kind_attention(kind, q, k, v))
            self.computes += 1
        src, out = self.cache[(block, kind)]
        assert src == source_step(step, self.lo, self.hi, self.intervals[kind])
        return dec, out
