"""Thin ctypes binding of libpab.so: argument marshalling only.

Every function here has the name and meaning of the C entry point it calls
(``include/pab.h``); tensors are torch CUDA tensors used purely as device
memory, the stream is torch's current stream unless one is passed.  There is no
fallback of any kind: if the library has not been built this module raises on
import, and every step of the path runs in the library's HIP kernels.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpab.so")

SPATIAL, TEMPORAL, CROSS = 0, 1, 2
COMPUTE, REUSE = 0, 1
OK, EINVAL, ESTATE, ENOMEM, EDEVICE = 0, -1, -2, -3, -4
BF16, F32 = 0, 1

EXPORTS = (
    "pab_schedule", "pab_source_step", "pab_window_from_timesteps", "pab_preset", "pab_workspace_bytes", "pab_create", "pab_reset", "pab_attention",
    "pab_attention_compute", "pab_linear", "pab_module_scratch_bytes", "pab_module_compute", "pab_module_attention",
    "pab_module_static_scratch_bytes", "pab_module_compute_static",
    "pab_mlp_schedule", "pab_mlp_source_step", "pab_steps_from_timesteps", "pab_mlp_scratch_bytes", "pab_mlp_compute",
    "pab_mlp_workspace_bytes", "pab_mlp_create", "pab_mlp_reset", "pab_mlp", "pab_mlp_launch_count", "pab_mlp_slot_ptr",
    "pab_mlp_destroy",
    "pab_launch_count", "pab_slot_ptr", "pab_destroy", "pab_last_error",
)


class PabError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("libpab status %d: %s" % (status, message))
        self.status = status


class pab_config(ctypes.Structure):
    _fields_ = [("n_blocks", ctypes.c_int), ("T", ctypes.c_int), ("S", ctypes.c_int), ("L", ctypes.c_int),
                ("heads", ctypes.c_int), ("head_dim", ctypes.c_int), ("dtype", ctypes.c_int),
                ("n_steps", ctypes.c_int), ("interval", ctypes.c_int * 3),
                ("range_lo", ctypes.c_int), ("range_hi", ctypes.c_int),
                ("block_kinds", ctypes.POINTER(ctypes.c_ubyte))]


class pab_module_weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("shift", "scale", "w_qkv", "b_qkv", "gamma_q", "beta_q", "gamma_k",
                                               "beta_k", "w_kv", "b_kv", "w_o", "b_o")]


class pab_mlp_weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("shift", "scale", "w1", "b1", "w2", "b2")]


class pab_mlp_config(ctypes.Structure):
    _fields_ = [("n_blocks", ctypes.c_int), ("n_steps", ctypes.c_int), ("n_tok", ctypes.c_longlong),
                ("hidden", ctypes.c_int), ("inner", ctypes.c_int), ("n_starts", ctypes.c_int), ("range", ctypes.c_int),
                ("block_lo", ctypes.c_int), ("block_hi", ctypes.c_int)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libpab.so is not built (%s missing): run `python -m paper_2408_12588_amd.build` "
            "or __graft_entry__.build(); there is no fallback path" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.pab_schedule.restype = ci
    lib.pab_schedule.argtypes = [ci] * 5
    lib.pab_source_step.restype = ci
    lib.pab_source_step.argtypes = [ci] * 5
    lib.pab_window_from_timesteps.restype = ci
    lib.pab_window_from_timesteps.argtypes = [ctypes.POINTER(ctypes.c_double), ci, ctypes.c_double, ctypes.c_double,
                                              ctypes.POINTER(ci), ctypes.POINTER(ci)]
    lib.pab_preset.restype = ci
    lib.pab_preset.argtypes = [ci, ci, ctypes.POINTER(ci), ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.pab_workspace_bytes.restype = ctypes.c_size_t
    lib.pab_workspace_bytes.argtypes = [ctypes.POINTER(pab_config)]
    lib.pab_create.restype = ci
    lib.pab_create.argtypes = [ctypes.POINTER(pab_config), vp, ctypes.c_size_t, ctypes.POINTER(vp)]
    lib.pab_reset.restype = ci
    lib.pab_reset.argtypes = [vp]
    lib.pab_attention.restype = ci
    lib.pab_attention.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp, ctypes.POINTER(vp)]
    lib.pab_attention_compute.restype = ci
    lib.pab_attention_compute.argtypes = [ci] * 7 + [vp] * 5
    lib.pab_linear.restype = ci
    lib.pab_linear.argtypes = [ci, ci, ci, vp, vp, vp, vp, ctypes.c_longlong, vp]
    lib.pab_module_scratch_bytes.restype = ctypes.c_size_t
    lib.pab_module_scratch_bytes.argtypes = [ctypes.POINTER(pab_config)]
    lib.pab_module_compute.restype = ci
    lib.pab_module_compute.argtypes = [ci] * 6 + [vp, vp, ctypes.POINTER(pab_module_weights), vp, ctypes.c_size_t, vp, vp]
    lib.pab_module_static_scratch_bytes.restype = ctypes.c_size_t
    lib.pab_module_static_scratch_bytes.argtypes = []
    lib.pab_module_compute_static.restype = ci
    lib.pab_module_compute_static.argtypes = [ci] * 6 + [vp, vp, ctypes.POINTER(pab_module_weights), vp, vp]
    lib.pab_module_attention.restype = ci
    lib.pab_module_attention.argtypes = [vp, ci, ci, ci, vp, vp, ctypes.POINTER(pab_module_weights), vp,
                                         ctypes.c_size_t, vp, ctypes.POINTER(vp)]
    ip, dp = ctypes.POINTER(ci), ctypes.POINTER(ctypes.c_double)
    lib.pab_mlp_schedule.restype = ci
    lib.pab_mlp_schedule.argtypes = [ci, ci, ip, ci, ci, ci, ci]
    lib.pab_mlp_source_step.restype = ci
    lib.pab_mlp_source_step.argtypes = [ci, ci, ip, ci, ci, ci, ci]
    lib.pab_steps_from_timesteps.restype = ci
    lib.pab_steps_from_timesteps.argtypes = [dp, ci, dp, ci, ip]
    lib.pab_mlp_scratch_bytes.restype = ctypes.c_size_t
    lib.pab_mlp_scratch_bytes.argtypes = [ctypes.c_longlong, ci, ci]
    lib.pab_mlp_compute.restype = ci
    lib.pab_mlp_compute.argtypes = [ctypes.c_longlong, ci, ci, vp, ctypes.POINTER(pab_mlp_weights), vp, ctypes.c_size_t, vp, vp]
    lib.pab_mlp_workspace_bytes.restype = ctypes.c_size_t
    lib.pab_mlp_workspace_bytes.argtypes = [ctypes.POINTER(pab_mlp_config)]
    lib.pab_mlp_create.restype = ci
    lib.pab_mlp_create.argtypes = [ctypes.POINTER(pab_mlp_config), ip, vp, ctypes.c_size_t, ctypes.POINTER(vp)]
    lib.pab_mlp_reset.restype = ci
    lib.pab_mlp_reset.argtypes = [vp]
    lib.pab_mlp.restype = ci
    lib.pab_mlp.argtypes = [vp, ci, ci, vp, ctypes.POINTER(pab_mlp_weights), vp, ctypes.c_size_t, vp, vp, ctypes.POINTER(vp)]
    lib.pab_mlp_launch_count.restype = ctypes.c_longlong
    lib.pab_mlp_launch_count.argtypes = [vp]
    lib.pab_mlp_slot_ptr.restype = vp
    lib.pab_mlp_slot_ptr.argtypes = [vp, ci]
    lib.pab_mlp_destroy.restype = ci
    lib.pab_mlp_destroy.argtypes = [vp]
    lib.pab_launch_count.restype = ctypes.c_longlong
    lib.pab_launch_count.argtypes = [vp]
    lib.pab_slot_ptr.restype = vp
    lib.pab_slot_ptr.argtypes = [vp, ci, ci]
    lib.pab_destroy.restype = ci
    lib.pab_destroy.argtypes = [vp]
    lib.pab_last_error.restype = ctypes.c_char_p
    lib.pab_last_error.argtypes = []
    return lib


lib = _load()


def pab_last_error() -> str:
    return lib.pab_last_error().decode()


def _check(status: int) -> int:
    if status < 0:
        raise PabError(status, pab_last_error())
    return status


def pab_schedule(kind: int, step: int, range_lo: int, range_hi: int, interval: int) -> int:
    return _check(lib.pab_schedule(kind, step, range_lo, range_hi, interval))


def pab_source_step(kind: int, step: int, range_lo: int, range_hi: int, interval: int) -> int:
    return _check(lib.pab_source_step(kind, step, range_lo, range_hi, interval))


OPEN_SORA, OPEN_SORA_PLAN, LATTE = 0, 1, 2


def pab_window_from_timesteps(timesteps, t_start: float, t_end: float):
    """(range_lo, range_hi) of the timestep window on this sampler's steps, or None if no step is inside."""
    n = len(timesteps)
    arr = (ctypes.c_double * n)(*[float(t) for t in timesteps])
    lo, hi = ctypes.c_int(-1), ctypes.c_int(-1)
    r = _check(lib.pab_window_from_timesteps(arr, n, float(t_start), float(t_end), ctypes.byref(lo), ctypes.byref(hi)))
    return None if r == 0 else (lo.value, hi.value)


def pab_preset(model: int, level: int):
    """((spatial, temporal, cross) broadcast ranges, t_start, t_end) of one of the paper's settings."""
    iv = (ctypes.c_int * 3)()
    a, b = ctypes.c_double(), ctypes.c_double()
    _check(lib.pab_preset(model, level, iv, ctypes.byref(a), ctypes.byref(b)))
    return tuple(iv), a.value, b.value


def make_config(n_blocks, T, S, L, heads, head_dim, dtype, n_steps, interval, range_lo, range_hi,
                block_kinds=None) -> pab_config:
    """``block_kinds``: optional sequence of n_blocks bit masks (bit k = the block has attention of kind k)."""
    cfg = pab_config(n_blocks, T, S, L, heads, head_dim, dtype, n_steps, (ctypes.c_int * 3)(*interval),
                     range_lo, range_hi, None)
    if block_kinds is not None:
        if len(block_kinds) != n_blocks:
            raise ValueError("block_kinds needs one entry per block")
        mask = (ctypes.c_ubyte * n_blocks)(*block_kinds)
        cfg.block_kinds = ctypes.cast(mask, ctypes.POINTER(ctypes.c_ubyte))
        cfg._mask = mask   # keeps the array alive as long as the struct
    return cfg


def config_of(wl, intervals=None) -> pab_config:
    """pab_config of a ``workloads.Workload`` (optionally with other broadcast ranges,
    e.g. (1, 1, 1) masked to the present kinds for the no-broadcast baseline)."""
    iv = tuple(wl.intervals if intervals is None else intervals)
    iv = tuple(i if w > 0 else 0 for i, w in zip(iv, wl.intervals))
    mask = None
    if wl.alternating:   # blocks that hold one kind each get one slot each
        mask = [sum(1 << k for k in wl.kinds_of_block(b)) for b in range(wl.n_blocks)]
    return make_config(wl.n_blocks, wl.T, wl.S, wl.L, wl.heads, wl.head_dim,
                       BF16 if wl.dtype == "bf16" else F32, wl.n_steps, iv, wl.lo, wl.hi, mask)


def pab_workspace_bytes(cfg: pab_config) -> int:
    n = lib.pab_workspace_bytes(ctypes.byref(cfg))
    if n == 0:
        raise PabError(EINVAL, pab_last_error())
    return n


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ptr(t) -> int:
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libpab takes dense device tensors")
    return t.data_ptr()


_TORCH_DTYPE = {BF16: torch.bfloat16, F32: torch.float32}


class PabContext:
    """pab_create / pab_attention / pab_reset / pab_destroy over a workspace
    tensor that this object keeps alive (the C library only borrows it)."""

    def __init__(self, cfg: pab_config, device="cuda:0", workspace: torch.Tensor | None = None):
        self.cfg = cfg
        need = pab_workspace_bytes(cfg)
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=device)
        self.workspace = workspace
        handle = ctypes.c_void_p()
        _check(lib.pab_create(ctypes.byref(cfg), workspace.data_ptr(), workspace.numel(), ctypes.byref(handle)))
        self._h = handle
        self.shape = (cfg.T, cfg.S, cfg.heads, cfg.head_dim)
        self.dtype = _TORCH_DTYPE[cfg.dtype]
        self._numel = cfg.T * cfg.S * cfg.heads * cfg.head_dim

    def pab_attention(self, block: int, kind: int, step: int, q, k, v, stream=None):
        """-> (decision, device pointer of the slot)."""
        out = ctypes.c_void_p()
        dec = _check(lib.pab_attention(self._h, block, kind, step, _ptr(q), _ptr(k), _ptr(v), _stream(stream),
                                       ctypes.byref(out)))
        return dec, out.value

    def pab_module_attention(self, block: int, kind: int, step: int, x, text, w, scratch, stream=None):
        """Module-level call -> (decision, device pointer of the slot holding the module output [T, S, C])."""
        out = ctypes.c_void_p()
        dec = _check(lib.pab_module_attention(
            self._h, block, kind, step, _ptr(x), _ptr(text), ctypes.byref(w) if w is not None else None,
            _ptr(scratch), scratch.numel() if scratch is not None else 0, _stream(stream), ctypes.byref(out)))
        return dec, out.value

    def slot_tensor(self, block: int, kind: int) -> torch.Tensor:
        """View of cache slot (block, kind) inside the workspace tensor (no copy)."""
        p = lib.pab_slot_ptr(self._h, block, kind)
        if not p:
            raise PabError(EINVAL, "no such slot")
        off = p - self.workspace.data_ptr()
        nbytes = self._numel * self.workspace.new_empty(0, dtype=self.dtype).element_size()
        return self.workspace[off:off + nbytes].view(self.dtype).view(self.shape)

    def pab_slot_ptr(self, block: int, kind: int) -> int:
        return lib.pab_slot_ptr(self._h, block, kind) or 0

    def pab_reset(self):
        _check(lib.pab_reset(self._h))

    def pab_launch_count(self) -> int:
        return lib.pab_launch_count(self._h)

    def pab_destroy(self):
        if self._h:
            _check(lib.pab_destroy(self._h))
            self._h = None

    def __del__(self):
        try:
            self.pab_destroy()
        except Exception:
            pass


def pab_attention_compute(kind: int, q, k, v, out=None, L: int | None = None, stream=None):
    """One attention launch without schedule or cache.  q ``[T, S, H, D]``;
    k, v ``[T, S, H, D]`` (spatial, temporal) or ``[L, H, D]`` (cross)."""
    T, S, H, D = q.shape
    dtype = BF16 if q.dtype == torch.bfloat16 else F32
    if q.dtype not in (torch.bfloat16, torch.float32) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share dtype bf16 or f32")
    if kind == CROSS:
        if k.dim() != 3 or tuple(k.shape[1:]) != (H, D) or v.shape != k.shape:
            raise ValueError("cross attention wants k, v of shape [L, H, D]")
        L = k.shape[0]
    else:
        if k.shape != q.shape or v.shape != q.shape:
            raise ValueError("k, v must have the shape of q")
        L = 0
    if out is None:
        out = torch.empty_like(q)
    _check(lib.pab_attention_compute(kind, dtype, T, S, L, H, D, _ptr(q), _ptr(k), _ptr(v), _ptr(out),
                                     _stream(stream)))
    return out


def pab_linear(a, w, bias=None, out=None, stream=None):
    """out = a @ w.T + bias (bf16).  a ``[..., K]`` dense, w ``[N, K]``, bias ``[N]`` or None.  ``out`` may be a
    view whose last axis is dense and whose rows are ``out.stride(-2)`` apart (several projections side by side)."""
    if a.dtype != torch.bfloat16 or w.dtype != torch.bfloat16 or (bias is not None and bias.dtype != torch.bfloat16):
        raise ValueError("pab_linear takes bf16 tensors")
    if not a.is_contiguous() or not w.is_contiguous():
        raise ValueError("a and w must be contiguous")
    K = a.shape[-1]
    N = w.shape[0]
    M = a.numel() // K
    if w.shape[1] != K:
        raise ValueError("w must be [N, K]")
    if out is None:
        out = torch.empty(a.shape[:-1] + (N,), device=a.device, dtype=torch.bfloat16)
    if out.stride(-1) != 1 or out.shape[-1] != N or out.numel() != M * N:
        raise ValueError("out must be [..., N] with a dense last axis")
    if not out.is_cuda:
        raise ValueError("libpab takes device tensors")
    ldc = out.stride(-2) if out.dim() >= 2 else N
    if out.dim() > 2 and any(out.stride(i) != out.stride(i + 1) * out.shape[i + 1] for i in range(out.dim() - 2)):
        raise ValueError("the leading axes of out must collapse into one row index")
    _check(lib.pab_linear(M, N, K, _ptr(a), _ptr(w), _ptr(bias) if bias is not None else None, out.data_ptr(), ldc,
                          _stream(stream)))
    return out


def module_weights(**tensors):
    """pab_module_weights from bf16 device tensors given by field name; keeps them alive on the result."""
    w = pab_module_weights()
    for name, t in tensors.items():
        if t is None:
            continue
        if t.dtype != torch.bfloat16:
            raise ValueError("module weights are bf16")
        setattr(w, name, _ptr(t))
    w._keep = tensors
    return w


def pab_module_scratch_bytes(cfg: pab_config) -> int:
    n = lib.pab_module_scratch_bytes(ctypes.byref(cfg))
    if n == 0:
        raise PabError(EINVAL, pab_last_error())
    return n


def module_scratch(T, S, L, heads, head_dim, device):
    """A scratch tensor (uint8, 256-byte aligned by the allocator) for module calls of this shape."""
    cfg = make_config(1, T, S, max(L, 1), heads, head_dim, BF16, 1, (1, 1, 1), 0, 0)
    return torch.empty(pab_module_scratch_bytes(cfg), dtype=torch.uint8, device=device)


def pab_module_compute(kind: int, x, text, w: pab_module_weights, heads: int, scratch=None, out=None, stream=None):
    """One attention module without schedule or cache: x ``[T, S, C]`` (text ``[L, C]`` for cross) -> ``[T, S, C]``."""
    T, S, C = x.shape
    D = C // heads
    L = text.shape[0] if text is not None else 0
    if scratch is None:
        scratch = module_scratch(T, S, L, heads, D, x.device)
    if out is None:
        out = torch.empty_like(x)
    _check(lib.pab_module_compute(kind, T, S, L, heads, D, _ptr(x), _ptr(text) if text is not None else None,
                                  ctypes.byref(w), _ptr(scratch), scratch.numel(), _ptr(out), _stream(stream)))
    return out


def pab_module_static_scratch_bytes() -> int:
    return lib.pab_module_static_scratch_bytes()


def pab_module_compute_static(kind: int, x, text, w: pab_module_weights, heads: int, out, stream=None):
    """pab_module_compute with the library's built-in scratch: nothing is allocated, ``out`` is the caller's."""
    T, S, C = x.shape
    D = C // heads
    L = text.shape[0] if text is not None else 0
    _check(lib.pab_module_compute_static(kind, T, S, L, heads, D, _ptr(x), _ptr(text) if text is not None else None,
                                         ctypes.byref(w), _ptr(out), _stream(stream)))
    return out


# ---- MLP broadcast ----------------------------------------------------------------------------
def _int_array(values):
    return (ctypes.c_int * max(len(values), 1))(*values)


def pab_mlp_schedule(step, block, start_steps, rng, block_lo, block_hi) -> int:
    return _check(lib.pab_mlp_schedule(step, block, _int_array(start_steps), len(start_steps), rng, block_lo, block_hi))


def pab_mlp_source_step(step, block, start_steps, rng, block_lo, block_hi) -> int:
    return _check(lib.pab_mlp_source_step(step, block, _int_array(start_steps), len(start_steps), rng, block_lo, block_hi))


def pab_steps_from_timesteps(timesteps, start_timesteps):
    """Step index of each starting timestep on the sampler's list (None where no step qualifies)."""
    ts = (ctypes.c_double * len(timesteps))(*[float(t) for t in timesteps])
    st = (ctypes.c_double * max(len(start_timesteps), 1))(*[float(t) for t in start_timesteps])
    out = (ctypes.c_int * max(len(start_timesteps), 1))()
    _check(lib.pab_steps_from_timesteps(ts, len(timesteps), st, len(start_timesteps), out))
    return [None if out[i] < 0 else out[i] for i in range(len(start_timesteps))]


def mlp_weights(**tensors):
    w = pab_mlp_weights()
    for name, t in tensors.items():
        if t is None:
            continue
        if t.dtype != torch.bfloat16:
            raise ValueError("MLP weights are bf16")
        setattr(w, name, _ptr(t))
    w._keep = tensors
    return w


def mlp_scratch(n_tok, hidden, inner, device):
    return torch.empty(lib.pab_mlp_scratch_bytes(n_tok, hidden, inner), dtype=torch.uint8, device=device)


def pab_mlp_compute(x, w: pab_mlp_weights, inner: int, scratch=None, out=None, stream=None):
    """One MLP module without schedule or cache: x ``[..., C]`` bf16 -> same shape."""
    C = x.shape[-1]
    n_tok = x.numel() // C
    if scratch is None:
        scratch = mlp_scratch(n_tok, C, inner, x.device)
    if out is None:
        out = torch.empty_like(x)
    _check(lib.pab_mlp_compute(n_tok, C, inner, _ptr(x), ctypes.byref(w), _ptr(scratch), scratch.numel(), _ptr(out),
                               _stream(stream)))
    return out


class MlpContext:
    """Owns the cache slab (a torch uint8 tensor) and the library context of one MLP-broadcast run."""

    def __init__(self, n_blocks, n_steps, n_tok, hidden, inner, start_steps, rng, block_lo, block_hi, device="cuda:0"):
        self.cfg = pab_mlp_config(n_blocks, n_steps, n_tok, hidden, inner, len(start_steps), rng, block_lo, block_hi)
        nbytes = lib.pab_mlp_workspace_bytes(ctypes.byref(self.cfg))
        self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        handle = ctypes.c_void_p()
        _check(lib.pab_mlp_create(ctypes.byref(self.cfg), _int_array(start_steps), _ptr(self.workspace), nbytes,
                                  ctypes.byref(handle)))
        self._h = handle
        self.shape = (n_tok, hidden)

    def pab_mlp(self, block, step, x, w, scratch, y=None, stream=None):
        """-> (decision, device pointer of the output)."""
        out = ctypes.c_void_p()
        dec = _check(lib.pab_mlp(self._h, block, step, _ptr(x), ctypes.byref(w) if w is not None else None, _ptr(scratch),
                                 scratch.numel() if scratch is not None else 0, _ptr(y), _stream(stream), ctypes.byref(out)))
        return dec, out.value

    def slot_tensor(self, block):
        """View of the cache slot of a participating block inside the workspace tensor (no copy)."""
        p = lib.pab_mlp_slot_ptr(self._h, block)
        if not p:
            raise PabError(EINVAL, "block %d has no MLP cache slot" % block)
        off = p - self.workspace.data_ptr()
        return self.workspace[off:off + self.shape[0] * self.shape[1] * 2].view(torch.bfloat16).view(self.shape)

    def pab_mlp_reset(self):
        _check(lib.pab_mlp_reset(self._h))

    def pab_mlp_launch_count(self) -> int:
        return lib.pab_mlp_launch_count(self._h)

    def pab_mlp_destroy(self):
        if self._h:
            lib.pab_mlp_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.pab_mlp_destroy()
        except Exception:
            pass
