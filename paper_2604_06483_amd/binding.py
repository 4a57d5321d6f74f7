"""ctypes binding of the C-ABI library (include/ll.h).

Argument marshalling only: every step of the path runs in the HIP kernels of libll.so.
PyTorch supplies device memory and the stream.  If the library has not been built
(`python -m paper_2604_06483_amd.build`) loading raises: there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

import torch

LL_OK, LL_EINVAL, LL_EWORKSPACE, LL_EHIP, LL_ESCRATCH = 0, -1, -2, -3, -4
LL_KMAX = 32
LL_STATIC_SCRATCH_BYTES = 64 << 20
LL_FLAG_TOPK_SOFTMAX = 1
LL_FLAG_REGISTER_STAGED = 2

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libll.so")
_lib = None


class ll_shape(Structure):
    _fields_ = [("N", c_int64), ("d", c_int32), ("V", c_int32)]


class LLError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().ll_error_string(code).decode()
        if code == LL_EHIP:
            msg += f" [hipError {lib().ll_last_hip_error()}]"
        super().__init__(f"{where}: {msg} ({code})")


class ll_capture_shape(Structure):
    _fields_ = [("L", c_int32), ("C", c_int32), ("T", c_int64), ("d", c_int32)]


_PROJECT_ARGS = [POINTER(ll_shape), c_void_p, c_size_t, c_void_p, c_void_p, c_void_p, c_float, c_int,
                 c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]


def lib() -> ctypes.CDLL:
    """The loaded shared library with its prototypes set."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2604_06483_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        L.ll_workspace_bytes.argtypes = [POINTER(ll_shape), c_int]
        L.ll_workspace_bytes.restype = c_size_t
        L.ll_project.argtypes = _PROJECT_ARGS
        L.ll_project.restype = c_int
        L.ll_project_ex.argtypes = _PROJECT_ARGS[:6] + [c_void_p, ctypes.c_uint] + _PROJECT_ARGS[6:]
        L.ll_project_ex.restype = c_int
        L.ll_project_timed.argtypes = _PROJECT_ARGS + [POINTER(c_float)]
        L.ll_project_timed.restype = c_int
        L.ll_project_static.argtypes = _PROJECT_ARGS[:1] + _PROJECT_ARGS[3:]
        L.ll_project_static.restype = c_int
        L.ll_project_static_pass_rows.argtypes = [POINTER(ll_shape), c_int]
        L.ll_project_static_pass_rows.restype = c_int64
        L.ll_steer_workspace_bytes.argtypes = [c_int32]
        L.ll_steer_workspace_bytes.restype = c_size_t
        L.ll_steer_vector.argtypes = [c_void_p, c_int64, c_void_p, c_int64, c_int32, c_int, c_void_p,
                                      c_void_p, c_size_t, c_void_p]
        L.ll_steer_vector.restype = c_int
        L.ll_steer_inject.argtypes = [POINTER(ll_shape), c_void_p, c_void_p, c_float, c_void_p, c_float,
                                      c_void_p, c_void_p]
        L.ll_steer_inject.restype = c_int
        L.ll_steer_sweep_workspace_bytes.argtypes = [POINTER(ll_shape), c_int]
        L.ll_steer_sweep_workspace_bytes.restype = c_size_t
        L.ll_steer_sweep.argtypes = [POINTER(ll_shape), c_void_p, c_size_t, c_void_p, c_void_p, c_void_p, c_float,
                                     c_void_p, POINTER(c_float), c_int, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                     c_void_p]
        L.ll_steer_sweep.restype = c_int
        L.ll_steer_sweep_topk_workspace_bytes.argtypes = [POINTER(ll_shape), c_int, c_int]
        L.ll_steer_sweep_topk_workspace_bytes.restype = c_size_t
        L.ll_steer_sweep_topk.argtypes = [POINTER(ll_shape), c_void_p, c_size_t, c_void_p, c_void_p, c_void_p, c_float,
                                          c_void_p, POINTER(c_float), c_int, c_int, c_void_p, c_void_p, c_void_p, c_void_p,
                                          c_void_p, c_void_p]
        L.ll_steer_sweep_topk.restype = c_int
        L.ll_steer_inject_raw.argtypes = [POINTER(ll_shape), c_void_p, c_void_p, c_float, c_float, c_float, c_void_p, c_void_p]
        L.ll_steer_inject_raw.restype = c_int
        L.ll_capture_append.argtypes = [POINTER(ll_capture_shape), c_void_p, c_void_p, c_int64, c_int64, c_void_p]
        L.ll_capture_append.restype = c_int
        L.ll_error_string.argtypes = [c_int]
        L.ll_error_string.restype = c_char_p
        L.ll_last_hip_error.argtypes = []
        L.ll_last_hip_error.restype = c_int
        _lib = L
    return _lib


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _check(t, dtype, name, shape=None):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous {dtype} tensor on the GPU")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return c_void_p(s.cuda_stream)


def _scratch(nbytes, device, stream):
    """A workspace of this call's own.  It is released when the call returns, while the kernels may
    still be queued: tell the allocator which stream uses it, so that the block is not handed to
    another stream's tensor before they have run."""
    ws = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    if stream is not None:
        ws.record_stream(stream)
    return ws


def ll_workspace_bytes(N: int, d: int, V: int, k: int) -> int:
    return int(lib().ll_workspace_bytes(ll_shape(N, d, V), k))


def ll_steer_workspace_bytes(d: int) -> int:
    return int(lib().ll_steer_workspace_bytes(d))


def ll_project(hidden, gamma, W_U, eps, k, target_ids=None, *, workspace=None, stream=None, out=None, timed=False,
               bias=None, topk_softmax=False, register_staged=False):
    """hidden [..., d] bf16, gamma [d] bf16 or None, W_U [V, d] bf16, target_ids [N] int32 or None.
    bias [V] fp32 (the b of Eq. 1), topk_softmax (probabilities over the k selected logits only, the paper's
    own output format) and register_staged (the kernel with the norm inside its A-tile load) go through
    ll_project_ex.

    Returns (topk_ids [N,k] int32, topk_p [N,k] fp32, target_logp [N] fp32 or None, entropy [N] fp32),
    plus the three phase times in ms when timed=True (that variant synchronises the stream).
    """
    d = hidden.shape[-1]
    h2 = hidden.reshape(-1, d)
    N = h2.shape[0]
    V = W_U.shape[0]
    _check(h2, torch.bfloat16, "hidden")
    _check(W_U, torch.bfloat16, "W_U", (V, d))
    if gamma is not None:
        _check(gamma, torch.bfloat16, "gamma", (d,))
    if target_ids is not None:
        _check(target_ids, torch.int32, "target_ids", (N,))
    shape = ll_shape(N, d, V)
    need = int(lib().ll_workspace_bytes(shape, k))
    if workspace is None:
        workspace = _scratch(need, hidden.device, stream)
    dev = hidden.device
    if out is None:
        ids = torch.empty((N, k), dtype=torch.int32, device=dev)
        p = torch.empty((N, k), dtype=torch.float32, device=dev)
        logp = torch.empty((N,), dtype=torch.float32, device=dev) if target_ids is not None else None
        ent = torch.empty((N,), dtype=torch.float32, device=dev)
    else:
        ids, p, logp, ent = out
    args = [shape, _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(h2), _ptr(gamma), _ptr(W_U),
            float(eps), int(k), _ptr(target_ids), _ptr(ids), _ptr(p), _ptr(logp), _ptr(ent), _stream(stream)]
    if bias is not None or topk_softmax or register_staged:
        if timed:
            raise ValueError("the timed variant has no bias / top-k-softmax / kernel-choice form")
        if bias is not None:
            _check(bias, torch.float32, "bias", (V,))
        flags = (LL_FLAG_TOPK_SOFTMAX if topk_softmax else 0) | (LL_FLAG_REGISTER_STAGED if register_staged else 0)
        rc = lib().ll_project_ex(*args[:6], _ptr(bias), flags, *args[6:])
        if rc != LL_OK:
            raise LLError(rc, "ll_project_ex")
        return ids, p, logp, ent
    if timed:
        ms = (c_float * 3)()
        rc = lib().ll_project_timed(*args, ms)
        if rc != LL_OK:
            raise LLError(rc, "ll_project_timed")
        return ids, p, logp, ent, [float(x) for x in ms]
    rc = lib().ll_project(*args)
    if rc != LL_OK:
        raise LLError(rc, "ll_project")
    return ids, p, logp, ent


def ll_project_static_pass_rows(N: int, d: int, V: int, k: int) -> int:
    return int(lib().ll_project_static_pass_rows(ll_shape(N, d, V), k))


def ll_project_static(hidden, gamma, W_U, eps, k, target_ids=None, *, stream=None, out=None):
    """ll_project without a workspace: the library's own static device buffer holds the partial results, and the
    call allocates nothing (pass `out` to keep this wrapper from allocating the result tensors).  Calls that may
    overlap on one GPU race on that buffer.  Same results as ll_project."""
    d = hidden.shape[-1]
    h2 = hidden.reshape(-1, d)
    N = h2.shape[0]
    V = W_U.shape[0]
    _check(h2, torch.bfloat16, "hidden")
    _check(W_U, torch.bfloat16, "W_U", (V, d))
    if gamma is not None:
        _check(gamma, torch.bfloat16, "gamma", (d,))
    if target_ids is not None:
        _check(target_ids, torch.int32, "target_ids", (N,))
    dev = hidden.device
    if out is None:
        ids = torch.empty((N, k), dtype=torch.int32, device=dev)
        p = torch.empty((N, k), dtype=torch.float32, device=dev)
        logp = torch.empty((N,), dtype=torch.float32, device=dev) if target_ids is not None else None
        ent = torch.empty((N,), dtype=torch.float32, device=dev)
    else:
        ids, p, logp, ent = out
    rc = lib().ll_project_static(ll_shape(N, d, V), _ptr(h2), _ptr(gamma), _ptr(W_U), float(eps), int(k), _ptr(target_ids),
                                 _ptr(ids), _ptr(p), _ptr(logp), _ptr(ent), _stream(stream))
    if rc != LL_OK:
        raise LLError(rc, "ll_project_static")
    return ids, p, logp, ent


def ll_steer_vector(base, target, normalize=True, *, workspace=None, stream=None, out=None):
    """base [Nb, d], target [Nt, d] bf16 -> v [d] fp32 (paper Eq. 2)."""
    _check(base, torch.bfloat16, "base")
    _check(target, torch.bfloat16, "target")
    d = base.shape[-1]
    if target.shape[-1] != d or base.dim() != 2 or target.dim() != 2:
        raise ValueError("base and target must be [rows, d] with the same d")
    v = torch.empty((d,), dtype=torch.float32, device=base.device) if out is None else out
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().ll_steer_vector(_ptr(base), base.shape[0], _ptr(target), target.shape[0], d, int(bool(normalize)),
                               _ptr(v), _ptr(workspace), wsb, _stream(stream))
    if rc != LL_OK:
        raise LLError(rc, "ll_steer_vector")
    return v


def ll_steer_inject(hidden, gamma, eps, v, alpha, *, stream=None, out=None):
    """bf16(RMSNorm(hidden) + alpha v), same shape as hidden (paper Eq. 3, post-norm)."""
    d = hidden.shape[-1]
    h2 = hidden.reshape(-1, d)
    _check(h2, torch.bfloat16, "hidden")
    _check(gamma, torch.bfloat16, "gamma", (d,))
    _check(v, torch.float32, "v", (d,))
    o = torch.empty_like(h2) if out is None else out.reshape(-1, d)
    rc = lib().ll_steer_inject(ll_shape(h2.shape[0], d, 0), _ptr(h2), _ptr(gamma), float(eps), _ptr(v), float(alpha),
                               _ptr(o), _stream(stream))
    if rc != LL_OK:
        raise LLError(rc, "ll_steer_inject")
    return o.reshape(hidden.shape)


LL_SWEEP_MAX = 9
LL_SWEEP_KMAX = 4


def ll_steer_sweep_workspace_bytes(N: int, d: int, V: int, n_alpha: int, k: int = 1) -> int:
    if k == 1:
        return int(lib().ll_steer_sweep_workspace_bytes(ll_shape(N, d, V), n_alpha))
    return int(lib().ll_steer_sweep_topk_workspace_bytes(ll_shape(N, d, V), n_alpha, k))


def ll_steer_sweep(hidden, gamma, W_U, eps, v, alphas, target_ids=None, *, k=None, workspace=None, stream=None):
    """Lens read-out of the steered rows RMSNorm(hidden) + alpha v for every alpha of the list in one pass over
    W_U (paper Eq. 3 / Sec. 3.4).  v [d] fp32 on the GPU, alphas a sequence of at most LL_SWEEP_MAX floats.

    Returns (top1_ids [A,N] int32, top1_p [A,N] fp32, target_logp [A,N] fp32 or None, entropy [A,N] fp32);
    with k given (1..LL_SWEEP_KMAX, through ll_steer_sweep_topk) the first two are [A,N,k] lists.
    """
    d = hidden.shape[-1]
    h2 = hidden.reshape(-1, d)
    N = h2.shape[0]
    V = W_U.shape[0]
    A = len(alphas)
    _check(h2, torch.bfloat16, "hidden")
    _check(W_U, torch.bfloat16, "W_U", (V, d))
    _check(v, torch.float32, "v", (d,))
    if gamma is not None:
        _check(gamma, torch.bfloat16, "gamma", (d,))
    if target_ids is not None:
        _check(target_ids, torch.int32, "target_ids", (N,))
    shape = ll_shape(N, d, V)
    need = ll_steer_sweep_workspace_bytes(N, d, V, A, 1 if k is None else int(k))
    if workspace is None:
        workspace = _scratch(need, hidden.device, stream)
    dev = hidden.device
    ids = torch.empty((A, N) if k is None else (A, N, int(k)), dtype=torch.int32, device=dev)
    p = torch.empty((A, N) if k is None else (A, N, int(k)), dtype=torch.float32, device=dev)
    logp = torch.empty((A, N), dtype=torch.float32, device=dev) if target_ids is not None else None
    ent = torch.empty((A, N), dtype=torch.float32, device=dev)
    al = (c_float * max(A, 1))(*[float(x) for x in alphas])
    if k is None:
        rc = lib().ll_steer_sweep(shape, _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(h2), _ptr(gamma),
                                  _ptr(W_U), float(eps), _ptr(v), al, A, _ptr(target_ids), _ptr(ids), _ptr(p), _ptr(logp),
                                  _ptr(ent), _stream(stream))
    else:
        rc = lib().ll_steer_sweep_topk(shape, _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(h2),
                                       _ptr(gamma), _ptr(W_U), float(eps), _ptr(v), al, A, int(k), _ptr(target_ids), _ptr(ids),
                                       _ptr(p), _ptr(logp), _ptr(ent), _stream(stream))
    if rc != LL_OK:
        raise LLError(rc, "ll_steer_sweep" if k is None else "ll_steer_sweep_topk")
    return ids, p, logp, ent


def ll_steer_inject_raw(hidden, v, alpha, layer_scale=1.0, clip_ratio=0.0, *, stream=None, out=None):
    """bf16(hidden + beta v) with beta = alpha * layer_scale clipped to clip_ratio * ||row||_2 (paper Sec. 3.4,
    in-model injection with its two safeguards); same shape as hidden."""
    d = hidden.shape[-1]
    h2 = hidden.reshape(-1, d)
    _check(h2, torch.bfloat16, "hidden")
    _check(v, torch.float32, "v", (d,))
    o = torch.empty_like(h2) if out is None else out.reshape(-1, d)
    rc = lib().ll_steer_inject_raw(ll_shape(h2.shape[0], d, 0), _ptr(h2), _ptr(v), float(alpha), float(layer_scale),
                                   float(clip_ratio), _ptr(o), _stream(stream))
    if rc != LL_OK:
        raise LLError(rc, "ll_steer_inject_raw")
    return o.reshape(hidden.shape)


def ll_capture_append(store, slices, t0, *, stream=None):
    """store [L, C, T, d] bf16, slices [L*C, n_tok, d] bf16: writes tokens t0 .. t0+n_tok-1 of every trajectory
    (paper Sec. 3.1 Stage 2).  store.reshape(-1, d) is then what ll_project takes."""
    _check(store, torch.bfloat16, "store")
    if store.dim() != 4:
        raise ValueError("store: need [L, C, T, d]")
    L, C, T, d = store.shape
    _check(slices, torch.bfloat16, "slices")
    if slices.dim() != 3 or slices.shape[0] != L * C or slices.shape[2] != d:
        raise ValueError(f"slices: shape {tuple(slices.shape)}, expected ({L * C}, n_tok, {d})")
    rc = lib().ll_capture_append(ll_capture_shape(L, C, T, d), _ptr(store), _ptr(slices), int(t0), int(slices.shape[1]),
                                 _stream(stream))
    if rc != LL_OK:
        raise LLError(rc, "ll_capture_append")

