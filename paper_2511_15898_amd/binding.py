"""Thin ctypes binding of libgr_verify.so: the same entry points as include/gr_verify.h.

Argument marshalling only -- every step of the verifier runs in the HIP kernels.  Tensors are
torch CUDA tensors (PyTorch is used for device memory and streams, nothing else).  There is no
CPU fallback: if the library is missing, loading fails loudly."""
from __future__ import annotations

import ctypes
import os

import torch

from .build import LIB_PATH

GR_MAX_SUPPORT = 256
GR_MAX_T = 128
GR_MAX_N = 16
GR_ROW_OK, GR_ROW_TRUNC_CAP, GR_ROW_ITER_CAP, GR_ROW_BAD = 0, 1, 2, 3
GR_OK, GR_EINVAL, GR_ENOMEM, GR_ESTATE, GR_EHIP, GR_EUNSUPPORTED, GR_ECAPACITY = 0, -1, -2, -3, -4, -5, -6
GR_NOALLOC_MAX_B = 256

EXPORTS = ("gr_create", "gr_destroy", "gr_solve", "gr_solve_logits", "gr_tree_walk", "gr_profile_stride", "gr_accept_sweep", "gr_accept_sweep_noalloc", "gr_verify", "gr_solve_verify", "gr_solve_logits_verify", "gr_policy_slice", "gr_policy_export",
           "gr_policy_export_row", "gr_solve_stats", "gr_profile_read", "gr_strerror")
GR_FLAG_PROFILE = 1


class GrConfig(ctypes.Structure):
    _fields_ = [("max_iter", ctypes.c_int), ("max_T", ctypes.c_int), ("rel_tol", ctypes.c_double),
                ("flags", ctypes.c_int), ("tail_mass", ctypes.c_double)]


class GrError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


_lib = None
_solved_shape: dict = {}      # handle -> (B, n, V) of its last gr_solve (argument checking only)


def load_library(path: str | None = None) -> ctypes.CDLL:
    """Load the built library (no build is attempted here)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: run `python __graft_entry__.py` (or paper_2511_15898_amd/build.py) first")
    lib = ctypes.CDLL(path)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.gr_create.argtypes = [ctypes.POINTER(vp), ci, ci, ci, ci, ctypes.POINTER(GrConfig)]
    lib.gr_destroy.argtypes = [vp]
    lib.gr_solve.argtypes = [vp, vp, vp, ci, ci, ctypes.c_float, ci, ci, vp, vp, vp]
    lib.gr_solve_logits.argtypes = [vp, vp, vp, vp, vp, ci, ci, ctypes.c_float, ci, ci, vp, vp, vp]
    lib.gr_accept_sweep.argtypes = [vp, vp, vp, ctypes.POINTER(ci), ci, ctypes.POINTER(ci), ci, ci, ci, vp, vp, vp]
    lib.gr_accept_sweep_noalloc.argtypes = [vp, vp, ctypes.POINTER(ci), ci, ctypes.POINTER(ci), ci, ci, ci, vp, vp, vp]
    lib.gr_verify.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.gr_solve_verify.argtypes = [vp, vp, vp, ci, ci, ctypes.c_float, ci, ci, vp, vp, vp, vp, vp, vp, vp]
    lib.gr_solve_logits_verify.argtypes = [vp, vp, vp, vp, vp, ci, ci, ctypes.c_float, ci, ci, vp, vp, vp, vp, vp, vp, vp]
    lib.gr_tree_walk.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ctypes.c_float, vp, vp, vp, vp, vp]
    lib.gr_policy_slice.argtypes = [vp, vp, vp, vp, vp]
    lib.gr_policy_export.argtypes = [vp] * 9
    lib.gr_solve_stats.argtypes = [vp] * 4
    lib.gr_policy_export_row.argtypes = [vp, ci, ci, vp, vp, vp, vp, vp]
    lib.gr_profile_stride.argtypes = [vp, ci]
    lib.gr_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                    ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ci)]
    lib.gr_strerror.argtypes = [ci]
    lib.gr_strerror.restype = ctypes.c_char_p
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().gr_strerror(int(code)).decode()


def _ptr(t: torch.Tensor | None, dtype: torch.dtype, what: str) -> int | None:
    if t is None:
        return None
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{what}: need a contiguous CUDA tensor of {dtype}")
    return t.data_ptr()


def _stream(stream) -> int:
    return (stream if stream is not None else torch.cuda.current_stream()).cuda_stream


def gr_create(max_B: int, max_V: int, max_k: int = GR_MAX_SUPPORT, max_n: int = GR_MAX_N, max_iter: int = 0, max_T: int = 0,
              rel_tol: float = 0.0, flags: int = 0, tail_mass: float = 0.0) -> int:
    """max_k: largest top-k support the handle will serve (<= 0: whole rows; above GR_MAX_SUPPORT the handle
    holds an HBM workspace of 128 bytes per token and row).  tail_mass: nucleus cut of the draft on that path."""
    cfg = GrConfig(max_iter, max_T, rel_tol, flags, tail_mass)
    h = ctypes.c_void_p()
    rc = load_library().gr_create(ctypes.byref(h), max_B, max_V, max_k, max_n, ctypes.byref(cfg))
    if rc != GR_OK:
        raise GrError(rc, "gr_create")
    return h.value


def gr_destroy(handle: int) -> None:
    _solved_shape.pop(handle, None)
    rc = load_library().gr_destroy(handle)
    if rc != GR_OK:
        raise GrError(rc, "gr_destroy")


def gr_solve(handle: int, p: torch.Tensor, q: torch.Tensor, n: int, k: int, tol: float,
             accept_prob: torch.Tensor | None = None, status: torch.Tensor | None = None, stream=None):
    """p, q: [B, V] float32 CUDA tensors.  Returns (accept_prob [B] float32, status [B] int32)."""
    if p.dim() != 2 or p.shape != q.shape:
        raise TypeError("gr_solve: p and q must both be [B, V]")
    B, V = p.shape
    if accept_prob is None:
        accept_prob = torch.empty(B, dtype=torch.float32, device=p.device)
    if status is None:
        status = torch.empty(B, dtype=torch.int32, device=p.device)
    rc = load_library().gr_solve(handle, _ptr(p, torch.float32, "p"), _ptr(q, torch.float32, "q"), n, k, tol, B, V,
                                 _ptr(accept_prob, torch.float32, "accept_prob"), _ptr(status, torch.int32, "status"),
                                 _stream(stream))
    if rc != GR_OK:
        _solved_shape.pop(handle, None)
        raise GrError(rc, "gr_solve")
    _solved_shape[handle] = (B, n, V)
    return accept_prob, status


def gr_solve_logits(handle: int, target_logits: torch.Tensor, draft_logits: torch.Tensor, temperature: torch.Tensor, n: int, k: int,
                    tol: float, accept_prob: torch.Tensor | None = None, status: torch.Tensor | None = None, stream=None,
                    draft_temperature: torch.Tensor | None = None):
    """target_logits, draft_logits: [B, V] float32 CUDA tensors; temperature: [B] float32 (draft_temperature: the draft's
    own, default the same).  Returns (accept_prob, status).
    The target logits and the temperatures stand in for p until the last gr_verify / gr_policy_slice of this solve."""
    if target_logits.dim() != 2 or target_logits.shape != draft_logits.shape:
        raise TypeError("gr_solve_logits: target_logits and draft_logits must both be [B, V]")
    B, V = target_logits.shape
    if temperature.dim() != 1 or temperature.shape[0] != B:
        raise TypeError("gr_solve_logits: temperature must be [B]")
    if draft_temperature is not None and (draft_temperature.dim() != 1 or draft_temperature.shape[0] != B):
        raise TypeError("gr_solve_logits: draft_temperature must be [B]")
    if accept_prob is None:
        accept_prob = torch.empty(B, dtype=torch.float32, device=target_logits.device)
    if status is None:
        status = torch.empty(B, dtype=torch.int32, device=target_logits.device)
    rc = load_library().gr_solve_logits(handle, _ptr(target_logits, torch.float32, "target_logits"),
                                        _ptr(draft_logits, torch.float32, "draft_logits"),
                                        _ptr(temperature, torch.float32, "temperature"),
                                        None if draft_temperature is None else _ptr(draft_temperature, torch.float32, "draft_temperature"),
                                        n, k, tol, B, V,
                                        _ptr(accept_prob, torch.float32, "accept_prob"), _ptr(status, torch.int32, "status"),
                                        _stream(stream))
    if rc != GR_OK:
        _solved_shape.pop(handle, None)
        raise GrError(rc, "gr_solve_logits")
    _solved_shape[handle] = (B, n, V)
    return accept_prob, status


def gr_accept_sweep(handle: int, p: torch.Tensor, q: torch.Tensor, ks, ns,
                    accept_prob: torch.Tensor | None = None, status: torch.Tensor | None = None, stream=None):
    """alpha* over a grid: ks top-k sizes, ns draft counts (host sequences of ints).
    Returns (accept_prob [B, len(ks), len(ns)] float32, status [B] int32)."""
    if p.dim() != 2 or p.shape != q.shape:
        raise TypeError("gr_accept_sweep: p and q must both be [B, V]")
    B, V = p.shape
    ks = [int(k) for k in ks]; ns = [int(n) for n in ns]
    if accept_prob is None:
        accept_prob = torch.empty((B, len(ks), len(ns)), dtype=torch.float32, device=p.device)
    elif tuple(accept_prob.shape) != (B, len(ks), len(ns)):
        raise TypeError("gr_accept_sweep: accept_prob must be [B, len(ks), len(ns)]")
    if status is None:
        status = torch.empty(B, dtype=torch.int32, device=p.device)
    ka = (ctypes.c_int * len(ks))(*ks); na = (ctypes.c_int * len(ns))(*ns)
    rc = load_library().gr_accept_sweep(handle, _ptr(p, torch.float32, "p"), _ptr(q, torch.float32, "q"), ka, len(ks), na, len(ns),
                                        B, V, _ptr(accept_prob, torch.float32, "accept_prob"), _ptr(status, torch.int32, "status"),
                                        _stream(stream))
    if rc != GR_OK:
        raise GrError(rc, "gr_accept_sweep")
    return accept_prob, status


def gr_accept_sweep_noalloc(p: torch.Tensor, q: torch.Tensor, ks, ns, accept_prob: torch.Tensor, status: torch.Tensor, stream=None):
    """gr_accept_sweep without a handle and without any allocation: the caller passes every buffer
    (accept_prob [B, len(ks), len(ns)] float32, status [B] int32); at most GR_NOALLOC_MAX_B rows."""
    if p.dim() != 2 or p.shape != q.shape:
        raise TypeError("gr_accept_sweep_noalloc: p and q must both be [B, V]")
    B, V = p.shape
    ks = [int(k) for k in ks]; ns = [int(n) for n in ns]
    if tuple(accept_prob.shape) != (B, len(ks), len(ns)) or tuple(status.shape) != (B,):
        raise TypeError("gr_accept_sweep_noalloc: accept_prob must be [B, len(ks), len(ns)] and status [B]")
    ka = (ctypes.c_int * len(ks))(*ks); na = (ctypes.c_int * len(ns))(*ns)
    rc = load_library().gr_accept_sweep_noalloc(_ptr(p, torch.float32, "p"), _ptr(q, torch.float32, "q"), ka, len(ks), na, len(ns),
                                                B, V, _ptr(accept_prob, torch.float32, "accept_prob"),
                                                _ptr(status, torch.int32, "status"), _stream(stream))
    if rc != GR_OK:
        raise GrError(rc, "gr_accept_sweep_noalloc")
    return accept_prob, status


def gr_tree_walk(handle: int, p: torch.Tensor, q: torch.Tensor, paths, uniforms, k: int, tol: float, temperature=None, stream=None):
    """p, q: [S, K, L, V] float32 CUDA tensors (the models' logits when `temperature`, a host array [S], is given);
    paths: [S, K, L] int32 and uniforms: [S, L] float32 host arrays (numpy).
    Returns host arrays (tokens [S, L], length [S], accepted [S], fallbacks [S])."""
    import numpy as np
    if p.dim() != 4 or p.shape != q.shape:
        raise TypeError("gr_tree_walk: p and q must both be [S, K, L, V]")
    S, K, L, V = p.shape
    paths = np.ascontiguousarray(paths, dtype=np.int32); uniforms = np.ascontiguousarray(uniforms, dtype=np.float32)
    if paths.shape != (S, K, L) or uniforms.shape != (S, L):
        raise TypeError("gr_tree_walk: paths must be [S, K, L] and uniforms [S, L]")
    tptr = None
    if temperature is not None:
        temperature = np.ascontiguousarray(temperature, dtype=np.float32)
        if temperature.shape != (S,):
            raise TypeError("gr_tree_walk: temperature must be [S]")
        tptr = temperature.ctypes.data
    tokens = np.empty((S, L), np.int32); length = np.empty(S, np.int32); accepted = np.empty(S, np.int32); fallbacks = np.empty(S, np.int32)
    rc = load_library().gr_tree_walk(handle, _ptr(p, torch.float32, "p"), _ptr(q, torch.float32, "q"), tptr, paths.ctypes.data, uniforms.ctypes.data,
                                     S, K, L, V, k, tol, tokens.ctypes.data, length.ctypes.data, accepted.ctypes.data,
                                     fallbacks.ctypes.data, _stream(stream))
    _solved_shape.pop(handle, None)
    if rc != GR_OK:
        raise GrError(rc, "gr_tree_walk")
    return tokens, length, accepted, fallbacks


def _check_drafts(handle: int, drafts: torch.Tensor, what: str, V: int | None = None) -> None:
    """The library trusts the sizes of the last solve: refuse buffers of another shape here."""
    shape = _solved_shape.get(handle)
    if shape is None:
        return                              # no solve yet: the library answers GR_ESTATE
    if drafts.dim() != 2 or tuple(drafts.shape) != shape[:2]:
        raise TypeError(f"{what}: drafts must be [B, n] = {shape[:2]} of the last gr_solve, got {tuple(drafts.shape)}")
    if V is not None and V != shape[2]:
        raise TypeError(f"{what}: V = {V} differs from the last gr_solve's {shape[2]}")


def gr_verify(handle: int, drafts: torch.Tensor, uniforms: torch.Tensor, token: torch.Tensor | None = None,
              accepted: torch.Tensor | None = None, stream=None):
    """drafts [B, n] int32, uniforms [B] float32.  Returns (token [B] int32, accepted [B] uint8)."""
    _check_drafts(handle, drafts, "gr_verify")
    B = drafts.shape[0]
    if uniforms.dim() != 1 or uniforms.shape[0] != B:
        raise TypeError("gr_verify: uniforms must be [B]")
    if token is None:
        token = torch.empty(B, dtype=torch.int32, device=drafts.device)
    if accepted is None:
        accepted = torch.empty(B, dtype=torch.uint8, device=drafts.device)
    rc = load_library().gr_verify(handle, _ptr(drafts, torch.int32, "drafts"), _ptr(uniforms, torch.float32, "uniforms"),
                                  _ptr(token, torch.int32, "token"), _ptr(accepted, torch.uint8, "accepted"), _stream(stream))
    if rc != GR_OK:
        raise GrError(rc, "gr_verify")
    return token, accepted


def gr_solve_verify(handle: int, p: torch.Tensor, q: torch.Tensor, n: int, k: int, tol: float, drafts: torch.Tensor,
                    uniforms: torch.Tensor, accept_prob: torch.Tensor | None = None, status: torch.Tensor | None = None,
                    token: torch.Tensor | None = None, accepted: torch.Tensor | None = None, stream=None):
    """gr_solve and gr_verify in one call.  Returns (accept_prob, status, token, accepted)."""
    if p.dim() != 2 or p.shape != q.shape:
        raise TypeError("gr_solve_verify: p and q must both be [B, V]")
    B, V = p.shape
    if drafts.dim() != 2 or tuple(drafts.shape) != (B, n):
        raise TypeError(f"gr_solve_verify: drafts must be [B, n] = {(B, n)}, got {tuple(drafts.shape)}")
    if uniforms.dim() != 1 or uniforms.shape[0] != B:
        raise TypeError("gr_solve_verify: uniforms must be [B]")
    dev = p.device
    accept_prob = torch.empty(B, dtype=torch.float32, device=dev) if accept_prob is None else accept_prob
    status = torch.empty(B, dtype=torch.int32, device=dev) if status is None else status
    token = torch.empty(B, dtype=torch.int32, device=dev) if token is None else token
    accepted = torch.empty(B, dtype=torch.uint8, device=dev) if accepted is None else accepted
    rc = load_library().gr_solve_verify(handle, _ptr(p, torch.float32, "p"), _ptr(q, torch.float32, "q"), n, k, tol, B, V,
                                        _ptr(drafts, torch.int32, "drafts"), _ptr(uniforms, torch.float32, "uniforms"),
                                        _ptr(accept_prob, torch.float32, "accept_prob"), _ptr(status, torch.int32, "status"),
                                        _ptr(token, torch.int32, "token"), _ptr(accepted, torch.uint8, "accepted"), _stream(stream))
    if rc != GR_OK:
        _solved_shape.pop(handle, None)
        raise GrError(rc, "gr_solve_verify")
    _solved_shape[handle] = (B, n, V)
    return accept_prob, status, token, accepted


def gr_solve_logits_verify(handle: int, target_logits: torch.Tensor, draft_logits: torch.Tensor, temperature: torch.Tensor, n: int,
                           k: int, tol: float, drafts: torch.Tensor, uniforms: torch.Tensor, accept_prob: torch.Tensor | None = None,
                           status: torch.Tensor | None = None, token: torch.Tensor | None = None,
                           accepted: torch.Tensor | None = None, stream=None, draft_temperature: torch.Tensor | None = None):
    """gr_solve_logits and gr_verify in one call.  Returns (accept_prob, status, token, accepted)."""
    if target_logits.dim() != 2 or target_logits.shape != draft_logits.shape:
        raise TypeError("gr_solve_logits_verify: target_logits and draft_logits must both be [B, V]")
    B, V = target_logits.shape
    if temperature.dim() != 1 or temperature.shape[0] != B:
        raise TypeError("gr_solve_logits_verify: temperature must be [B]")
    if draft_temperature is not None and (draft_temperature.dim() != 1 or draft_temperature.shape[0] != B):
        raise TypeError("gr_solve_logits_verify: draft_temperature must be [B]")
    if drafts.dim() != 2 or tuple(drafts.shape) != (B, n):
        raise TypeError(f"gr_solve_logits_verify: drafts must be [B, n] = {(B, n)}, got {tuple(drafts.shape)}")
    if uniforms.dim() != 1 or uniforms.shape[0] != B:
        raise TypeError("gr_solve_logits_verify: uniforms must be [B]")
    dev = target_logits.device
    accept_prob = torch.empty(B, dtype=torch.float32, device=dev) if accept_prob is None else accept_prob
    status = torch.empty(B, dtype=torch.int32, device=dev) if status is None else status
    token = torch.empty(B, dtype=torch.int32, device=dev) if token is None else token
    accepted = torch.empty(B, dtype=torch.uint8, device=dev) if accepted is None else accepted
    rc = load_library().gr_solve_logits_verify(
        handle, _ptr(target_logits, torch.float32, "target_logits"), _ptr(draft_logits, torch.float32, "draft_logits"),
        _ptr(temperature, torch.float32, "temperature"),
        None if draft_temperature is None else _ptr(draft_temperature, torch.float32, "draft_temperature"), n, k, tol, B, V,
        _ptr(drafts, torch.int32, "drafts"), _ptr(uniforms, torch.float32, "uniforms"),
        _ptr(accept_prob, torch.float32, "accept_prob"), _ptr(status, torch.int32, "status"),
        _ptr(token, torch.int32, "token"), _ptr(accepted, torch.uint8, "accepted"), _stream(stream))
    if rc != GR_OK:
        _solved_shape.pop(handle, None)
        raise GrError(rc, "gr_solve_logits_verify")
    _solved_shape[handle] = (B, n, V)
    return accept_prob, status, token, accepted


def gr_policy_slice(handle: int, drafts: torch.Tensor, V: int, stream=None):
    """Dense pi(.|drafts) [B, V] float32 and the conditional acceptance [B] float32."""
    _check_drafts(handle, drafts, "gr_policy_slice", V)
    B = drafts.shape[0]
    pi = torch.empty((B, V), dtype=torch.float32, device=drafts.device)
    acc = torch.empty(B, dtype=torch.float32, device=drafts.device)
    rc = load_library().gr_policy_slice(handle, _ptr(drafts, torch.int32, "drafts"), pi.data_ptr(), acc.data_ptr(),
                                        _stream(stream))
    if rc != GR_OK:
        raise GrError(rc, "gr_policy_slice")
    return pi, acc


def gr_profile_read(handle: int) -> dict:
    """Average per-kernel milliseconds since the last read (handle created with GR_FLAG_PROFILE)."""
    a, b, c, n = ctypes.c_double(), ctypes.c_double(), ctypes.c_double(), ctypes.c_int()
    rc = load_library().gr_profile_read(handle, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(n))
    if rc != GR_OK:
        raise GrError(rc, "gr_profile_read")
    return {"select_ms": a.value, "solve_ms": b.value, "verify_ms": c.value, "steps": n.value}


def gr_policy_export_row(handle: int, row: int, count: int, device, stream=None) -> dict:
    """The first `count` ranks of one row's policy object (works for any support size)."""
    out = {
        "order": torch.empty(count, dtype=torch.int32, device=device),
        "block": torch.empty(count, dtype=torch.int32, device=device),
        "weight": torch.empty(count, dtype=torch.float64, device=device),
        "rho": torch.empty(count, dtype=torch.float64, device=device),
    }
    rc = load_library().gr_policy_export_row(handle, row, count, *(out[k].data_ptr() for k in ("order", "block", "weight", "rho")),
                                             _stream(stream))
    if rc != GR_OK:
        raise GrError(rc, "gr_policy_export_row")
    return out


def gr_profile_stride(handle: int, stride: int) -> None:
    rc = load_library().gr_profile_stride(handle, stride)
    if rc != GR_OK:
        raise GrError(rc, "gr_profile_stride")


def gr_solve_stats(handle: int, B: int, device, stream=None) -> dict:
    """Per-row work of the last solve: evaluator calls and (nodes x active tokens) summed over them."""
    ev = torch.empty(B, dtype=torch.int32, device=device)
    nt = torch.empty(B, dtype=torch.float64, device=device)
    rc = load_library().gr_solve_stats(handle, ev.data_ptr(), nt.data_ptr(), _stream(stream))
    if rc != GR_OK:
        raise GrError(rc, "gr_solve_stats")
    return {"evaluations": ev, "node_tokens": nt}


def gr_policy_export(handle: int, B: int, device, stream=None) -> dict:
    """The per-row policy object of the last solve, as tensors (see gr_verify.h)."""
    out = {
        "order": torch.empty((B, GR_MAX_SUPPORT), dtype=torch.int32, device=device),
        "block": torch.empty((B, GR_MAX_SUPPORT), dtype=torch.int32, device=device),
        "weight": torch.empty((B, GR_MAX_SUPPORT), dtype=torch.float64, device=device),
        "rho": torch.empty((B, GR_MAX_SUPPORT), dtype=torch.float64, device=device),
        "support": torch.empty(B, dtype=torch.int32, device=device),
        "h_size": torch.empty(B, dtype=torch.int32, device=device),
        "iterations": torch.empty(B, dtype=torch.int32, device=device),
    }
    rc = load_library().gr_policy_export(handle, *(out[k].data_ptr() for k in
                                                   ("order", "block", "weight", "rho", "support", "h_size", "iterations")),
                                         _stream(stream))
    if rc != GR_OK:
        raise GrError(rc, "gr_policy_export")
    return out
