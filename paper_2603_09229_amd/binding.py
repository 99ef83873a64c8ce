"""ctypes binding of libflashkm.so: same names as include/flashkm.h, argument marshalling only.

Tensors are torch tensors (device memory, streams); every step of the path runs inside the
library's HIP kernels.  There is no fallback: if the library has not been built, or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libflashkm.so"

FK_F32, FK_F16, FK_BF16 = 0, 1, 2
_DTYPE = {torch.float32: FK_F32, torch.float16: FK_F16, torch.bfloat16: FK_BF16}
_STATUS = {0: "FK_OK", 1: "FK_EINVAL", 2: "FK_EUNSUPPORTED", 3: "FK_EWORKSPACE", 4: "FK_EHIP"}

# every symbol include/flashkm.h declares
EXPORTS = ("fk_last_error", "fk_workspace_bytes", "fk_assign", "fk_sort_inverse", "fk_update",
           "fk_lloyd_iter", "fk_lloyd_ooc", "fk_ooc_workspace_bytes", "fk_stage_timer_start",
           "fk_stage_timer_stop", "fk_plan", "fk_set_option", "fk_standard_assign",
           "fk_standard_update", "fk_assign_static", "fk_assign_static_limit")
STAGES = ("assign", "sort", "reduce", "finalize")


class FlashKMError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Open libflashkm.so (built by paper_2603_09229_amd.build); fail loudly if absent."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2603_09229_amd.build` "
                "(or __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(str(LIB_PATH))
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
        L.fk_last_error.restype = ctypes.c_char_p
        L.fk_last_error.argtypes = []
        L.fk_workspace_bytes.restype = sz
        L.fk_workspace_bytes.argtypes = [i32, i64, i32, i32, i32]
        L.fk_ooc_workspace_bytes.restype = sz
        L.fk_ooc_workspace_bytes.argtypes = [i64, i32, i32, i32]
        L.fk_assign.restype = i32
        L.fk_assign.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32, vp, sz, vp]
        L.fk_assign_static.restype = i32
        L.fk_assign_static.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32, vp]
        L.fk_assign_static_limit.restype = sz
        L.fk_assign_static_limit.argtypes = []
        L.fk_sort_inverse.restype = i32
        L.fk_sort_inverse.argtypes = [vp, vp, vp, i32, i64, i32, vp, sz, vp]
        L.fk_update.restype = i32
        L.fk_update.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, i32, vp, sz, vp]
        L.fk_lloyd_iter.restype = i32
        L.fk_lloyd_iter.argtypes = [vp, vp, vp, vp, vp, i32, i64, i32, i32, i32, i32, vp, sz, vp]
        L.fk_lloyd_ooc.restype = i32
        L.fk_lloyd_ooc.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, i32, i64, vp, sz, vp]
        L.fk_standard_assign.restype = i32
        L.fk_standard_assign.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32, vp, sz, vp]
        L.fk_standard_update.restype = i32
        L.fk_standard_update.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, i32, vp]
        L.fk_plan.restype = i32
        L.fk_plan.argtypes = [i32, i64, i32, i32, i32, ctypes.c_char_p, sz]
        L.fk_set_option.restype = i32
        L.fk_set_option.argtypes = [ctypes.c_char_p, i32]
        L.fk_stage_timer_start.restype = None
        L.fk_stage_timer_start.argtypes = []
        L.fk_stage_timer_stop.restype = i32
        L.fk_stage_timer_stop.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
        _lib = L
    return _lib


def _check(status: int):
    if status != 0:
        raise FlashKMError(status, lib().fk_last_error().decode())


def _ptr(t: torch.Tensor | None):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(device) -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def _dev(t: torch.Tensor, name: str, dtype=None, shape=None) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return t


def _shape3(X: torch.Tensor, C: torch.Tensor):
    if X.dim() != 3 or C.dim() != 3 or X.shape[0] != C.shape[0] or X.shape[2] != C.shape[2]:
        raise ValueError("X must be [B,N,d] and C [B,K,d]")
    return X.shape[0], X.shape[1], X.shape[2], C.shape[1]


def fk_workspace_bytes(B: int, N: int, d: int, K: int, dtype: torch.dtype) -> int:
    return int(lib().fk_workspace_bytes(B, N, d, K, _DTYPE[dtype]))


def fk_ooc_workspace_bytes(chunk_rows: int, d: int, K: int, dtype: torch.dtype) -> int:
    return int(lib().fk_ooc_workspace_bytes(chunk_rows, d, K, _DTYPE[dtype]))


def make_workspace(B: int, N: int, d: int, K: int, dtype: torch.dtype, device) -> torch.Tensor:
    n = fk_workspace_bytes(B, N, d, K, dtype)
    if n == 0:
        raise FlashKMError(2, f"unsupported shape B={B} N={N} d={d} K={K} {dtype}")
    return torch.empty(n, dtype=torch.uint8, device=device)


def fk_assign(X, C, *, min_dist: bool = False, ws=None, out=None):
    """X [B,N,d], C [B,K,d] (same dtype) -> assign [B,N] int32 (and min_dist [B,N] float32)."""
    B, N, d, K = _shape3(X, C)
    _dev(X, "X"); _dev(C, "C", X.dtype)
    ws = ws if ws is not None else make_workspace(B, N, d, K, X.dtype, X.device)
    a = out if out is not None else torch.empty((B, N), dtype=torch.int32, device=X.device)
    _dev(a, "out", torch.int32, (B, N))
    md = torch.empty((B, N), dtype=torch.float32, device=X.device) if min_dist else None
    _check(lib().fk_assign(_ptr(X), _ptr(C), _ptr(a), _ptr(md), B, N, d, K, _DTYPE[X.dtype],
                           _ptr(ws), ws.numel(), _stream(X.device)))
    return (a, md) if min_dist else a


def fk_assign_static(X, C, *, min_dist: bool = False, out=None):
    """fk_assign without a workspace: the library's static scratch holds the centroid layout.
    The outputs are the caller's (allocated here when not passed in)."""
    B, N, d, K = _shape3(X, C)
    _dev(X, "X"); _dev(C, "C", X.dtype)
    a = out if out is not None else torch.empty((B, N), dtype=torch.int32, device=X.device)
    _dev(a, "out", torch.int32, (B, N))
    md = torch.empty((B, N), dtype=torch.float32, device=X.device) if min_dist else None
    _check(lib().fk_assign_static(_ptr(X), _ptr(C), _ptr(a), _ptr(md), B, N, d, K,
                                  _DTYPE[X.dtype], _stream(X.device)))
    return (a, md) if min_dist else a


def fk_sort_inverse(assign, K: int, *, ws=None):
    """assign [B,N] int32 -> (sorted_idx [B,N] int32, seg_offsets [B,K+1] int32)."""
    _dev(assign, "assign", torch.int32)
    B, N = assign.shape
    ws = ws if ws is not None else make_workspace(B, N, 8, K, torch.float32, assign.device)
    si = torch.empty((B, N), dtype=torch.int32, device=assign.device)
    so = torch.empty((B, K + 1), dtype=torch.int32, device=assign.device)
    _check(lib().fk_sort_inverse(_ptr(assign), _ptr(si), _ptr(so), B, N, K, _ptr(ws), ws.numel(),
                                 _stream(assign.device)))
    return si, so


def fk_update(X, assign, C_prev_f32, *, ws=None):
    """-> (C_f32 [B,K,d] float32, C_lp [B,K,d] in X's dtype, counts [B,K] int32)."""
    B, N, d, K = _shape3(X, C_prev_f32)
    _dev(X, "X"); _dev(assign, "assign", torch.int32, (B, N))
    _dev(C_prev_f32, "C_prev_f32", torch.float32)
    ws = ws if ws is not None else make_workspace(B, N, d, K, X.dtype, X.device)
    C_out = torch.empty_like(C_prev_f32)
    C_lp = torch.empty((B, K, d), dtype=X.dtype, device=X.device)
    counts = torch.empty((B, K), dtype=torch.int32, device=X.device)
    _check(lib().fk_update(_ptr(X), _ptr(assign), _ptr(C_prev_f32), _ptr(C_out), _ptr(C_lp),
                           _ptr(counts), B, N, d, K, _DTYPE[X.dtype], _ptr(ws), ws.numel(),
                           _stream(X.device)))
    return C_out, C_lp, counts


def fk_lloyd_iter(X, C_f32, iters: int, *, ws=None, C_lp=None, assign=None, counts=None):
    """`iters` Lloyd iterations in place on C_f32.  -> (assign, counts, C_lp)."""
    B, N, d, K = _shape3(X, C_f32)
    _dev(X, "X"); _dev(C_f32, "C_f32", torch.float32)
    ws = ws if ws is not None else make_workspace(B, N, d, K, X.dtype, X.device)
    if C_lp is None:
        C_lp = torch.empty((B, K, d), dtype=X.dtype, device=X.device)
    if assign is None:
        assign = torch.empty((B, N), dtype=torch.int32, device=X.device)
    if counts is None:
        counts = torch.empty((B, K), dtype=torch.int32, device=X.device)
    _dev(C_lp, "C_lp", X.dtype, (B, K, d))
    _dev(assign, "assign", torch.int32, (B, N)); _dev(counts, "counts", torch.int32, (B, K))
    _check(lib().fk_lloyd_iter(_ptr(X), _ptr(C_f32), _ptr(C_lp), _ptr(assign), _ptr(counts), B, N,
                               d, K, _DTYPE[X.dtype], iters, _ptr(ws), ws.numel(),
                               _stream(X.device)))
    return assign, counts, C_lp


def fk_lloyd_ooc(X_host, C_f32, iters: int, *, dev_ws, chunk_rows: int = 0, keep_assign=True):
    """X_host: pinned CPU tensor [N,d]; C_f32: device [K,d] float32, updated in place.

    -> (assign [N] int32 device or None, counts [K] int32 device).  Blocks until done.
    """
    if X_host.is_cuda or not X_host.is_pinned() or not X_host.is_contiguous() or X_host.dim() != 2:
        raise ValueError("X_host must be a contiguous pinned host tensor [N,d]")
    N, d = X_host.shape
    _dev(C_f32, "C_f32", torch.float32)
    if C_f32.dim() != 2 or C_f32.shape[1] != d:
        raise ValueError("C_f32 must be [K,d]")
    K = C_f32.shape[0]
    _dev(dev_ws, "dev_ws", torch.uint8)
    dev = C_f32.device
    a = torch.empty((N,), dtype=torch.int32, device=dev) if keep_assign else None
    counts = torch.empty((K,), dtype=torch.int32, device=dev)
    _check(lib().fk_lloyd_ooc(_ptr(X_host), _ptr(C_f32), _ptr(a), _ptr(counts), N, d, K,
                              _DTYPE[X_host.dtype], iters, chunk_rows, _ptr(dev_ws),
                              dev_ws.numel(), _stream(dev)))
    return a, counts


def fk_stage_timer_start() -> None:
    lib().fk_stage_timer_start()


def fk_stage_timer_stop() -> dict:
    """-> {stage: (total_ms, intervals)} for the stages recorded since the start call."""
    ms = (ctypes.c_double * 4)()
    n = (ctypes.c_int * 4)()
    rc = lib().fk_stage_timer_stop(ms, n)
    if rc < 0:
        raise FlashKMError(4, "stage timer: HIP event error")
    return {STAGES[i]: (float(ms[i]), int(n[i])) for i in range(4)}


def fk_plan(B: int, N: int, d: int, K: int, dtype: torch.dtype) -> str:
    """One-line description of the kernels and tilings chosen for this shape."""
    buf = ctypes.create_string_buffer(512)
    st = lib().fk_plan(B, N, d, K, _DTYPE[dtype], buf, len(buf))
    if st not in (0, 2):
        _check(st)
    return buf.value.decode()


def fk_set_option(name: str, value: int) -> None:
    _check(lib().fk_set_option(name.encode(), int(value)))


def fk_standard_assign(X, C, *, D=None, ws=None):
    """Comparator (paper Algorithm 1, kernels 1-2): materialises D [B,N,K] float32, then argmin.

    -> (assign [B,N] int32, D)."""
    B, N, d, K = _shape3(X, C)
    _dev(X, "X"); _dev(C, "C", X.dtype)
    ws = ws if ws is not None else make_workspace(B, N, d, K, X.dtype, X.device)
    if D is None:
        D = torch.empty((B, N, K), dtype=torch.float32, device=X.device)
    _dev(D, "D", torch.float32, (B, N, K))
    a = torch.empty((B, N), dtype=torch.int32, device=X.device)
    _check(lib().fk_standard_assign(_ptr(X), _ptr(C), _ptr(D), _ptr(a), B, N, d, K, _DTYPE[X.dtype],
                                    _ptr(ws), ws.numel(), _stream(X.device)))
    return a, D


def fk_standard_update(X, assign, C_prev_f32, *, sums=None):
    """Comparator (paper Algorithm 1, kernels 3-4): atomic scatter, then normalise.

    -> (C_f32 [B,K,d], counts [B,K] int32)."""
    B, N, d, K = _shape3(X, C_prev_f32)
    _dev(X, "X"); _dev(assign, "assign", torch.int32, (B, N))
    _dev(C_prev_f32, "C_prev_f32", torch.float32)
    if sums is None:
        sums = torch.empty((B, K, d), dtype=torch.float32, device=X.device)
    C_out = torch.empty_like(C_prev_f32)
    counts = torch.empty((B, K), dtype=torch.int32, device=X.device)
    _check(lib().fk_standard_update(_ptr(X), _ptr(assign), _ptr(C_prev_f32), _ptr(C_out),
                                    _ptr(counts), _ptr(sums), B, N, d, K, _DTYPE[X.dtype],
                                    _stream(X.device)))
    return C_out, counts
