"""fp64 CPU oracle for one exact Lloyd k-means iteration (Flash-KMeans paper, Eq. 1-3).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by
the ``cpu_baseline`` leg of ``bench.py``; never by the GPU library or its binding, with
which it shares no code.  The arithmetic lives in ``lloyd_oracle.c`` (plain C, fp64,
OpenMP over points); this module only compiles it with gcc, marshals numpy arrays and
loops over batch instances and iterations.

Inputs are the *stored* values: fp16 / bf16 data are widened exactly to float32 by the
caller, fp32 and fp64 are passed as they are.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "lloyd_oracle.c"
_LIB = _HERE / "liblloyd_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile lloyd_oracle.c into liblloyd_oracle.so beside it (gcc, OpenMP)."""
    if force or (not _LIB.exists()) or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        cmd = ["gcc", "-O3", "-mavx2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-std=c11", "-o", str(tmp), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        lib.fko_num_threads.restype = ctypes.c_int
        lib.fko_assign.restype = None
        lib.fko_assign.argtypes = [vp, i32, vp, i64, i32, i32, vp, vp, vp, vp]
        lib.fko_update.restype = ctypes.c_int
        lib.fko_update.argtypes = [vp, i32, vp, vp, i64, i32, i32, vp, vp, vp]
        lib.fko_inertia.restype = ctypes.c_double
        lib.fko_inertia.argtypes = [vp, i32, vp, vp, i64, i32]
        lib.fko_pair_dist.restype = ctypes.c_double
        lib.fko_pair_dist.argtypes = [vp, i32, vp, i64, i32, i32]
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the assignment loop runs on (OpenMP default for this process)."""
    return int(_load().fko_num_threads())


def _as_x(X) -> tuple[np.ndarray, int]:
    X = np.asarray(X)
    if X.dtype == np.float64:
        return np.ascontiguousarray(X), 1
    if X.dtype in (np.float32, np.float16):
        return np.ascontiguousarray(X, dtype=np.float32), 0
    raise TypeError(f"oracle takes float16/float32/float64 arrays, got {X.dtype}")


def _p(a: np.ndarray | None):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def assign(X, C) -> dict:
    """Eq. (2) for one instance.  X [N,d], C [K,d].

    Returns dict(assign int32 [N], best, second, xnorm2 float64 [N]): the argmin with the
    lowest index on ties, its squared distance, the smallest squared distance to any other
    centroid (+inf if K == 1) and ||x_i||^2.
    """
    Xc, f64 = _as_x(X)
    Cc = np.ascontiguousarray(C, dtype=np.float64)
    N, d = Xc.shape
    K, d2 = Cc.shape
    if d != d2 or K < 1:
        raise ValueError("shape mismatch")
    a = np.empty(N, dtype=np.int32)
    best = np.empty(N, dtype=np.float64)
    second = np.empty(N, dtype=np.float64)
    xn = np.empty(N, dtype=np.float64)
    if N:
        _load().fko_assign(_p(Xc), f64, _p(Cc), N, d, K, _p(a), _p(best), _p(second), _p(xn))
    return {"assign": a, "best": best, "second": second, "xnorm2": xn}


def update(X, a, C_prev) -> dict:
    """Eq. (3) for one instance; an empty cluster keeps its row of C_prev.

    Returns dict(C float64 [K,d], counts int64 [K], sums float64 [K,d]).
    """
    Xc, f64 = _as_x(X)
    Cp = np.ascontiguousarray(C_prev, dtype=np.float64)
    av = np.ascontiguousarray(a, dtype=np.int32)
    N, d = Xc.shape
    K = Cp.shape[0]
    if av.shape != (N,) or Cp.shape[1] != d:
        raise ValueError("shape mismatch")
    Cn = np.empty_like(Cp)
    counts = np.zeros(K, dtype=np.int64)
    sums = np.zeros((K, d), dtype=np.float64)
    rc = _load().fko_update(_p(Xc), f64, _p(av), _p(Cp), N, d, K, _p(Cn), _p(counts), _p(sums))
    if rc != 0:
        raise ValueError("assignment out of range")
    return {"C": Cn, "counts": counts, "sums": sums}


def inertia(X, C, a) -> float:
    """Eq. (1): sum_i ||x_i - c_{a_i}||^2 in fp64."""
    Xc, f64 = _as_x(X)
    Cc = np.ascontiguousarray(C, dtype=np.float64)
    av = np.ascontiguousarray(a, dtype=np.int32)
    N, d = Xc.shape
    if N == 0:
        return 0.0
    return float(_load().fko_inertia(_p(Xc), f64, _p(Cc), _p(av), N, d))


def pair_dist(X, C, i: int, k: int) -> float:
    """D_ik for a single (point, centroid) pair, fp64."""
    Xc, f64 = _as_x(X)
    Cc = np.ascontiguousarray(C, dtype=np.float64)
    return float(_load().fko_pair_dist(_p(Xc), f64, _p(Cc), int(i), int(k), Xc.shape[1]))


def lloyd(X, C0, iters: int) -> dict:
    """`iters` rounds of (assign with the current C; update), free-running in fp64.

    Returns dict(C final, assign and counts of the last round, inertia: list holding,
    per round, J after the assignment step and J after the update step).
    """
    C = np.array(C0, dtype=np.float64, copy=True)
    hist = []
    a = None
    counts = None
    for _ in range(iters):
        r = assign(X, C)
        a = r["assign"]
        j_assign = float(r["best"].sum())
        u = update(X, a, C)
        C = u["C"]
        counts = u["counts"]
        hist.append((j_assign, inertia(X, C, a)))
    return {"C": C, "assign": a, "counts": counts, "inertia": hist}


def assign_batched(X, C) -> list[dict]:
    """B independent instances: X [B,N,d], C [B,K,d]."""
    return [assign(X[b], C[b]) for b in range(len(X))]


def update_batched(X, a, C_prev) -> list[dict]:
    return [update(X[b], a[b], C_prev[b]) for b in range(len(X))]
