"""Comparison rules between the GPU library and the fp64 oracle (used by the gpu tests,
smoke() and nothing else).  Tolerances:

assignments   must equal the oracle's except where the oracle's own top-2 squared-distance
              gap is below 1e-3 * (||x||^2 + ||c||^2), c being the centroid the GPU chose;
centroids     per element |gpu - ref| <= tol * max(|ref|, ||ref_k||_2 / sqrt(d)) with
              tol = 1e-3 for fp16/bf16 inputs and 1e-5 for fp32 inputs (the RMS floor keeps
              near-zero coordinates from failing on absolute noise);
counts        bit-exact (they are compared for identical assignments).
"""
from __future__ import annotations

import numpy as np
import torch

import oracle

ASSIGN_GAP = 1e-3
CENTROID_TOL = {torch.float32: 1e-5, torch.float16: 1e-3, torch.bfloat16: 1e-3}


def widen(t: torch.Tensor) -> np.ndarray:
    """Stored values of a (possibly 16-bit, possibly device) tensor as float32/float64 numpy."""
    t = t.detach().cpu()
    if t.dtype in (torch.float16, torch.bfloat16):
        t = t.to(torch.float32)
    return t.numpy()


def check_assign(X: np.ndarray, C: np.ndarray, a_gpu: np.ndarray, ref: dict | None = None) -> dict:
    """One instance.  X [N,d], C [K,d] as consumed by the kernel (widened), a_gpu [N].

    Returns counts of exact / excused mismatches; raises AssertionError on an unexcused one.
    """
    C64 = np.asarray(C, dtype=np.float64)
    K = C64.shape[0]
    assert a_gpu.min() >= 0 and a_gpu.max() < K, "assignment out of range"
    r = ref if ref is not None else oracle.assign(X, C64)
    diff = np.nonzero(r["assign"] != a_gpu)[0]
    excused = 0
    if diff.size:
        cn = (C64 ** 2).sum(1)
        g = a_gpu[diff]
        tol = ASSIGN_GAP * (r["xnorm2"][diff] + cn[g])
        gap = r["second"][diff] - r["best"][diff]
        bad = diff[gap >= tol]
        if bad.size:
            i = int(bad[0])
            raise AssertionError(
                f"{bad.size} unexcused assignment mismatches; first: point {i} gpu={a_gpu[i]} "
                f"oracle={r['assign'][i]} best={r['best'][i]:.6g} second={r['second'][i]:.6g} "
                f"tol={ASSIGN_GAP * (r['xnorm2'][i] + cn[a_gpu[i]]):.6g}")
        # stricter, reported only: how much worse than the optimum the chosen centroid is
        Xd = np.asarray(X, dtype=np.float64)[diff]
        dg = ((Xd - C64[g]) ** 2).sum(1)
        assert (dg - r["best"][diff] < tol).all(), "GPU choice is farther than the tolerance allows"
        excused = int(diff.size)
    return {"n": int(a_gpu.size), "mismatch": int(diff.size), "excused": excused}


def check_centroids(C_gpu: np.ndarray, C_ref: np.ndarray, tol: float, what: str = "centroids"):
    C_ref = np.asarray(C_ref, dtype=np.float64)
    C_gpu = np.asarray(C_gpu, dtype=np.float64)
    d = C_ref.shape[-1]
    floor = np.sqrt((C_ref ** 2).sum(-1, keepdims=True) / d)
    bound = tol * np.maximum(np.abs(C_ref), floor)
    err = np.abs(C_gpu - C_ref)
    if not (err <= bound).all():
        w = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: element {w} gpu={C_gpu[w]!r} ref={C_ref[w]!r} "
                             f"err={err[w]:.3g} bound={bound[w]:.3g}")


def check_update(X: np.ndarray, a: np.ndarray, C_prev: np.ndarray, C_gpu: np.ndarray,
                 counts_gpu: np.ndarray, tol: float) -> None:
    """One instance: the update computed from the SAME assignments must match Eq. (3)."""
    u = oracle.update(X, a, np.asarray(C_prev, dtype=np.float64))
    assert (counts_gpu.astype(np.int64) == u["counts"]).all(), "counts differ"
    check_centroids(C_gpu, u["C"], tol)
    empty = u["counts"] == 0
    if empty.any():   # kept rows must be bit-identical to the previous fp32 master
        assert (np.asarray(C_gpu)[empty] == np.asarray(C_prev)[empty]).all(), "empty cluster moved"
