"""Pins for the fp64 CPU oracle (no GPU, no GPU library).

The paper (Section 3.1, Eq. 1-3) prints no worked numeric example, so the oracle is pinned
to things that do not come from the oracle itself: a hand-worked integer case, exact
rational brute force, closed forms, invariants of Lloyd's algorithm and an independent
library distance routine.  Each check is aimed at a mistake someone could plausibly make in
``oracle/lloyd_oracle.c``: a transposed operand, a wrong tie rule, a dropped or doubled
term, an off-by-one in the second-best scan, a division for an empty cluster.
"""
import json
import math
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest
from scipy.spatial.distance import cdist

import oracle

GOLDEN = Path(__file__).resolve().parent / "golden"


# ----------------------------------------------------------------------------- hand-worked
def test_handworked_2d_case():
    g = json.loads((GOLDEN / "handworked_2d.json").read_text())
    X = np.array(g["X"], dtype=np.float64)
    C = np.array(g["C"], dtype=np.float64)
    for Xin in (X, X.astype(np.float32)):          # both input widths of the C code
        r = oracle.assign(Xin, C)
        assert r["assign"].tolist() == g["assign"]          # includes 2- and 3-way ties
        assert r["best"].tolist() == g["best"]
        assert r["second"].tolist() == g["second"]
        assert r["xnorm2"].tolist() == g["xnorm2"]
        u = oracle.update(Xin, r["assign"], C)
        assert u["counts"].tolist() == g["counts"]
        assert u["sums"].tolist() == g["sums"]
        assert u["C"].tolist() == g["C_new"]                # empty cluster kept (11,10)
        assert oracle.inertia(Xin, C, r["assign"]) == g["J_assign"]
        assert oracle.inertia(Xin, u["C"], r["assign"]) == g["J_update"]


def test_lloyd_driver_on_handworked_case():
    g = json.loads((GOLDEN / "handworked_2d.json").read_text())
    out = oracle.lloyd(np.array(g["X"], float), np.array(g["C"], float), 1)
    assert out["inertia"][0] == (g["J_assign"], g["J_update"])
    assert out["C"].tolist() == g["C_new"]
    assert out["counts"].tolist() == g["counts"]


# ------------------------------------------------------------------ exact rational brute force
def _exact_assign(X, C):
    """argmin_k sum_j (x_ij - c_kj)^2 in exact rational arithmetic, lowest k on ties."""
    out, dist = [], []
    for x in X:
        row = [sum((Fraction(float(xj)) - Fraction(float(cj))) ** 2 for xj, cj in zip(x, c)) for c in C]
        k = min(range(len(C)), key=lambda kk: (row[kk], kk))
        out.append(k)
        dist.append(row)
    return out, dist


@pytest.mark.parametrize("seed,N,K,d", [(0, 40, 5, 3), (1, 64, 8, 4), (2, 17, 1, 2), (3, 9, 9, 1), (4, 30, 7, 5)])
def test_assign_against_exact_rational_bruteforce(seed, N, K, d):
    rng = np.random.default_rng(seed)
    # small integers / quarters: many exact ties, all exactly representable
    X = rng.integers(-6, 7, size=(N, d)).astype(np.float64) / 4.0
    C = rng.integers(-6, 7, size=(K, d)).astype(np.float64) / 4.0
    a_ref, D = _exact_assign(X, C)
    r = oracle.assign(X, C)
    assert r["assign"].tolist() == a_ref
    for i in range(N):
        srt = sorted((D[i][k], k) for k in range(K))
        assert Fraction(r["best"][i]) == srt[0][0]
        if K > 1:
            others = [D[i][k] for k in range(K) if k != a_ref[i]]
            assert Fraction(r["second"][i]) == min(others)
        else:
            assert math.isinf(r["second"][i])
        assert Fraction(r["xnorm2"][i]) == sum(Fraction(float(v)) ** 2 for v in X[i])


def test_assign_norm_expansion_longdouble_random():
    """Second formulation (||x||^2 + ||c||^2 - 2 x.c in long double) on generic data."""
    rng = np.random.default_rng(11)
    X = rng.standard_normal((64, 4))
    C = rng.standard_normal((8, 4))
    Xl, Cl = X.astype(np.longdouble), C.astype(np.longdouble)
    D = (Xl ** 2).sum(1)[:, None] + (Cl ** 2).sum(1)[None, :] - 2 * Xl @ Cl.T
    r = oracle.assign(X, C)
    gap = np.sort(D, 1)
    clear = (gap[:, 1] - gap[:, 0]) > 1e-12
    assert clear.all()
    assert (r["assign"] == D.argmin(1)).all()
    np.testing.assert_allclose(r["best"], D.min(1).astype(np.float64), rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- library routine
@pytest.mark.parametrize("N,K,d,dt", [(500, 37, 19, np.float64), (300, 64, 33, np.float32), (257, 3, 128, np.float32)])
def test_against_scipy_cdist(N, K, d, dt):
    """Non-square, non-symmetric shapes: a transposed operand or a swapped N/K/d fails here."""
    rng = np.random.default_rng(5)
    X = (rng.standard_normal((N, d)) * 3).astype(dt)
    C = (rng.standard_normal((K, d)) * 3).astype(dt).astype(np.float64)
    D = cdist(X.astype(np.float64), C, "sqeuclidean")
    r = oracle.assign(X, C)
    assert (r["assign"] == D.argmin(1)).all()
    np.testing.assert_allclose(r["best"], D.min(1), rtol=1e-12)
    np.testing.assert_allclose(r["second"], np.sort(D, 1)[:, 1], rtol=1e-12)
    np.testing.assert_allclose(r["xnorm2"], (X.astype(np.float64) ** 2).sum(1), rtol=1e-13)
    for i, k in [(0, 0), (N - 1, K - 1), (N // 2, 1)]:
        assert oracle.pair_dist(X, C, i, k) == pytest.approx(D[i, k], rel=1e-12)
    assert oracle.inertia(X, C, r["assign"]) == pytest.approx(D.min(1).sum(), rel=1e-12)


# ----------------------------------------------------------------------------- closed forms
def test_k_equals_one_gives_global_mean():
    rng = np.random.default_rng(7)
    X = rng.standard_normal((1000, 6)).astype(np.float32)
    C0 = np.full((1, 6), 123.0)
    r = oracle.assign(X, C0)
    assert (r["assign"] == 0).all() and np.isinf(r["second"]).all()
    u = oracle.update(X, r["assign"], C0)
    exact = [math.fsum(float(v) for v in X[:, j]) / 1000 for j in range(6)]
    np.testing.assert_allclose(u["C"][0], exact, rtol=1e-13, atol=1e-15)
    assert u["counts"].tolist() == [1000]


def test_k_equals_n_identity():
    rng = np.random.default_rng(8)
    X = rng.standard_normal((50, 7))
    r = oracle.assign(X, X)
    assert r["assign"].tolist() == list(range(50))
    assert (r["best"] == 0).all()
    u = oracle.update(X, r["assign"], X + 1.0)
    assert (u["C"] == X).all() and (u["counts"] == 1).all()
    assert oracle.inertia(X, X, r["assign"]) == 0.0


def test_one_dimensional_intervals():
    """d = 1: a point belongs to the interval between midpoints of neighbouring centroids;
    a point exactly on a midpoint goes to the lower index.  Integers keep it exact."""
    c = np.array([-20.0, -6.0, 0.0, 4.0, 30.0])[:, None]
    x = np.arange(-40, 41, dtype=np.float64)[:, None]
    mid = (c[:-1, 0] + c[1:, 0]) / 2.0
    expect = np.searchsorted(mid, x[:, 0], side="left")
    r = oracle.assign(x, c)
    assert (r["assign"] == expect).all()
    # centroid order must not matter for *which* centroid wins, only ties follow the index
    perm = np.array([3, 0, 4, 2, 1])
    r2 = oracle.assign(x, c[perm])
    on_mid = np.isin(x[:, 0], mid)
    assert (perm[r2["assign"]][~on_mid] == expect[~on_mid]).all()


def test_duplicate_centroids_leave_higher_index_empty():
    rng = np.random.default_rng(9)
    X = rng.standard_normal((200, 3))
    C = rng.standard_normal((4, 3))
    C2 = np.vstack([C, C[1:2]])                     # index 4 duplicates index 1
    r = oracle.assign(X, C2)
    assert not (r["assign"] == 4).any()
    u = oracle.update(X, r["assign"], C2)
    assert u["counts"][4] == 0 and (u["C"][4] == C2[4]).all()


# ----------------------------------------------------------------------------- invariants
def _mixture(seed, N, K, d, dt=np.float32):
    rng = np.random.default_rng(seed)
    cen = rng.standard_normal((K, d)) * 4
    lab = rng.integers(0, K, N)
    X = (cen[lab] + rng.standard_normal((N, d))).astype(dt)
    C0 = X[rng.choice(N, K, replace=False)].astype(np.float64)
    return X, C0


def test_update_invariants():
    X, C0 = _mixture(21, 3000, 12, 9)
    a = oracle.assign(X, C0)["assign"]
    u = oracle.update(X, a, C0)
    assert u["counts"].sum() == len(X)
    assert (u["counts"] == np.bincount(a, minlength=12)).all()
    X64 = X.astype(np.float64)
    for k in range(12):
        np.testing.assert_allclose(u["C"][k], X64[a == k].mean(0), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose((u["counts"][:, None] * u["C"]).sum(0), X64.sum(0), rtol=1e-11)
    with pytest.raises(ValueError):
        oracle.update(X, np.full(len(X), 12, np.int32), C0)


def test_inertia_never_increases():
    X, C0 = _mixture(22, 4000, 16, 8)
    out = oracle.lloyd(X, C0, 8)
    flat = [v for pair in out["inertia"] for v in pair]
    for prev, nxt in zip(flat, flat[1:]):
        assert nxt <= prev * (1 + 1e-12)
    assert flat[-1] < flat[0]


def test_point_permutation_equivariance():
    X, C0 = _mixture(23, 1500, 10, 5, np.float64)
    p = np.random.default_rng(1).permutation(len(X))
    r, rp = oracle.assign(X, C0), oracle.assign(X[p], C0)
    assert (rp["assign"] == r["assign"][p]).all()
    u, up = oracle.update(X, r["assign"], C0), oracle.update(X[p], rp["assign"], C0)
    assert (u["counts"] == up["counts"]).all()
    np.testing.assert_allclose(u["C"], up["C"], rtol=1e-12, atol=1e-13)


def test_float32_and_float64_inputs_agree_on_same_values():
    X, C0 = _mixture(24, 800, 6, 4, np.float32)
    r32, r64 = oracle.assign(X, C0), oracle.assign(X.astype(np.float64), C0)
    assert (r32["assign"] == r64["assign"]).all()
    assert (r32["best"] == r64["best"]).all()


def test_batched_wrappers_are_independent_instances():
    Xa, Ca = _mixture(30, 300, 5, 4)
    Xb, Cb = _mixture(31, 300, 5, 4)
    rs = oracle.assign_batched(np.stack([Xa, Xb]), np.stack([Ca, Cb]))
    assert (rs[0]["assign"] == oracle.assign(Xa, Ca)["assign"]).all()
    assert (rs[1]["assign"] == oracle.assign(Xb, Cb)["assign"]).all()
    us = oracle.update_batched(np.stack([Xa, Xb]), np.stack([rs[0]["assign"], rs[1]["assign"]]),
                               np.stack([Ca, Cb]))
    assert (us[1]["C"] == oracle.update(Xb, rs[1]["assign"], Cb)["C"]).all()


def test_empty_input_and_threads():
    r = oracle.assign(np.zeros((0, 3), np.float32), np.zeros((2, 3)))
    assert r["assign"].shape == (0,)
    assert oracle.num_threads() >= 1
