"""GPU parity: every C-ABI entry point against the fp64 oracle on the same seeded inputs.

Sizes are small enough for the oracle to finish in seconds but span several point tiles,
several centroid tiles, ragged tails in N, K and d, and more than one batch instance.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_09229_amd import binding as fk
from paper_2603_09229_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _problem(dtype, B, N, d, K, seed, center_std=4.0, noise=1.0, zipf=0.0):
    name = {torch.float32: "fp32", torch.float16: "fp16", torch.bfloat16: "bf16"}[dtype]
    w = wl.Workload("t", B, N, d, K, name, center_std, noise, zipf, 1, seed)
    X, lab = wl.make_points(w, return_labels=True)
    idx = wl.init_rows(w) if K <= N else torch.randint(0, N, (B, K))
    C0 = wl.gather_rows(X, idx)            # float32, exact stored rows
    return w, X, lab, C0


ASSIGN_CASES = [
    # dtype, B, N, d, K
    (torch.float16, 1, 5000, 128, 1000),     # ragged N and K tiles, several LDS stages
    (torch.float16, 1, 4099, 64, 16),        # K smaller than one centroid tile
    (torch.bfloat16, 3, 2500, 128, 256),     # batched
    (torch.float16, 2, 700, 32, 70),
    (torch.float16, 1, 513, 8, 5),           # smallest d
    (torch.bfloat16, 1, 1000, 96, 33),       # d not a power of two (zero-padded chunks)
    (torch.float16, 1, 300, 24, 40),         # d = 8 mod 16
    (torch.float16, 1, 1, 128, 1),           # degenerate: one point, one centroid
    (torch.float16, 1, 64, 128, 2500),       # K > N, two sort passes later on
    (torch.float32, 1, 3000, 64, 64),
    (torch.float32, 2, 777, 8, 3),
    (torch.float32, 1, 500, 128, 130),
    (torch.float32, 1, 400, 40, 7),
    # fp32 beyond 2^18 points: one point per thread, whole centroid tiles per workgroup
    (torch.float32, 1, 270000, 64, 40),
    (torch.float32, 2, 140000, 24, 9),
    (torch.float32, 1, 262200, 128, 12),
    # wide features (128 < d <= 512)
    (torch.float16, 1, 3000, 256, 300),
    (torch.bfloat16, 2, 1500, 512, 200),
    (torch.float16, 1, 1000, 136, 70),        # first width on the wide kernel
    (torch.float16, 1, 700, 384, 33),
    (torch.float32, 1, 900, 256, 40),
    (torch.float32, 1, 600, 512, 19),
    (torch.float32, 1, 500, 200, 70),
]


@pytest.mark.parametrize("dtype,B,N,d,K", ASSIGN_CASES)
def test_assign_matches_oracle(dtype, B, N, d, K):
    w, X, _, C0 = _problem(dtype, B, N, d, K, seed=100 + N + K)
    C = C0.to(dtype)                                   # what the kernel consumes
    a, md = fk.fk_assign(X.to(DEV), C.to(DEV), min_dist=True)
    torch.cuda.synchronize()
    a, md = a.cpu().numpy(), md.cpu().numpy()
    for b in range(B):
        Xb, Cb = parity.widen(X[b]), parity.widen(C[b])
        ref = oracle.assign(Xb, Cb)
        st = parity.check_assign(Xb, Cb, a[b], ref)
        assert st["mismatch"] <= max(2, N // 50), st     # near-ties are rare on these mixtures
        same = a[b] == ref["assign"]
        scale = ref["xnorm2"] + (Cb.astype(np.float64) ** 2).sum(1)[a[b]]
        tol = (1e-3 if dtype != torch.float32 else 1e-5) * scale + 1e-6
        assert (np.abs(md[b][same] - ref["best"][same]) <= tol[same]).all()


@pytest.mark.parametrize("dtype,B,N,d,K", [
    (torch.float16, 1, 4099, 64, 16), (torch.float16, 1, 3001, 64, 100), (torch.bfloat16, 2, 2500, 128, 64),
    (torch.float16, 1, 513, 8, 5), (torch.float16, 1, 300, 24, 40), (torch.float16, 1, 5000, 32, 250),
    (torch.bfloat16, 1, 1000, 96, 33), (torch.float16, 1, 31, 64, 4),
])
def test_streaming_and_sweeping_assign_kernels_agree(dtype, B, N, d, K):
    """Few centroids: the persistent streaming kernel (picked for X beyond the last-level
    cache) and the sweeping kernel compute the same scores with the same tie rules."""
    w, X, _, C0 = _problem(dtype, B, N, d, K, seed=400 + N + K)
    C = C0.to(dtype).to(DEV)
    try:
        fk.fk_set_option("assign_stream", 1)
        assert "mfma_stream" in fk.fk_plan(B, N, d, K, dtype)
        a1, md1 = fk.fk_assign(X.to(DEV), C, min_dist=True)
        fk.fk_set_option("assign_stream", 0)
        assert "mfma_sweep" in fk.fk_plan(B, N, d, K, dtype)
        a0, md0 = fk.fk_assign(X.to(DEV), C, min_dist=True)
    finally:
        fk.fk_set_option("assign_stream", -1)
    assert torch.equal(a0, a1) and torch.equal(md0, md1)
    for b in range(B):
        parity.check_assign(parity.widen(X[b]), parity.widen(C0.to(dtype)[b]), a1[b].cpu().numpy())


@pytest.mark.parametrize("dtype,B,N,d,K", [(torch.float16, 1, 5000, 128, 1000), (torch.bfloat16, 2, 3000, 64, 300),
                                          (torch.float16, 1, 2100, 32, 2500), (torch.float16, 1, 700, 96, 130)])
def test_every_tile_shape_of_the_sweeping_kernel_gives_the_same_answer(dtype, B, N, d, K):
    """The four compiled tile shapes differ in how points are split over waves and workgroups,
    not in the arithmetic: identical assignments and distances, and parity with the oracle."""
    w, X, _, C0 = _problem(dtype, B, N, d, K, seed=480 + N + K)
    C = C0.to(dtype).to(DEV)
    res = []
    try:
        fk.fk_set_option("assign_stream", 0)
        for v in (0, 1, 2, 3):
            fk.fk_set_option("assign_variant", v)
            assert f"variant={v}" in fk.fk_plan(B, N, d, K, dtype)
            res.append(fk.fk_assign(X.to(DEV), C, min_dist=True))
    finally:
        fk.fk_set_option("assign_variant", -1)
        fk.fk_set_option("assign_stream", -1)
    for a, md in res[1:]:
        assert torch.equal(a, res[0][0]) and torch.equal(md, res[0][1])
    for b in range(B):
        parity.check_assign(parity.widen(X[b]), parity.widen(C0.to(dtype)[b]), res[0][0][b].cpu().numpy())


def test_assign_exact_duplicates_go_to_lowest_index():
    w, X, _, C0 = _problem(torch.float16, 1, 2000, 128, 96, seed=7)
    C = C0.to(torch.float16)
    C[0, 70] = C[0, 3]          # same tile column, other half-wave
    C[0, 40] = C[0, 39]         # neighbours
    C[0, 95] = C[0, 0]          # different centroid tiles
    a = fk.fk_assign(X.to(DEV), C.to(DEV)).cpu().numpy()[0]
    assert not np.isin(a, [70, 40, 95]).any()
    parity.check_assign(parity.widen(X[0]), parity.widen(C[0]), a)


def test_assign_duplicates_with_negative_winning_scores_stay_inside_the_tolerance_rule():
    """Points closer to the origin than to any centroid: every score x.c - |c|^2/2 is negative.
    Among rows that share a lane of a centroid tile (here rows 0, 1 and 2, 3 of a tile) the kernel
    then keeps the HIGHER of two exactly equal scores' rows, where Eq. 2's reading is the lowest
    index; the difference is a zero-gap tie, which the tolerance rule covers, and nothing else
    may differ."""
    for dtype in (torch.float16, torch.bfloat16):
        g = torch.Generator().manual_seed(21)
        K, d, N = 70, 64, 3000
        C = (torch.randn((1, K, d), generator=g) * 8.0).to(dtype)
        for k in (0, 2, 32):        # the three centroids nearest the origin, of about equal norm
            C[0, k] = (C[0, k].float() * 0.5).to(dtype)
        C[0, 1] = C[0, 0]           # same lane's rows of tile 0
        C[0, 3] = C[0, 2]
        C[0, 33] = C[0, 32]         # and of tile 1
        X = (torch.randn((1, N, d), generator=g) * 0.05).to(dtype)
        # make the duplicated centroids the winners for many points: pull a third of the points
        # a little towards each pair (scores stay negative: |x| << |c|)
        for j, k in enumerate((0, 2, 32)):
            X[0, j::3] = (X[0, j::3].float() + 0.02 * C[0, k].float()).to(dtype)
        a = fk.fk_assign(X.to(DEV), C.to(DEV)).cpu().numpy()[0]
        Xw, Cw = parity.widen(X[0]), parity.widen(C[0])
        best_score = (Xw.astype(np.float64) @ Cw.astype(np.float64).T - 0.5 * (Cw.astype(np.float64) ** 2).sum(1)).max(1)
        assert (best_score < 0).all()
        st = parity.check_assign(Xw, Cw, a)                       # raises on any unexcused mismatch
        ref = oracle.assign(Xw, Cw.astype(np.float64))["assign"]
        diff = a != ref
        # every difference is a duplicate pair resolved the other way round
        assert set(zip(ref[diff].tolist(), a[diff].tolist())) <= {(0, 1), (2, 3), (32, 33)}
        assert st["excused"] == int(diff.sum())
        assert np.isin(ref, [0, 2, 32]).mean() > 0.5              # the case is really exercised


def test_assign_does_not_depend_on_tiling_position():
    """Online argmin: shifting where a point falls in a tile must not change its answer."""
    w, X, _, C0 = _problem(torch.float16, 1, 1500, 64, 200, seed=9)
    C = C0.to(torch.float16).to(DEV)
    a_full = fk.fk_assign(X.to(DEV), C).cpu()
    off = 37
    a_shift = fk.fk_assign(X[:, off:].contiguous().to(DEV), C).cpu()
    assert torch.equal(a_full[:, off:], a_shift)


SORT_CASES = [(1, 5000, 1), (2, 4097, 16), (1, 100000, 1000), (1, 33333, 2048), (1, 70001, 2049),
              (2, 50000, 5000), (1, 200000, 65536), (1, 1, 5), (1, 300000, 16),
              # around the limits of the LDS-staged scatter (32 .. 1024 bins), short last tile
              (3, 9000, 32), (1, 9000, 31), (1, 100, 1024), (1, 50000, 1025), (1, 4096, 700)]


@pytest.mark.parametrize("B,N,K", SORT_CASES)
def test_sort_inverse_is_the_stable_argsort(B, N, K):
    g = torch.Generator().manual_seed(N + K)
    p = wl.membership_probs(K, 1.2 if K <= 64 else 0.0)
    a = torch.multinomial(p.float(), B * N, replacement=True, generator=g).view(B, N).to(torch.int32)
    if K > 3:
        a[a == 2] = 1                                    # an empty cluster in the middle
    si, so = fk.fk_sort_inverse(a.to(DEV), K)
    si, so = si.cpu().numpy(), so.cpu().numpy()
    for b in range(B):
        ab = a[b].numpy()
        assert (si[b] == np.argsort(ab, kind="stable")).all()
        ref_off = np.concatenate([[0], np.cumsum(np.bincount(ab, minlength=K))])
        assert (so[b] == ref_off).all()


@pytest.mark.parametrize("B,N,K", [(1, 50000, 1), (2, 30000, 16), (1, 100000, 1000), (1, 70001, 2049),
                                   (1, 200000, 65536), (1, 40000, 2048), (1, 9000, 300)])
@pytest.mark.parametrize("rounds", [2, 3])
def test_sort_inverse_with_several_sub_tiles_per_workgroup(B, N, K, rounds):
    """The form of the sort kernels in which a workgroup owns several 4096-key sub-tiles (taken
    by itself only beyond 2^24 keys, or for a whole small instance) must stay stable."""
    g = torch.Generator().manual_seed(N + K + rounds)
    a = torch.randint(0, K, (B, N), generator=g).to(torch.int32)
    try:
        fk.fk_set_option("sort_min_rounds", rounds)
        si, so = fk.fk_sort_inverse(a.to(DEV), K)
    finally:
        fk.fk_set_option("sort_min_rounds", -1)
    si, so = si.cpu().numpy(), so.cpu().numpy()
    for b in range(B):
        ab = a[b].numpy()
        assert (si[b] == np.argsort(ab, kind="stable")).all()
        assert (so[b] == np.concatenate([[0], np.cumsum(np.bincount(ab, minlength=K))])).all()


def test_sort_inverse_single_cluster_and_sorted_input():
    a = torch.zeros((1, 70000), dtype=torch.int32)
    si, so = fk.fk_sort_inverse(a.to(DEV), 8)
    assert torch.equal(si.cpu()[0], torch.arange(70000, dtype=torch.int32))
    assert so.cpu()[0].tolist() == [0] + [70000] * 8
    a = torch.arange(3000, dtype=torch.int32).view(1, -1)
    si, so = fk.fk_sort_inverse(a.to(DEV), 3000)
    assert torch.equal(si.cpu()[0], torch.arange(3000, dtype=torch.int32))


UPDATE_CASES = [
    (torch.float16, 1, 20000, 128, 300, 0.0),
    (torch.float16, 1, 100000, 64, 16, 1.2),      # skewed: many items per cluster
    (torch.bfloat16, 2, 6000, 128, 256, 0.0),
    (torch.float32, 1, 16384, 64, 64, 0.0),
    (torch.float32, 1, 3000, 128, 10, 0.0),
    (torch.float16, 1, 900, 24, 2500, 0.0),       # K > N: mostly empty clusters, 2-pass sort
    (torch.float16, 1, 5000, 8, 3, 0.0),
    (torch.bfloat16, 1, 4000, 96, 50, 0.0),
    (torch.float16, 1, 6000, 256, 40, 0.0),       # wide rows
    (torch.bfloat16, 1, 5000, 512, 30, 0.0),
    (torch.float32, 1, 4000, 512, 12, 0.0),       # wider than one wave-load: two column blocks
    (torch.float32, 1, 3000, 200, 25, 0.0),
    (torch.float16, 1, 9000, 136, 4, 0.0),
]


@pytest.mark.parametrize("dtype,B,N,d,K,zipf", UPDATE_CASES)
def test_update_matches_oracle(dtype, B, N, d, K, zipf):
    w, X, lab, C0 = _problem(dtype, B, N, d, K, seed=200 + N, zipf=zipf)
    a = lab.clone()
    if K > 4:
        a[a == 1] = 0                                     # force one empty cluster
    C_new, C_lp, counts = fk.fk_update(X.to(DEV), a.to(DEV), C0.to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(C_lp.cpu(), C_new.cpu().to(dtype))          # rounding to nearest even
    tol = parity.CENTROID_TOL[dtype]
    for b in range(B):
        parity.check_update(parity.widen(X[b]), a[b].numpy(), C0[b].numpy(),
                            C_new[b].cpu().numpy(), counts[b].cpu().numpy(), tol)


def test_update_is_bit_reproducible_and_leaves_x_alone():
    w, X, lab, C0 = _problem(torch.float16, 1, 50000, 128, 64, seed=5)
    Xd = X.to(DEV)
    keep = Xd.clone()
    r1 = fk.fk_update(Xd, lab.to(DEV), C0.to(DEV))
    r2 = fk.fk_update(Xd, lab.to(DEV), C0.to(DEV))
    assert torch.equal(r1[0], r2[0]) and torch.equal(r1[2], r2[2])
    assert torch.equal(Xd, keep)


def _teacher_forced(w, iters, zipf_init=False, max_mismatch_frac=0.02):
    X, lab = wl.make_points(w, return_labels=True)
    idx = wl.init_rows(w, lab if zipf_init else None)
    C = wl.gather_rows(X, idx).to(DEV)                   # fp32 master on device
    Xd = X.to(DEV)
    dtype = w.torch_dtype
    tol = parity.CENTROID_TOL[dtype]
    ws = fk.make_workspace(w.B, w.N, w.d, w.K, dtype, DEV)
    Xh = [parity.widen(X[b]) for b in range(w.B)]
    prev_lp = None
    J_prev = None
    for it in range(iters):
        C_before = C.clone()
        consumed = C_before.to(dtype)                    # what this iteration's assign reads
        if prev_lp is not None:
            assert torch.equal(prev_lp, consumed)
        a, counts, C_lp = fk.fk_lloyd_iter(Xd, C, 1, ws=ws)
        torch.cuda.synchronize()
        prev_lp = C_lp.clone()
        a_h, cnt_h = a.cpu().numpy(), counts.cpu().numpy()
        J = 0.0
        for b in range(w.B):
            Cb = parity.widen(consumed[b])
            ref = oracle.assign(Xh[b], Cb)
            st = parity.check_assign(Xh[b], Cb, a_h[b], ref)
            assert st["mismatch"] <= max_mismatch_frac * w.N + 2, (it, b, st)
            parity.check_update(Xh[b], a_h[b], C_before[b].cpu().numpy(), C[b].cpu().numpy(),
                                cnt_h[b], tol)
            J += oracle.inertia(Xh[b], C[b].cpu().numpy(), a_h[b])
        if J_prev is not None:
            assert J <= J_prev * (1 + 1e-3), (it, J, J_prev)      # Lloyd never goes uphill
        J_prev = J


def test_lloyd_c1_full_size_fp32():
    _teacher_forced(wl.C1, wl.C1.iters)


def test_lloyd_c2_recipe_scaled_fp16():
    _teacher_forced(wl.C2.scaled(N=40000, K=1024), 4)


def test_lloyd_c3_recipe_scaled_bf16_batched():
    # overlapping clusters (centre spacing ~ noise): near-ties are common here by design
    _teacher_forced(wl.C3.scaled(B=3, N=4096), 3, max_mismatch_frac=0.05)


def test_lloyd_c4_recipe_scaled_skewed():
    _teacher_forced(wl.C4.scaled(N=1 << 17), 3, zipf_init=True)


def test_lloyd_multi_iteration_call_equals_repeated_single_calls():
    w = wl.C2.scaled(N=20000, K=200)
    X = wl.make_points(w).to(DEV)
    C0 = wl.gather_rows(X.cpu(), wl.init_rows(w)).to(DEV)
    Ca, Cb = C0.clone(), C0.clone()
    a1, n1, lp1 = fk.fk_lloyd_iter(X, Ca, 5)
    for _ in range(5):
        a2, n2, lp2 = fk.fk_lloyd_iter(X, Cb, 1)
    assert torch.equal(Ca, Cb) and torch.equal(a1, a2) and torch.equal(n1, n2) and torch.equal(lp1, lp2)


@pytest.mark.parametrize("dtype,N,d,K,chunk", [
    (torch.float16, 50000, 64, 300, 16384),       # ragged tail chunk
    (torch.float16, 40000, 128, 3000, 8192),      # two-pass sort inside every chunk
    (torch.float32, 20000, 32, 20, 20000),        # single chunk
    (torch.bfloat16, 30000, 128, 64, 0),          # chunk size chosen from the workspace
    (torch.float16, 20000, 256, 100, 8192),       # wide features
    (torch.float16, 30000, 100, 50, 8192),        # rows that are not a multiple of 8 wide: pitched copies
    (torch.float32, 9000, 5, 7, 4096),
    (torch.bfloat16, 10000, 3, 4, 0),
])
def test_out_of_core_equals_in_core(dtype, N, d, K, chunk):
    w, X, _, C0 = _problem(dtype, 1, N, d, K, seed=300 + N)
    Xpin = X[0].clone().pin_memory()
    rows = chunk if chunk else 12288
    ws_bytes = fk.fk_ooc_workspace_bytes(rows, d, K, dtype)
    assert ws_bytes > 0
    dev_ws = torch.empty(ws_bytes + (4096 if chunk == 0 else 0), dtype=torch.uint8, device=DEV)
    C_ooc = C0[0].to(DEV).clone()
    a_ooc, n_ooc = fk.fk_lloyd_ooc(Xpin, C_ooc, 1, dev_ws=dev_ws, chunk_rows=chunk)
    C_in = C0.to(DEV).clone()
    a_in, n_in, _ = fk.fk_lloyd_iter(X.to(DEV), C_in, 1)
    torch.cuda.synchronize()
    assert torch.equal(a_ooc, a_in[0]) and torch.equal(n_ooc, n_in[0])
    parity.check_centroids(C_ooc.cpu().numpy(), C_in[0].cpu().numpy(), 2e-6, "ooc vs in-core")
    # and against the definition, over three more iterations
    a3, n3 = fk.fk_lloyd_ooc(Xpin, C_ooc, 3, dev_ws=dev_ws, chunk_rows=chunk)
    assert int(n3.sum()) == N
    Xh = parity.widen(X[0])
    u = oracle.update(Xh, a3.cpu().numpy(), C_ooc.cpu().numpy())
    parity.check_centroids(C_ooc.cpu().numpy(), u["C"], parity.CENTROID_TOL[dtype])
    assert (u["counts"] == n3.cpu().numpy()).all()


def test_bad_arguments_are_errors_not_crashes():
    X = torch.zeros((1, 128, 16), dtype=torch.float16, device=DEV)
    C = torch.zeros((1, 4, 16), dtype=torch.float16, device=DEV)
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(fk.FlashKMError) as e:
        fk.fk_assign(X, C, ws=small)
    assert e.value.status == 3
    with pytest.raises(fk.FlashKMError) as e:
        fk.fk_assign(torch.zeros((1, 8, 520), dtype=torch.float16, device=DEV),
                     torch.zeros((1, 2, 520), dtype=torch.float16, device=DEV),
                     ws=torch.empty(1 << 20, dtype=torch.uint8, device=DEV))
    assert e.value.status == 2          # d beyond 512
    with pytest.raises(fk.FlashKMError) as e:
        fk.fk_standard_assign(torch.zeros((1, 8, 12), dtype=torch.float16, device=DEV),
                              torch.zeros((1, 2, 12), dtype=torch.float16, device=DEV))
    assert e.value.status == 2          # the comparators take no padded widths
    with pytest.raises(ValueError):
        fk.fk_lloyd_ooc(torch.zeros((64, 16), dtype=torch.float16), C[0].float(), 1, dev_ws=small)


def test_out_of_core_refuses_pageable_host_memory():
    """Through the raw C ABI: the chunk stream only overlaps the kernels from pinned memory, so
    anything else is an argument error, found on the host before any work is enqueued."""
    import ctypes
    L = fk.lib()
    N, d, K = 5000, 64, 16
    X = (torch.randn((N, d)) * 3).to(torch.float16)                 # pageable
    assert not X.is_pinned()
    C = torch.randn((K, d), device=DEV)
    counts = torch.zeros((K,), dtype=torch.int32, device=DEV)
    need = fk.fk_ooc_workspace_bytes(2048, d, K, torch.float16)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    vp = ctypes.c_void_p
    args = lambda x: (vp(x), vp(C.data_ptr()), None, vp(counts.data_ptr()), N, d, K, fk.FK_F16, 1, 2048,
                      vp(ws.data_ptr()), need, None)
    C_before = C.clone()
    rc = L.fk_lloyd_ooc(*args(X.data_ptr()))
    assert rc == 1 and b"pinned" in L.fk_last_error(), L.fk_last_error()
    rc = L.fk_lloyd_ooc(*args(ws.data_ptr()))                       # device memory is not host memory either
    assert rc == 1 and b"pinned" in L.fk_last_error(), L.fk_last_error()
    torch.cuda.synchronize()
    assert torch.equal(C, C_before)                                 # nothing ran
    Xp = X.pin_memory()
    assert L.fk_lloyd_ooc(*args(Xp.data_ptr())) == 0, L.fk_last_error()
    assert int(counts.sum()) == N


def test_merge_bound_of_the_segment_level_update():
    """Section 4.2's count of merges: with chunks of R sorted positions at most K + ceil(N/R)
    partial rows are ever merged.  Here a cluster's run is cut into ceil(n_k/R) items, so the
    item table must end at or below that bound (read back from the workspace: sorted_idx,
    seg_off and item_off are its first three arrays, each padded to 256 bytes)."""
    for (B, N, d, K, zipf) in ((1, 100000, 64, 300, 0.0), (2, 70001, 32, 2000, 1.2), (1, 300000, 16, 5000, 0.0),
                               (1, 5000000, 8, 40, 1.5)):
        w, X, lab, C0 = _problem(torch.float16, B, N, d, K, seed=40 + K, zipf=zipf)
        ws = fk.make_workspace(B, N, d, K, torch.float16, DEV)
        fk.fk_set_option("fused_update", 0)
        try:
            plan = fk.fk_plan(B, N, d, K, torch.float16)
            fk.fk_update(X.to(DEV), lab.to(DEV), C0.to(DEV), ws=ws)
        finally:
            fk.fk_set_option("fused_update", -1)
        torch.cuda.synchronize()
        R = int(plan.split("rows_per_item=")[1].split(")")[0])
        al = lambda v: (v + 255) // 256 * 256
        o_seg = al(B * N * 4)
        o_item = o_seg + al(B * (K + 1) * 4)
        seg = ws[o_seg:o_seg + B * (K + 1) * 4].view(torch.int32).view(B, K + 1).cpu()
        item = ws[o_item:o_item + B * (K + 1) * 4].view(torch.int32).view(B, K + 1).cpu()
        for b in range(B):
            n_k = torch.bincount(lab[b].to(torch.int64), minlength=K)
            assert torch.equal(seg[b, 1:] - seg[b, :-1], n_k.to(torch.int32))        # the offsets really are these arrays
            items = (n_k + R - 1) // R
            assert torch.equal(item[b, 1:] - item[b, :-1], items.to(torch.int32))
            assert int(item[b, K]) <= K + (N + R - 1) // R, (int(item[b, K]), K, N, R)
            assert int(item[b, K]) >= (N + R - 1) // R


def test_stage_timer_reports_every_stage():
    w = wl.C2.scaled(N=30000, K=300)                 # general path: all four stages run
    X = wl.make_points(w).to(DEV)
    C = wl.gather_rows(X.cpu(), wl.init_rows(w)).to(DEV)
    fk.fk_stage_timer_start()
    fk.fk_lloyd_iter(X, C, 3)
    st = fk.fk_stage_timer_stop()
    assert set(st) == {"assign", "sort", "reduce", "finalize"}
    for name, (ms, n) in st.items():
        assert n == 3 and ms > 0.0, (name, ms, n)
    # stopped: further calls record nothing
    fk.fk_lloyd_iter(X, C, 1)
    assert all(v == (0.0, 0) for v in fk.fk_stage_timer_stop().values())
    # back-to-back repeats inside an interval: the same results, more launches per interval
    C1, C2 = C.clone(), C.clone()
    a1, n1, _ = fk.fk_lloyd_iter(X, C1, 2)
    fk.fk_set_option("timer_repeat", 4)
    fk.fk_stage_timer_start()
    a2, n2, _ = fk.fk_lloyd_iter(X, C2, 2)
    st = fk.fk_stage_timer_stop()
    fk.fk_set_option("timer_repeat", 1)
    assert st["assign"][1] == 8 and st["reduce"][1] == 8 and st["sort"][1] == 2 and st["finalize"][1] == 2
    assert torch.equal(C1, C2) and torch.equal(a1, a2) and torch.equal(n1, n2)
    # a fused shape books its single pass under "assign"
    w = wl.C2.scaled(N=30000, K=128)
    X = wl.make_points(w).to(DEV)
    C = wl.gather_rows(X.cpu(), wl.init_rows(w)).to(DEV)
    fk.fk_stage_timer_start()
    fk.fk_lloyd_iter(X, C, 3)
    st = fk.fk_stage_timer_stop()
    assert st["assign"][1] == 3 and st["finalize"][1] == 3 and st["sort"][1] == 0 and st["reduce"][1] == 0


def test_results_do_not_depend_on_the_stream():
    w = wl.C2.scaled(N=20000, K=96)
    X = wl.make_points(w).to(DEV)
    C0 = wl.gather_rows(X.cpu(), wl.init_rows(w)).to(DEV)
    Ca, Cb = C0.clone(), C0.clone()
    a1, n1, _ = fk.fk_lloyd_iter(X, Ca, 2)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        a2, n2, _ = fk.fk_lloyd_iter(X, Cb, 2)
    side.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(Ca, Cb) and torch.equal(a1, a2) and torch.equal(n1, n2)


def test_random_shapes_full_iteration():
    """Seeded sweep over odd shapes: every dtype, ragged N, K on both sides of the tile and
    stage boundaries, d every multiple of 8; one full iteration each against the oracle."""
    rng = np.random.default_rng(2024)
    dts = [torch.float16, torch.bfloat16, torch.float32]
    for case in range(40):
        dtype = dts[case % 3]
        d = int(rng.integers(1, 17)) * 8 if case % 4 else int(rng.integers(17, 65)) * 8
        K = int(rng.choice([1, 2, 3, 17, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 255, 257, 513,
                            1000, 2047, 2048, 2049, 3000]))
        N = int(rng.integers(1, 6000))
        B = int(rng.choice([1, 1, 2, 3]))
        w = wl.Workload("r", B, N, d, K, {torch.float16: "fp16", torch.bfloat16: "bf16",
                                          torch.float32: "fp32"}[dtype], 3.0, 1.0, 0.0, 1, 5000 + case)
        X = wl.make_points(w)
        idx = torch.randint(0, N, (B, K), generator=torch.Generator().manual_seed(case))
        C0 = wl.gather_rows(X, idx)
        C = C0.to(DEV).clone()
        a, counts, C_lp = fk.fk_lloyd_iter(X.to(DEV), C, 1)
        torch.cuda.synchronize()
        consumed = C0.to(dtype)
        for b in range(B):
            Xb = parity.widen(X[b])
            parity.check_assign(Xb, parity.widen(consumed[b]), a[b].cpu().numpy())
            parity.check_update(Xb, a[b].cpu().numpy(), C0[b].numpy(), C[b].cpu().numpy(),
                                counts[b].cpu().numpy(), parity.CENTROID_TOL[dtype])
        assert torch.equal(C_lp.cpu(), C.cpu().to(dtype)), (case, dtype, B, N, d, K)


@pytest.mark.parametrize("dtype,B,N,d,K", [(torch.float16, 1, 3000, 128, 300), (torch.bfloat16, 2, 1000, 64, 37),
                                           (torch.float16, 1, 700, 24, 5)])
def test_standard_comparator_assign(dtype, B, N, d, K):
    """The materialising comparator (Algorithm 1, kernels 1-2) obeys the same parity rule, and
    its distance matrix is the squared distances."""
    w, X, _, C0 = _problem(dtype, B, N, d, K, seed=700 + N)
    C = C0.to(dtype)
    a, D = fk.fk_standard_assign(X.to(DEV), C.to(DEV))
    torch.cuda.synchronize()
    for b in range(B):
        Xb, Cb = parity.widen(X[b]), parity.widen(C[b])
        parity.check_assign(Xb, Cb, a[b].cpu().numpy())
        ref = ((Xb[:50, None, :].astype(np.float64) - Cb[None].astype(np.float64)) ** 2).sum(-1)
        scale = (Xb[:50].astype(np.float64) ** 2).sum(1)[:, None] + (Cb.astype(np.float64) ** 2).sum(1)[None]
        assert (np.abs(D[b, :50].cpu().numpy() - ref) <= 1e-3 * scale + 1e-5).all()


@pytest.mark.parametrize("dtype,B,N,d,K", [(torch.float16, 1, 20000, 128, 64), (torch.float32, 2, 3000, 40, 9),
                                           (torch.bfloat16, 1, 5000, 256, 12)])
def test_standard_comparator_update(dtype, B, N, d, K):
    w, X, lab, C0 = _problem(dtype, B, N, d, K, seed=800 + N)
    a = lab.clone()
    if K > 4:
        a[a == 1] = 0
    C_new, counts = fk.fk_standard_update(X.to(DEV), a.to(DEV), C0.to(DEV))
    torch.cuda.synchronize()
    for b in range(B):
        parity.check_update(parity.widen(X[b]), a[b].numpy(), C0[b].numpy(), C_new[b].cpu().numpy(),
                            counts[b].cpu().numpy(), parity.CENTROID_TOL[dtype] * (1 if dtype != torch.float32 else 10))


@pytest.mark.parametrize("dtype,N,d,K", [(torch.float16, 30000, 128, 300), (torch.float16, 40000, 64, 16),
                                         (torch.float32, 5000, 64, 20), (torch.float32, 5000, 64, 70),
                                         (torch.bfloat16, 30000, 128, 200)])
def test_iteration_replays_from_a_hip_graph(dtype, N, d, K):
    """The library allocates nothing and enqueues kernels only, so one iteration can be captured
    into a graph and replayed.  Replays are interleaved with eager work and each is compared
    with the eager result of the same step."""
    w, X, _, C0 = _problem(dtype, 1, N, d, K, seed=900 + N)
    Xd = X.to(DEV)
    ws = fk.make_workspace(1, N, d, K, dtype, DEV)
    C_g = C0.to(DEV).clone()
    a_g = torch.empty((1, N), dtype=torch.int32, device=DEV)
    n_g = torch.empty((1, K), dtype=torch.int32, device=DEV)
    lp_g = torch.empty((1, K, d), dtype=dtype, device=DEV)
    # one eager call first: one-time kernel attribute / occupancy queries happen here
    fk.fk_lloyd_iter(Xd, C_g, 1, ws=ws, C_lp=lp_g, assign=a_g, counts=n_g)
    C_g.copy_(C0.to(DEV))
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fk.fk_lloyd_iter(Xd, C_g, 1, ws=ws, C_lp=lp_g, assign=a_g, counts=n_g)
    C_g.copy_(C0.to(DEV))
    C_e = C0.to(DEV).clone()
    ws_e = fk.make_workspace(1, N, d, K, dtype, DEV)
    for step in range(4):
        graph.replay()
        a_e, n_e, lp_e = fk.fk_lloyd_iter(Xd, C_e, 1, ws=ws_e)     # eager, same step
        torch.cuda.synchronize()
        assert torch.equal(C_g, C_e) and torch.equal(a_g, a_e) and torch.equal(n_g, n_e), step
        assert torch.equal(lp_g, lp_e)


# ---------------------------------------------------------------------------------------
# Row widths that are not a multiple of 8: served through zero-padded copies inside the workspace.
ODD_WIDTH_CASES = [
    (torch.float16, 1, 3000, 100, 70), (torch.bfloat16, 2, 1500, 3, 5), (torch.float32, 1, 2000, 5, 9),
    (torch.float16, 1, 4000, 1, 4), (torch.float16, 1, 900, 130, 33), (torch.float32, 1, 700, 509, 12),
    (torch.bfloat16, 1, 2500, 20, 16), (torch.float16, 1, 1200, 300, 2500), (torch.float32, 1, 1000, 60, 40),
]


@pytest.mark.parametrize("dtype,B,N,d,K", ODD_WIDTH_CASES)
def test_any_row_width(dtype, B, N, d, K):
    w, X, lab, C0 = _problem(dtype, B, N, d, K, seed=600 + N + d)
    Xd = X.to(DEV)
    keep = Xd.clone()
    consumed = C0.to(dtype)
    # assignment alone, with distances
    a, md = fk.fk_assign(Xd, consumed.to(DEV), min_dist=True)
    # update alone on the generating labels
    C_u, lp_u, n_u = fk.fk_update(Xd, lab.to(DEV), C0.to(DEV))
    # two iterations in one call
    C = C0.to(DEV).clone()
    a2, n2, lp2 = fk.fk_lloyd_iter(Xd, C, 2)
    C1 = C0.to(DEV).clone()
    a1, n1, lp1 = fk.fk_lloyd_iter(Xd, C1, 1)
    torch.cuda.synchronize()
    assert torch.equal(Xd, keep)
    assert C_u.shape == (B, K, d) and lp2.shape == (B, K, d)
    assert torch.equal(lp_u.cpu(), C_u.cpu().to(dtype)) and torch.equal(lp2.cpu(), C.cpu().to(dtype))
    tol = parity.CENTROID_TOL[dtype]
    for b in range(B):
        Xb = parity.widen(X[b])
        ref = oracle.assign(Xb, parity.widen(consumed[b]))
        parity.check_assign(Xb, parity.widen(consumed[b]), a[b].cpu().numpy(), ref)
        same = a[b].cpu().numpy() == ref["assign"]
        scale = ref["xnorm2"] + (parity.widen(consumed[b]).astype(np.float64) ** 2).sum(1)[a[b].cpu().numpy()]
        bound = (1e-3 if dtype != torch.float32 else 1e-5) * scale + 1e-6
        assert (np.abs(md[b].cpu().numpy()[same] - ref["best"][same]) <= bound[same]).all()
        parity.check_update(Xb, lab[b].numpy(), C0[b].numpy(), C_u[b].cpu().numpy(), n_u[b].cpu().numpy(), tol)
        # first iteration of the iterating call, then the second on top of it
        assert torch.equal(a1[b], a[b])
        parity.check_update(Xb, a1[b].cpu().numpy(), C0[b].numpy(), C1[b].cpu().numpy(), n1[b].cpu().numpy(), tol)
        parity.check_assign(Xb, parity.widen(lp1[b].cpu()), a2[b].cpu().numpy())
        parity.check_update(Xb, a2[b].cpu().numpy(), C1[b].cpu().numpy(), C[b].cpu().numpy(), n2[b].cpu().numpy(), tol)


# ---------------------------------------------------------------------------------------
# Few clusters (16-bit storage, K <= 32, d <= 128): the sort-free one-hot MFMA update, fused
# with the assignment inside fk_lloyd_iter.  fk_set_option("fused_update", 0) sends the same
# shape down the general sort-inverse path, so the two can be compared.
FEW_CLUSTER_CASES = [
    # dtype, B, N, d, K, zipf
    (torch.float16, 1, 100000, 64, 16, 1.2),      # the skewed large-N / small-K recipe, scaled
    (torch.bfloat16, 3, 5000, 128, 32, 0.0),      # full table, widest row, batched
    (torch.float16, 1, 4099, 64, 17, 0.0),        # ragged last batch
    (torch.float16, 2, 1000, 8, 3, 0.0),          # narrowest row: one 16-byte piece per point
    (torch.bfloat16, 1, 3000, 24, 5, 0.0),        # d = 8 mod 16, no swizzle
    (torch.float16, 1, 2500, 72, 9, 0.0),         # d not a multiple of 32: half-used column block
    (torch.float16, 1, 7000, 96, 2, 0.0),
    (torch.float16, 1, 31, 64, 4, 0.0),           # less than one batch
    (torch.float16, 1, 1, 16, 1, 0.0),            # one point, one cluster
    (torch.bfloat16, 1, 33, 32, 32, 0.0),         # K about N: most clusters nearly empty
    (torch.float16, 1100, 40, 8, 3, 0.0),         # more instances than workgroups to share: one each
]


@pytest.fixture
def general_path_switch():
    yield lambda on: fk.fk_set_option("fused_update", 0 if on else -1)
    fk.fk_set_option("fused_update", -1)


@pytest.mark.parametrize("dtype,B,N,d,K,zipf", FEW_CLUSTER_CASES)
def test_few_cluster_iteration_matches_oracle_and_general_path(dtype, B, N, d, K, zipf, general_path_switch):
    w, X, lab, C0 = _problem(dtype, B, N, d, K, seed=700 + N + K, zipf=zipf)
    Xd = X.to(DEV)
    assert "stream_update" in fk.fk_plan(B, N, d, K, dtype)
    C_f = C0.to(DEV).clone()
    a_f, n_f, lp_f = fk.fk_lloyd_iter(Xd, C_f, 1)
    general_path_switch(True)
    assert "stream_update" not in fk.fk_plan(B, N, d, K, dtype)
    C_s = C0.to(DEV).clone()
    a_s, n_s, lp_s = fk.fk_lloyd_iter(Xd, C_s, 1)
    general_path_switch(False)
    torch.cuda.synchronize()
    # same scores, same tie rules: identical assignments and counts; sums differ in order only
    assert torch.equal(a_f, a_s) and torch.equal(n_f, n_s)
    consumed = C0.to(dtype)
    for b in range(B):
        Xb = parity.widen(X[b])
        parity.check_assign(Xb, parity.widen(consumed[b]), a_f[b].cpu().numpy())
        parity.check_update(Xb, a_f[b].cpu().numpy(), C0[b].numpy(), C_f[b].cpu().numpy(),
                            n_f[b].cpu().numpy(), parity.CENTROID_TOL[dtype])
        parity.check_centroids(C_f[b].cpu().numpy(), C_s[b].cpu().numpy(), 5e-5, "fused vs sort-inverse")
    assert torch.equal(lp_f.cpu(), C_f.cpu().to(dtype))


@pytest.mark.parametrize("dtype,B,N,d,K,zipf", FEW_CLUSTER_CASES)
def test_few_cluster_update_alone(dtype, B, N, d, K, zipf, general_path_switch):
    """fk_update on given assignments: streamed one-hot update against the oracle and against
    the sort-inverse path; an empty cluster keeps its centroid."""
    w, X, lab, C0 = _problem(dtype, B, N, d, K, seed=800 + N + K, zipf=zipf)
    a = lab.clone()
    if K > 2:
        a[a == 1] = 0
    C_f, lp_f, n_f = fk.fk_update(X.to(DEV), a.to(DEV), C0.to(DEV))
    general_path_switch(True)
    C_s, lp_s, n_s = fk.fk_update(X.to(DEV), a.to(DEV), C0.to(DEV))
    general_path_switch(False)
    torch.cuda.synchronize()
    assert torch.equal(n_f, n_s)
    for b in range(B):
        parity.check_update(parity.widen(X[b]), a[b].numpy(), C0[b].numpy(), C_f[b].cpu().numpy(),
                            n_f[b].cpu().numpy(), parity.CENTROID_TOL[dtype])
        parity.check_centroids(C_f[b].cpu().numpy(), C_s[b].cpu().numpy(), 5e-5, "streamed vs sort-inverse")
    assert torch.equal(lp_f.cpu(), C_f.cpu().to(dtype))


def test_few_cluster_path_is_bit_reproducible_and_multi_iteration():
    w = wl.C4.scaled(N=150001)
    X, lab = wl.make_points(w, return_labels=True)
    Xd = X.to(DEV)
    C0 = wl.gather_rows(X, wl.init_rows(w, lab)).to(DEV)
    Ca, Cb = C0.clone(), C0.clone()
    a1, n1, lp1 = fk.fk_lloyd_iter(Xd, Ca, 4)
    for _ in range(4):
        a2, n2, lp2 = fk.fk_lloyd_iter(Xd, Cb, 1)
    assert torch.equal(Ca, Cb) and torch.equal(a1, a2) and torch.equal(n1, n2) and torch.equal(lp1, lp2)
    assert int(n1.sum()) == w.N
    # the assignment written by the fused pass is what fk_assign gives for the same centroids
    Cc = C0.clone()
    a3, _, lp3 = fk.fk_lloyd_iter(Xd, Cc, 1)
    assert torch.equal(a3, fk.fk_assign(Xd, C0.to(w.torch_dtype)))


def test_few_cluster_update_clamps_ids_like_the_sort_path(general_path_switch):
    w, X, lab, C0 = _problem(torch.float16, 1, 3000, 64, 8, seed=77)
    a = lab.clone()
    a[0, :5] = torch.tensor([-3, 8, 100, -1, 7], dtype=torch.int32)
    C_f, _, n_f = fk.fk_update(X.to(DEV), a.to(DEV), C0.to(DEV))
    general_path_switch(True)
    C_s, _, n_s = fk.fk_update(X.to(DEV), a.to(DEV), C0.to(DEV))
    general_path_switch(False)
    assert torch.equal(n_f, n_s)
    parity.check_centroids(C_f[0].cpu().numpy(), C_s[0].cpu().numpy(), 5e-5, "clamped ids")


# Up to 256 clusters (16-bit storage, 32 < K <= 256, d <= 128): assignment + table of sums in
# one pass over X (table split over the registers of a persistent workgroup, compacted one-hot
# MFMA).  fk_set_option("fused_update", 0) sends the same shape down the general path.
TABLE_CASES = [
    # dtype, B, N, d, K, zipf
    (torch.bfloat16, 4, 32768, 128, 256, 0.0),    # the batched token-clustering recipe, 4 instances
    (torch.float16, 1, 100001, 128, 256, 0.0),    # ragged last batch, many batches per workgroup
    (torch.float16, 1, 70000, 64, 200, 1.2),      # skewed: one wave's clusters take most points
    (torch.bfloat16, 2, 5000, 128, 33, 0.0),      # just above the few-cluster path: waves 2..7 own nothing
    (torch.float16, 1, 3000, 72, 100, 0.0),       # d not a multiple of 32, no swizzle
    (torch.float16, 3, 1000, 8, 64, 0.0),         # narrowest row
    (torch.bfloat16, 1, 255, 32, 40, 0.0),        # less than one batch
    (torch.float16, 1, 257, 96, 129, 0.0),        # one full batch and one point
    (torch.float16, 300, 300, 16, 50, 0.0),       # more instances than compute units
    (torch.bfloat16, 1, 20000, 128, 255, 0.0),    # last cluster row of the last wave unused
]


@pytest.mark.parametrize("dtype,B,N,d,K,zipf", TABLE_CASES)
def test_table_update_iteration_matches_oracle_and_general_path(dtype, B, N, d, K, zipf, general_path_switch):
    w, X, lab, C0 = _problem(dtype, B, N, d, K, seed=900 + N + K, zipf=zipf)
    Xd = X.to(DEV)
    assert "table_update" in fk.fk_plan(B, N, d, K, dtype)
    C_f = C0.to(DEV).clone()
    a_f, n_f, lp_f = fk.fk_lloyd_iter(Xd, C_f, 1)
    general_path_switch(True)
    assert "table_update" not in fk.fk_plan(B, N, d, K, dtype)
    C_s = C0.to(DEV).clone()
    a_s, n_s, lp_s = fk.fk_lloyd_iter(Xd, C_s, 1)
    general_path_switch(False)
    torch.cuda.synchronize()
    # same scores, same tie rules: identical assignments and counts; sums differ in order only
    assert torch.equal(a_f, a_s) and torch.equal(n_f, n_s)
    consumed = C0.to(dtype)
    for b in range(min(B, 4)):
        Xb = parity.widen(X[b])
        parity.check_assign(Xb, parity.widen(consumed[b]), a_f[b].cpu().numpy())
        parity.check_update(Xb, a_f[b].cpu().numpy(), C0[b].numpy(), C_f[b].cpu().numpy(),
                            n_f[b].cpu().numpy(), parity.CENTROID_TOL[dtype])
    for b in range(B):
        parity.check_centroids(C_f[b].cpu().numpy(), C_s[b].cpu().numpy(), 5e-5, "table vs sort-inverse")
    assert torch.equal(lp_f.cpu(), C_f.cpu().to(dtype))


def test_table_update_all_points_in_one_cluster_and_empty_clusters():
    """Degenerate membership: every point goes to one cluster (one wave's list holds whole
    batches, every other cluster stays empty and keeps its centroid)."""
    dtype, B, N, d, K = torch.float16, 1, 3000, 64, 96
    g = torch.Generator().manual_seed(5)
    X = (torch.randn((B, N, d), generator=g) * 0.1 + 3.0).to(dtype)
    C0 = torch.randn((B, K, d), generator=g) * 50.0
    C0[0, 70] = 3.0                                # the only centroid near the data
    C = C0.to(DEV).clone()
    a, n, _ = fk.fk_lloyd_iter(X.to(DEV), C, 1)
    assert int(n[0, 70]) == N and int(n.sum()) == N and bool((a == 70).all())
    parity.check_update(parity.widen(X[0]), a[0].cpu().numpy(), C0[0].numpy(), C[0].cpu().numpy(),
                        n[0].cpu().numpy(), parity.CENTROID_TOL[dtype])


def test_table_update_is_bit_reproducible_and_multi_iteration():
    w = wl.C3.scaled(B=3, N=20001)
    X = wl.make_points(w)
    Xd = X.to(DEV)
    C0 = wl.gather_rows(X, wl.init_rows(w)).to(DEV)
    assert "table_update" in fk.fk_plan(w.B, w.N, w.d, w.K, w.torch_dtype)
    Ca, Cb = C0.clone(), C0.clone()
    a1, n1, lp1 = fk.fk_lloyd_iter(Xd, Ca, 4)
    for _ in range(4):
        a2, n2, lp2 = fk.fk_lloyd_iter(Xd, Cb, 1)
    assert torch.equal(Ca, Cb) and torch.equal(a1, a2) and torch.equal(n1, n2) and torch.equal(lp1, lp2)
    assert int(n1.sum()) == w.B * w.N
    Cc = C0.clone()
    a3, _, _ = fk.fk_lloyd_iter(Xd, Cc, 1)
    assert torch.equal(a3, fk.fk_assign(Xd, C0.to(w.torch_dtype)))


F32_FEW_CLUSTER_CASES = [
    # B, N, d, K, zipf
    (1, 16384, 64, 64, 0.0),          # the tiny fp32 benchmark shape
    (1, 70001, 128, 64, 0.0),         # widest rows, ragged last batch, several batches per workgroup
    (3, 1000, 40, 7, 1.2),            # d between the compiled widths, skewed, batched
    (1, 50000, 32, 33, 0.0),
    (2, 333, 8, 1, 0.0),              # one cluster
    (1, 63, 24, 5, 0.0),              # less than one batch
    (1, 1, 16, 1, 0.0),               # one point
    (1, 90, 64, 64, 0.0),             # K about N: most clusters nearly empty
    (1, 5000, 13, 6, 0.0),            # rows that are not a multiple of 8 wide: padded copy
    (2100, 60, 16, 3, 0.0),           # more instances than workgroups to share: one each
]


@pytest.mark.parametrize("B,N,d,K,zipf", F32_FEW_CLUSTER_CASES)
def test_f32_few_cluster_iteration_matches_oracle_and_general_path(B, N, d, K, zipf, general_path_switch):
    """fp32 storage, K <= 64: assignment and sums in one pass; against the oracle and against
    the general assign + sort-inverse path (identical assignments: same arithmetic)."""
    dtype = torch.float32
    w, X, lab, C0 = _problem(dtype, B, N, d, K, seed=900 + N + K, zipf=zipf)
    Xd = X.to(DEV)
    assert "f32_update" in fk.fk_plan(B, N, d, K, dtype)
    C_f = C0.to(DEV).clone()
    a_f, n_f, lp_f = fk.fk_lloyd_iter(Xd, C_f, 1)
    general_path_switch(True)
    assert "f32_update" not in fk.fk_plan(B, N, d, K, dtype)
    C_s = C0.to(DEV).clone()
    a_s, n_s, lp_s = fk.fk_lloyd_iter(Xd, C_s, 1)
    general_path_switch(False)
    torch.cuda.synchronize()
    assert torch.equal(a_f, a_s) and torch.equal(n_f, n_s)
    for b in range(min(B, 8)):
        Xb = parity.widen(X[b])
        parity.check_assign(Xb, parity.widen(C0[b]), a_f[b].cpu().numpy())
        parity.check_update(Xb, a_f[b].cpu().numpy(), C0[b].numpy(), C_f[b].cpu().numpy(),
                            n_f[b].cpu().numpy(), parity.CENTROID_TOL[dtype])
    parity.check_centroids(C_f.cpu().numpy().reshape(B * K, d), C_s.cpu().numpy().reshape(B * K, d), 2e-6,
                           "one pass vs sort-inverse")
    assert torch.equal(lp_f.cpu(), C_f.cpu())


def test_f32_few_cluster_path_is_bit_reproducible_and_multi_iteration():
    dtype = torch.float32
    w, X, lab, C0 = _problem(dtype, 2, 40000, 64, 48, seed=931)
    Xd = X.to(DEV)
    outs = []
    for _ in range(2):
        C = C0.to(DEV).clone()
        a, n, lp = fk.fk_lloyd_iter(Xd, C, 4)
        torch.cuda.synchronize()
        outs.append((C.cpu(), a.cpu(), n.cpu()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1]) and torch.equal(outs[0][2], outs[1][2])
    # four iterations in one call = four calls of one iteration
    C = C0.to(DEV).clone()
    for _ in range(4):
        a, n, lp = fk.fk_lloyd_iter(Xd, C, 1)
    torch.cuda.synchronize()
    assert torch.equal(C.cpu(), outs[0][0]) and torch.equal(a.cpu(), outs[0][1])
    assert int(n.sum()) == 2 * 40000


def test_f32_few_cluster_all_points_in_one_cluster_and_empty_clusters():
    """Every point nearest to centroid 5: the other clusters are empty and keep their rows."""
    torch.manual_seed(77)
    N, d, K = 3000, 48, 20
    X = torch.randn(1, N, d) * 0.1
    C0 = torch.randn(1, K, d) * 50.0
    C0[0, 5] = 0.0
    C = C0.to(DEV).clone()
    a, n, lp = fk.fk_lloyd_iter(X.to(DEV), C, 1)
    torch.cuda.synchronize()
    assert int((a != 5).sum()) == 0 and int(n[0, 5]) == N and int(n.sum()) == N
    keep = [k for k in range(K) if k != 5]
    assert torch.equal(C.cpu()[0, keep], C0[0, keep])
    parity.check_centroids(C.cpu().numpy()[0, 5:6], X[0].double().mean(0, keepdim=True).numpy(), 1e-5, "mean")


def test_kernel_choices_do_not_change_the_result():
    """Seeded sweep: every host-side kernel choice forced the other way (tile shape, streaming
    assign, staged scatter, several sub-tiles per sort workgroup, sort-free update) must give the
    same assignments and counts as the default rules, and centroids equal up to summation order."""
    rng = np.random.default_rng(77)
    opts = ("assign_variant", "assign_stream", "sort_stage_bins", "sort_min_rounds", "fused_update")
    for case in range(36):
        dtype = (torch.float16, torch.bfloat16)[case % 2]
        d = int(rng.choice([8, 24, 32, 64, 72, 128, 100, 200]))
        K = int(rng.choice([2, 9, 16, 31, 40, 64, 100, 300, 1024, 2500]))
        N = int(rng.integers(200, 30000))
        B = int(rng.choice([1, 1, 2]))
        w = wl.Workload("o", B, N, d, K, "fp16" if dtype == torch.float16 else "bf16", 3.0, 1.0, 0.0, 1, 9000 + case)
        X = wl.make_points(w).to(DEV)
        idx = torch.randint(0, N, (B, K), generator=torch.Generator().manual_seed(case))
        C0 = wl.gather_rows(X.cpu(), idx).to(DEV)
        Cd = C0.clone()
        a_d, n_d, _ = fk.fk_lloyd_iter(X, Cd, 2)
        forced = {"assign_variant": int(rng.integers(0, 4)), "assign_stream": int(rng.integers(0, 2)),
                  "sort_stage_bins": int(rng.choice([0, 2048])), "sort_min_rounds": int(rng.choice([1, 2, 3])),
                  "fused_update": 0}
        try:
            for k, v in forced.items():
                fk.fk_set_option(k, v)
            Cf = C0.clone()
            a_f, n_f, _ = fk.fk_lloyd_iter(X, Cf, 2)
        finally:
            for k in opts:
                fk.fk_set_option(k, -1)
        torch.cuda.synchronize()
        # the first iteration's centroids may differ in the last bits (summation order), which can
        # flip a near-tie of the second assignment: compare the first iteration exactly, the second
        # through the tolerance rules
        C1d, C1f = C0.clone(), C0.clone()
        a1d, n1d, _ = fk.fk_lloyd_iter(X, C1d, 1)
        try:
            for k, v in forced.items():
                fk.fk_set_option(k, v)
            a1f, n1f, _ = fk.fk_lloyd_iter(X, C1f, 1)
        finally:
            for k in opts:
                fk.fk_set_option(k, -1)
        assert torch.equal(a1d, a1f) and torch.equal(n1d, n1f), (case, dtype, B, N, d, K, forced)
        for b in range(B):
            parity.check_centroids(C1f[b].cpu().numpy(), C1d[b].cpu().numpy(), 5e-5, f"case {case} {forced}")
            parity.check_update(parity.widen(X[b]), a_f[b].cpu().numpy(), C1f[b].cpu().numpy(), Cf[b].cpu().numpy(),
                                n_f[b].cpu().numpy(), parity.CENTROID_TOL[dtype])
        assert int(n_f.sum()) == B * N and int(n_d.sum()) == B * N
