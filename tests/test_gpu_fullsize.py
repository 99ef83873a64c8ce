"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot redo a full-size problem in seconds, so each case checks
  * assignments of a seeded sample of points, one by one, against the oracle (same rule
    as the small cases),
  * the update of a seeded sample of whole clusters against the oracle's mean of the
    members the GPU assigned to them,
  * properties that hold at any size: counts equal the histogram of the assignments and
    sum to N, every index is in range, X is left untouched.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_09229_amd import binding as fk
from paper_2603_09229_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def _checksum(X: torch.Tensor) -> int:
    return int(X.view(torch.int16).to(torch.int64).sum()) if X.element_size() == 2 \
        else int(X.view(torch.int32).to(torch.int64).sum())


def _check_instance(w, Xb, consumed_b, C_prev_b, C_new_b, a_b, counts_b, n_points, n_clusters, seed):
    """Xb [N,d] device, consumed_b [K,d] device (kernel dtype), a_b [N], counts_b [K]."""
    g = torch.Generator().manual_seed(seed)
    N, K = Xb.shape[0], consumed_b.shape[0]
    assert int(a_b.min()) >= 0 and int(a_b.max()) < K
    hist = torch.bincount(a_b.to(torch.int64), minlength=K)
    assert torch.equal(hist, counts_b.to(torch.int64)) and int(hist.sum()) == N
    # sampled points, all K centroids
    # (Xb may live in host memory while the results are on the device: index each on its own side)
    pick = torch.randint(0, N, (n_points,), generator=g)
    Xs = parity.widen(Xb[pick.to(Xb.device)])
    st = parity.check_assign(Xs, parity.widen(consumed_b), a_b[pick.to(a_b.device)].cpu().numpy())
    # sampled clusters, all their members (non-empty ones and, if any, an empty one)
    tol = parity.CENTROID_TOL[w.torch_dtype]
    ks = torch.randint(0, K, (n_clusters,), generator=g).tolist()
    ks.append(int(hist.argmax()))
    empties = torch.nonzero(hist == 0).flatten()
    if empties.numel():
        ks.append(int(empties[0]))
    for k in set(ks):
        members = torch.nonzero(a_b == k).flatten()
        if members.numel() == 0:
            assert torch.equal(C_new_b[k], C_prev_b[k])
            continue
        Xm = parity.widen(Xb[members.to(Xb.device)])
        u = oracle.update(Xm, np.zeros(len(Xm), np.int32), C_prev_b[k:k + 1].cpu().numpy())
        assert int(u["counts"][0]) == int(counts_b[k])
        parity.check_centroids(C_new_b[k:k + 1].cpu().numpy(), u["C"], tol, f"cluster {k}")
    return st


def _run_incore(w, n_points, n_clusters, instances, iters=None):
    """Runs the configuration's whole iteration count; iterations 1, 2, the middle one and the
    last are checked (teacher-forced: the oracle sees the centroids the GPU consumed and the
    assignments the GPU produced), the others only run."""
    X, lab = wl.make_points(w, device=DEV, return_labels=True)
    idx = wl.init_rows(w, lab if w.zipf_s > 0 else None)
    del lab
    C = wl.gather_rows(X, idx).contiguous()
    before = _checksum(X)
    ws = fk.make_workspace(w.B, w.N, w.d, w.K, w.torch_dtype, DEV)
    iters = w.iters if iters is None else iters
    checked = {0, 1, iters // 2, iters - 1}
    for it in range(iters):
        if it not in checked:
            fk.fk_lloyd_iter(X, C, 1, ws=ws)
            continue
        C_prev = C.clone()
        consumed = C_prev.to(w.torch_dtype)
        a, counts, C_lp = fk.fk_lloyd_iter(X, C, 1, ws=ws)
        torch.cuda.synchronize()
        assert torch.equal(C_lp, C.to(w.torch_dtype))
        for b in instances:
            st = _check_instance(w, X[b], consumed[b], C_prev[b], C[b], a[b], counts[b],
                                 n_points, n_clusters, seed=17 * it + b)
            print(f"{w.name} iter {it} instance {b}: {st}", flush=True)
    assert _checksum(X) == before


def test_c2_full_size():
    _run_incore(wl.C2, n_points=4096, n_clusters=24, instances=[0])


def test_c3_full_size_batched():
    _run_incore(wl.C3, n_points=2048, n_clusters=12, instances=[0, 13, 31])


def test_c4_full_size_skewed():
    """Few clusters: fk_lloyd_iter takes the fused one-hot pass here."""
    assert "stream_update" in fk.fk_plan(wl.C4.B, wl.C4.N, wl.C4.d, wl.C4.K, wl.C4.torch_dtype)
    _run_incore(wl.C4, n_points=8192, n_clusters=4, instances=[0])


def test_c4_full_size_skewed_general_path():
    """The same shape down the general path (streaming assign, sort-inverse, gather-reduce)."""
    fk.fk_set_option("fused_update", 0)
    try:
        _run_incore(wl.C4, n_points=8192, n_clusters=4, instances=[0], iters=2)
    finally:
        fk.fk_set_option("fused_update", -1)


def test_c4_full_size_update_alone_with_the_true_labels():
    """fk_update on the generating labels (the skew is then exactly the recipe's Zipf law):
    streamed one-hot update and sort-inverse update agree on the counts exactly and on the
    centroids to summation order, and sampled clusters match the oracle's means."""
    w = wl.C4
    X, lab = wl.make_points(w, device=DEV, return_labels=True)
    C0 = wl.gather_rows(X, wl.init_rows(w, lab)).contiguous()
    ws = fk.make_workspace(w.B, w.N, w.d, w.K, w.torch_dtype, DEV)
    C_f, _, n_f = fk.fk_update(X, lab, C0, ws=ws)
    fk.fk_set_option("fused_update", 0)
    try:
        C_s, _, n_s = fk.fk_update(X, lab, C0, ws=ws)
    finally:
        fk.fk_set_option("fused_update", -1)
    torch.cuda.synchronize()
    hist = torch.bincount(lab[0].to(torch.int64), minlength=w.K)
    assert torch.equal(n_f[0].to(torch.int64), hist) and torch.equal(n_f, n_s)
    parity.check_centroids(C_f[0].cpu().numpy(), C_s[0].cpu().numpy(), 5e-5, "streamed vs sort-inverse")
    for k in (0, 7, 15):                       # largest, middle and smallest cluster
        Xm = parity.widen(X[0][lab[0] == k])
        u = oracle.update(Xm, np.zeros(len(Xm), np.int32), C0[0][k:k + 1].cpu().numpy())
        parity.check_centroids(C_f[0][k:k + 1].cpu().numpy(), u["C"],
                               parity.CENTROID_TOL[w.torch_dtype], f"cluster {k}")


def test_paper_large_k_d512_shape():
    """N = 2^20, K = 65536, d = 512 (a shape the paper quotes for its large-N / large-K
    regime): wide-feature kernels and the two-pass sort at scale, sampled against the oracle."""
    _run_incore(wl.P512, n_points=512, n_clusters=32, instances=[0], iters=1)


def test_c5_recipe_out_of_core_large_k():
    """The out-of-core configuration's recipe (K = 65536, d = 128, fp16, X in pinned host
    memory, streamed in chunks) at N = 2^22 so the host buffer stays at 1 GiB."""
    w = wl.C5.scaled(N=1 << 22)
    Xh = torch.empty((1, w.N, w.d), dtype=w.torch_dtype, pin_memory=True)
    Xd = wl.make_points(w, device=DEV, rows_per_block=1 << 20)
    Xh.copy_(Xd)
    idx = wl.init_rows(w)
    C = wl.gather_rows(Xd, idx)[0].contiguous()
    chunk = 1 << 20
    dev_ws = torch.empty(fk.fk_ooc_workspace_bytes(chunk, w.d, w.K, w.torch_dtype),
                         dtype=torch.uint8, device=DEV)
    for it in range(2):
        C_prev = C.clone()
        consumed = C_prev.to(w.torch_dtype)
        a, counts = fk.fk_lloyd_ooc(Xh[0], C, 1, dev_ws=dev_ws, chunk_rows=chunk)
        st = _check_instance(w, Xd[0], consumed, C_prev, C, a, counts, 1024, 48, seed=it)
        print(f"{w.name} (N=2^22) iter {it}: {st}", flush=True)


def test_incore_many_points_many_clusters():
    """In-core shapes that take the same kernel forms as the out-of-core configuration's chunks:
    more than 2^22 points (a workgroup per reduction item) together with more than 2048 clusters
    (two-pass sort, segment table from the sorted ids, item table from its own scan kernel)."""
    for (N, d, K, npts, ncl) in ((1 << 23, 128, 4096, 2048, 24), ((1 << 23) + 12345, 64, 65536, 1024, 64)):
        w = wl.C5.scaled(N=N, d=d, K=K, seed=1300 + d)
        plan = fk.fk_plan(1, N, d, K, w.torch_dtype)
        assert "sort=2pass" in plan and "workgroup_per_item" in plan, plan
        _run_incore(w, n_points=npts, n_clusters=ncl, instances=[0], iters=2)
