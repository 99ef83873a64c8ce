"""The allocation-free entry point fk_assign_static against fk_assign (same kernels, scratch in
the library's static device array instead of the caller's workspace): called through the raw C
ABI, two calls in a row on the same stream, the second with a smaller input, results bit-equal
to fk_assign's.  Collected last on purpose."""
import ctypes

import pytest
import torch

from paper_2603_09229_amd import binding as fk
from paper_2603_09229_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def _raw_static(X, C, want_dist):
    L = fk.lib()
    B, N, d = X.shape
    K = C.shape[1]
    a = torch.full((B, N), -7, dtype=torch.int32, device=DEV)
    md = torch.full((B, N), -1.0, dtype=torch.float32, device=DEV) if want_dist else None
    s = ctypes.c_void_p(torch.cuda.current_stream(DEV).cuda_stream)
    rc = L.fk_assign_static(ctypes.c_void_p(X.data_ptr()), ctypes.c_void_p(C.data_ptr()),
                            ctypes.c_void_p(a.data_ptr()),
                            ctypes.c_void_p(md.data_ptr()) if want_dist else None,
                            B, N, d, K, fk._DTYPE[X.dtype], s)
    assert rc == 0, L.fk_last_error()
    return a, md


def _case(dtype_name, B, N, d, K, seed):
    w = wl.C2.scaled(B=B, N=N, d=d, K=K, dtype=dtype_name, seed=seed)
    X = wl.make_points(w, device=DEV)
    C = wl.gather_rows(X, wl.init_rows(w)).to(w.torch_dtype).contiguous()
    return X, C


def test_static_scratch_assign_equals_workspace_assign_twice_in_a_row():
    # big first (fills a large part of the scratch), then a smaller shape of another type and
    # width: whatever the first call left behind must not leak into the second
    cases = [("fp16", 2, 70001, 128, 2500, 11), ("bf16", 1, 3001, 64, 45, 12), ("fp32", 1, 2000, 64, 33, 13)]
    for name, B, N, d, K, seed in cases:
        X, C = _case(name, B, N, d, K, seed)
        a_s, md_s = _raw_static(X, C, want_dist=True)
        a_w, md_w = fk.fk_assign(X, C, min_dist=True)
        torch.cuda.synchronize()
        assert torch.equal(a_s, a_w), (name, B, N, d, K)
        assert torch.equal(md_s, md_w), (name, B, N, d, K)
        assert int(a_s.min()) >= 0 and int(a_s.max()) < K


def test_static_scratch_limit_is_an_error_not_a_fault():
    L = fk.lib()
    p = ctypes.c_void_p(256)          # never dereferenced: the size check comes first
    assert L.fk_assign_static_limit() == 16 << 20
    rc = L.fk_assign_static(p, p, p, None, 1, 1000, 256, 65536, fk.FK_F16, None)
    assert rc == 3 and b"static scratch" in L.fk_last_error()
    rc = L.fk_assign_static(p, p, p, None, 1, 1000, 12, 16, fk.FK_F16, None)
    assert rc == 2
    # the largest shape that fits runs
    g = torch.Generator(device=DEV).manual_seed(14)
    X = (torch.randn((1, 4096, 128), generator=g, device=DEV) * 3).to(torch.float16)
    C = (torch.randn((1, 65536, 128), generator=g, device=DEV) * 3).to(torch.float16)
    a_s, _ = _raw_static(X, C, want_dist=False)
    assert torch.equal(a_s, fk.fk_assign(X, C))
