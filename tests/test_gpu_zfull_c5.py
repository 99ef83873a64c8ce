"""The out-of-core configuration at its full size (64 GiB of pinned host memory), in a file of
its own that pytest collects after the other GPU parity tests: the pinned block is created late
and handed back to the system before anything else runs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_09229_amd import binding as fk
from paper_2603_09229_amd import workloads as wl
from tests import parity
from tests.test_gpu_fullsize import _check_instance

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def _host_checksum(Xh2d: torch.Tensor, rows_per_block: int = 1 << 24) -> int:
    """Sum of the stored 32-bit words of a pinned host matrix, computed on the device block by
    block (one pass over PCIe instead of a slow host reduction)."""
    total = 0
    for r0 in range(0, Xh2d.shape[0], rows_per_block):
        blk = Xh2d[r0:r0 + rows_per_block].to(DEV, non_blocking=False)
        total += int(blk.view(torch.int32).sum(dtype=torch.int64))
        del blk
    return total


def test_c5_full_size_out_of_core():
    """The out-of-core configuration at its full size and in the geometry bench.py times:
    N = 2^28 rows of d = 128 fp16 in 64 GiB of pinned host memory, K = 65536, chunks of 2^24 rows
    (workgroup-per-item reduction with 65536 clusters, two-pass sort of 2^24 keys per chunk,
    sums and counts accumulated over 16 chunks), device workspace under the 32 GB cap.  Two
    iterations, each checked on >= 2^14 sampled points against all centroids and on all members
    of >= 256 whole clusters (gathered from the host copy)."""
    w = wl.C5
    chunk = 1 << 24
    N = w.N
    Xh = None
    while N >= (1 << 25):
        try:
            Xh = torch.empty((1, N, w.d), dtype=w.torch_dtype, pin_memory=True)
            break
        except RuntimeError as e:                 # the box cannot pin that much: halve, say so
            print(f"cannot pin {N * w.d * 2 / 2**30:.0f} GiB ({e}); trying half", flush=True)
            N //= 2
    if Xh is None:
        pytest.skip("this box cannot pin even 8 GiB of host memory")
    w = w.scaled(N=N)
    print(f"c5: N = 2^{N.bit_length() - 1}, chunk = 2^24, pinned {N * w.d * 2 / 2**30:.0f} GiB", flush=True)
    wl.make_points(w, device=DEV, rows_per_block=1 << 24, out=Xh)
    torch.cuda.synchronize()
    before = _host_checksum(Xh[0])
    idx = wl.init_rows(w)
    C = Xh[0][idx[0]].to(torch.float32).to(DEV).contiguous()
    need = fk.fk_ooc_workspace_bytes(chunk, w.d, w.K, w.torch_dtype)
    assert 0 < need <= (32 << 30) - (2 << 30), need          # C, counts and assign come on top
    dev_ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    for it in range(2):
        C_prev = C.clone()
        consumed = C_prev.to(w.torch_dtype)
        a, counts = fk.fk_lloyd_ooc(Xh[0], C, 1, dev_ws=dev_ws, chunk_rows=chunk)
        st = _check_instance(w, Xh[0], consumed, C_prev, C, a, counts, 1 << 14, 288, seed=500 + it)
        print(f"{w.name} (N={N}) iter {it}: {st}", flush=True)
        del a
    same = _host_checksum(Xh[0]) == before
    # hand the 64 GiB back to the system before the other tests run (the pinned block would
    # otherwise stay in torch's host cache, to be split among later small pinned tensors)
    del Xh, dev_ws
    import gc
    gc.collect()
    torch.cuda.synchronize()
    torch._C._host_emptyCache()
    torch.cuda.empty_cache()
    assert same
