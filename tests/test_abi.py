"""CPU-side checks of the boundary: the library loads without a GPU, exports every symbol the
header declares, and its host-only logic (workspace sizing, argument validation, which all
happens before the first HIP call) behaves.  No kernel is launched here."""
import ctypes
import re
from pathlib import Path

import pytest
import torch

from paper_2603_09229_amd import binding as fk

ROOT = Path(__file__).resolve().parent.parent
HEADER = ROOT / "include" / "flashkm.h"


def _declared():
    text = re.sub(r"/\*.*?\*/", "", HEADER.read_text(), flags=re.S)
    return sorted(set(re.findall(r"\b(fk_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_all_exported():
    names = _declared()
    assert set(names) == set(fk.EXPORTS)
    L = fk.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_workspace_sizes_are_sane():
    f16, f32 = torch.float16, torch.float32
    base = fk.fk_workspace_bytes(1, 1 << 20, 128, 1024, f16)
    assert base >= (1 << 20) * 4                            # at least sorted_idx
    assert base < (1 << 20) * 128 * 2                       # and well below one copy of X
    assert fk.fk_workspace_bytes(2, 1 << 20, 128, 1024, f16) > base
    assert fk.fk_workspace_bytes(1, 1 << 20, 128, 65536, f16) > base
    assert fk.fk_workspace_bytes(1, 1000, 64, 10, f32) % 256 == 0
    # a width that is not a multiple of 8 is served through a zero-padded copy: room for it
    assert fk.fk_workspace_bytes(1, 1000, 12, 4, f16) >= fk.fk_workspace_bytes(1, 1000, 16, 4, f16) + 1000 * 16 * 2
    assert fk.fk_ooc_workspace_bytes(1 << 16, 100, 16, f16) >= 2 * (1 << 16) * 104 * 2   # chunk rows padded to 104
    for bad in [(0, 10, 64, 4), (1, 0, 64, 4), (1, 10, 0, 4), (1, 10, 520, 4), (1, 10, 64, 0),
                (1, 10, 64, 65537), (3, 1 << 30, 64, 4), (65536, 4, 64, 4)]:
        assert fk.fk_workspace_bytes(*bad, f16) == 0
    assert fk.fk_ooc_workspace_bytes(1 << 16, 128, 65536, f16) > 2 * (1 << 16) * 256
    assert fk.fk_ooc_workspace_bytes(0, 128, 16, f16) == 0


def test_argument_validation_happens_on_the_host():
    L = fk.lib()
    buf = ctypes.create_string_buffer(1 << 16)
    p = ctypes.c_void_p((ctypes.addressof(buf) + 255) & ~255)
    # NULL data pointers -> FK_EINVAL, before any GPU call
    rc = L.fk_assign(None, None, None, None, 1, 16, 16, 2, fk.FK_F16, p, 1 << 15, None)
    assert rc == 1 and b"NULL" in L.fk_last_error()
    # unsupported shape
    rc = L.fk_assign(p, p, p, None, 1, 16, 513, 2, fk.FK_F16, p, 1 << 15, None)
    assert rc == 2
    # workspace too small
    rc = L.fk_update(p, p, p, p, None, p, 1, 1 << 20, 128, 1024, fk.FK_F16, p, 1024, None)
    assert rc == 3 and b"workspace too small" in L.fk_last_error()
    # bad dtype enum
    rc = L.fk_lloyd_iter(p, p, None, p, p, 1, 16, 16, 2, 7, 1, p, 1 << 15, None)
    assert rc == 1
    rc = L.fk_lloyd_iter(p, p, None, p, p, 1, 16, 16, 2, fk.FK_F16, -1, p, 1 << 15, None)
    assert rc == 1
    # iters == 0 is a no-op that touches nothing
    assert L.fk_lloyd_iter(p, p, None, p, p, 1, 16, 16, 2, fk.FK_F16, 0, p, 1 << 15, None) == 0
    rc = L.fk_sort_inverse(p, p, p, 1, 100, 70000, p, 1 << 15, None)
    assert rc == 2
    rc = L.fk_lloyd_ooc(None, p, None, p, 100, 16, 4, fk.FK_F16, 1, 0, p, 1 << 15, None)
    assert rc == 1


def test_binding_rejects_host_tensors():
    X = torch.zeros((1, 8, 16), dtype=torch.float16)
    with pytest.raises(ValueError):
        fk.fk_assign(X, X[:, :2], ws=torch.empty(1024, dtype=torch.uint8))


def test_plan_describes_the_choice_per_shape():
    f16 = torch.float16
    # no GPU here: the heuristic assumes 256 CUs
    assert "mfma_sweep(variant=2" in fk.fk_plan(1, 1 << 20, 128, 1024, f16)     # whole rounds of 512
    assert "mfma_sweep(variant=3" in fk.fk_plan(1, 1 << 16, 128, 1024, f16)     # few points: small groups
    assert "mfma_sweep(variant=0" in fk.fk_plan(1, 300000, 128, 1024, f16)      # least idle last round
    assert "mfma_stream" in fk.fk_plan(1, 1 << 24, 64, 16, f16)             # X far beyond the cache
    assert "mfma_sweep" in fk.fk_plan(1, 1 << 20, 64, 16, f16)              # X cache-sized: bulk loads
    assert "mfma_stream" in fk.fk_plan(1, 1 << 24, 64, 64, f16)             # two centroid tiles: still streaming
    assert "mfma_sweep(variant=0" in fk.fk_plan(1, 1 << 24, 64, 100, f16)   # more: sweeping, HBM-bound shape
    assert "mfma_sweep" in fk.fk_plan(1, 1 << 24, 128, 100, f16)
    assert "mfma_sweep(variant=2" in fk.fk_plan(1, 1 << 19, 64, 100, f16)   # same K with X inside the last-level cache
    assert "device(cus=256,lds=160KiB,llc=256MiB)" in fk.fk_plan(1, 1000, 64, 8, f16)   # no GPU: MI355X figures
    assert "mfma_sweep" in fk.fk_plan(1, 1 << 25, 32, 16, f16)              # narrow rows
    assert "mfma_wide(chunks=32" in fk.fk_plan(1, 1 << 20, 512, 65536, f16)
    assert "sort=2pass" in fk.fk_plan(1, 1 << 20, 512, 65536, f16)
    # few clusters: the sort-free update fused into the assignment pass, unless switched off
    assert "stream_update" in fk.fk_plan(1, 1 << 24, 64, 16, f16)
    assert "stream_update" not in fk.fk_plan(1, 1 << 24, 64, 16, torch.float32)
    assert "stream_update" not in fk.fk_plan(1, 1 << 24, 64, 33, f16)
    # small fp32 problems: one pass as well; larger ones keep assign + sort-inverse
    f32 = torch.float32
    assert "f32_update" in fk.fk_plan(1, 16384, 64, 64, f32)
    assert "f32_update" in fk.fk_plan(4, 32768, 128, 8, f32)
    assert "f32_update" not in fk.fk_plan(1, (1 << 17) + 1, 64, 64, f32)
    assert "f32_update" not in fk.fk_plan(1, 16384, 64, 65, f32)
    assert "f32_update" not in fk.fk_plan(1, 16384, 136, 64, f32)
    fk.fk_set_option("fused_update", 0)
    assert "workgroup_per_item" in fk.fk_plan(1, 1 << 24, 64, 16, f16)
    assert "f32_update" not in fk.fk_plan(1, 16384, 64, 64, f32)
    fk.fk_set_option("fused_update", -1)
    assert fk.fk_plan(1, 100, 600, 3, f16) == "unsupported"
    assert "rows_padded=12->16" in fk.fk_plan(1, 100, 12, 40, f16)
    fk.fk_set_option("assign_variant", 1)
    assert "variant=1" in fk.fk_plan(1, 1 << 20, 128, 1024, f16)
    fk.fk_set_option("assign_variant", -1)
    with pytest.raises(fk.FlashKMError):
        fk.fk_set_option("assign_variant", 9)
