"""Compile the HIP sources under csrc/ into libflashkm.so (gfx950 only), in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
CSRC = PKG / "csrc"
LIB = PKG / "libflashkm.so"

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-fno-gpu-rdc", "-Wall", "-Wno-unused-function",
    # MFMA accumulators in ordinary VGPRs: the argmin epilogue reads them with VALU
    # instructions, which cannot address AGPRs (saves one copy per accumulator element)
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    f"-I{ROOT / 'include'}", f"-I{CSRC}",
]
# the HSA runtime (already a dependency of the HIP runtime) is asked for the cache sizes
LIBS = ["-L/opt/rocm/lib", "-lhsa-runtime64"]


def sources() -> list[Path]:
    return sorted(CSRC.glob("*.hip"))


def build(verbose: bool = True) -> Path:
    """Always recompiles (a few tens of seconds); raises on any compiler error."""
    tmp = LIB.with_suffix(f".tmp{os.getpid()}.so")
    cmd = [HIPCC, *FLAGS, "-o", str(tmp), *map(str, sources()), *LIBS]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    if proc.returncode != 0:
        if tmp.exists():
            tmp.unlink()
        raise RuntimeError(f"hipcc failed ({proc.returncode}):\n{err}")
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
