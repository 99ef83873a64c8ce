"""Host-side sanitizer builds (no GPU): the CPU oracle under gcc's AddressSanitizer + UBSan, and
the C-ABI library's host code (geometry, workspace carving, plan strings, options, argument
validation) under clang's, each driven by a small program of its own.  Sanitizers run on host code
only; nothing here launches a kernel."""
import json
import os
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SAN = ROOT / "tests" / "sanitize"
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = tmp_path / "oracle_asan"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-o", str(exe), str(ROOT / "oracle" / "lloyd_oracle.c"),
           str(SAN / "oracle_driver.c"), "-lm"]
    subprocess.run(cmd, check=True)
    g = json.loads((ROOT / "tests" / "golden" / "handworked_2d.json").read_text())
    X, C = g["X"], g["C"]
    args = [len(X), len(X[0]), len(C)] + [v for r in X for v in r] + [v for r in C for v in r] + g["assign"] + g["best"]
    env = dict(ENV, OMP_NUM_THREADS="4")
    # the OpenMP runtime keeps its thread pool alive at exit: not a leak of the oracle's
    env["ASAN_OPTIONS"] = ENV["ASAN_OPTIONS"].replace("detect_leaks=1", "detect_leaks=0")
    r = subprocess.run([str(exe)] + [repr(float(a)) if isinstance(a, float) else str(a) for a in args],
                       capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "oracle sanitizer run ok" in r.stdout, r.stdout + r.stderr


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    from paper_2603_09229_amd import build as fk_build
    lib = tmp_path / "libflashkm_san.so"
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]
    flags = [f for f in fk_build.FLAGS if f != "-O3"]
    cmd = [fk_build.HIPCC, *flags, "-O1", "-g", *san, "-shared-libsan", "-o", str(lib), *map(str, fk_build.sources()), *fk_build.LIBS]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    exe = tmp_path / "api_san"
    # the driver is plain host C++: ROCm's clang (same sanitizer runtime as the library's host code)
    clangxx = str(Path(fk_build.HIPCC).resolve().parent.parent / "lib" / "llvm" / "bin" / "clang++")
    if not Path(clangxx).exists():
        clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    cmd = [clangxx, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-shared-libsan", f"-I{ROOT / 'include'}", "-o", str(exe), str(SAN / "api_driver.cpp"),
           f"-L{tmp_path}", "-lflashkm_san", f"-Wl,-rpath,{tmp_path}"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    # (leak checking off: the HIP runtime the library links against keeps allocations of its own)
    env = dict(ENV)
    env["ASAN_OPTIONS"] = ENV["ASAN_OPTIONS"].replace("detect_leaks=1", "detect_leaks=0")
    rt = subprocess.run([clangxx, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    rtdir = str(Path(rt).parent) if "/" in rt else next(
        (str(q.parent) for q in Path(clangxx).resolve().parent.parent.glob("lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")), "")
    env["LD_LIBRARY_PATH"] = rtdir + os.pathsep + env.get("LD_LIBRARY_PATH", "")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0 and "api sanitizer run ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
