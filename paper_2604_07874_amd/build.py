"""Builds libvalvekv.so in-tree with hipcc for gfx950.  Usage: python -m paper_2604_07874_amd.build
With --host-sanitizers it also builds libvalvekv_hostsan.so: the same sources with AddressSanitizer and
UndefinedBehaviorSanitizer on the host side only (pool, plans, scheduler, policies; device code is
compiled as always), for the host tests that run without a GPU."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvalvekv.so")
SOURCES = ["pool.hip", "attn.hip", "reclaim.hip", "policy.hip", "prefill.hip", "probe.hip", "arena.hip"]
DRIVER = os.path.join(HERE, "vkv_pmc_driver")
HOSTSAN_LIB = os.path.join(HERE, "libvalvekv_hostsan.so")


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found (set HIPCC)")


def build(verbose: bool = True) -> str:
    """Compiles every HIP source; always rebuilds.  Returns the library path."""
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Wall", "-Wno-unused-command-line-argument",
           # packed fp32 VALU forms are kept off for device code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    tmp = LIB + ".tmp"
    cmd += ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    os.replace(tmp, LIB)
    build_driver(verbose)
    return LIB


def source_paths():
    inc = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".h", ".inc"))]
    return [os.path.join(CSRC, s) for s in SOURCES] + inc + [os.path.join(ROOT, "include", "valvekv.h")]


def asan_runtime() -> str:
    """The shared AddressSanitizer runtime of hipcc's clang; a process that loads the sanitized
    library without being instrumented itself (python) has to preload it."""
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc_path())), "..", "lib", "llvm", "bin", "clang")
    for cand in (clang, "/opt/rocm/llvm/bin/clang"):
        if os.path.exists(cand):
            out = subprocess.run([cand, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
            path = out.stdout.strip()
            if os.path.isabs(path) and os.path.exists(path):
                return path
    raise RuntimeError("the AddressSanitizer runtime of hipcc's clang was not found")


def build_host_sanitized(verbose: bool = True) -> str:
    """Same sources, host code instrumented (address + undefined), device code untouched."""
    host_san = "-Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined -Xarch_host -fno-omit-frame-pointer"
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-shared-libsan",
           "-Wno-unused-command-line-argument", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           *host_san.split(), "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    tmp = HOSTSAN_LIB + ".tmp"
    cmd += ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        noise = "is not a recognized feature for this target"
        raise RuntimeError("hipcc failed (host sanitizers):\n" +
                           "\n".join(l for l in res.stderr.splitlines() if noise not in l))
    os.replace(tmp, HOSTSAN_LIB)
    return HOSTSAN_LIB


def build_driver(verbose: bool = True) -> str:
    """The native counter-run driver / call-sequence example, linked against the library."""
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wno-unused-command-line-argument",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), os.path.join(CSRC, "pmc_driver.hip"),
           "-L", HERE, "-lvalvekv", "-Wl,-rpath,$ORIGIN", "-o", DRIVER + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        noise = "is not a recognized feature for this target"
        raise RuntimeError("hipcc failed (driver):\n" + "\n".join(l for l in res.stderr.splitlines() if noise not in l))
    os.replace(DRIVER + ".tmp", DRIVER)
    return DRIVER


if __name__ == "__main__":
    print(build())
    if "--host-sanitizers" in sys.argv[1:]:
        print(build_host_sanitized())
