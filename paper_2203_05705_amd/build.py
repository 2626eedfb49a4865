"""Builds libard.so (the C-ABI HIP library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libard.so")
BUILD_DIR = os.path.join(HERE, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep hipcc from forming packed fp32 instructions (gfx950 guidance for the test machines)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
] + os.environ.get("ARD_EXTRA_HIPCC_FLAGS", "").split()


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; libard.so cannot be built")


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


# host code under AddressSanitizer + UBSan (device code untouched): for running the CPU test-suite -- dispatch,
# class tables, the host-side bounds proofs -- against, see build_library(host_sanitizers=True)
HOST_SAN_FLAGS = ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                  "-Xarch_host", "-fno-omit-frame-pointer"]
LIB_HOSTSAN = os.path.join(HERE, "libard_hostsan.so")


def build_library(verbose: bool = True, jobs: int = 8, host_sanitizers: bool = False) -> str:
    """Compile every csrc/*.hip and link libard.so next to this file. Always recompiles.
    host_sanitizers: build libard_hostsan.so instead (load it with ARD_LIBRARY=<path> and the ASan runtime
    preloaded: LD_PRELOAD=$(hipcc -print-file-name=libclang_rt.asan-x86_64.so) ASAN_OPTIONS=detect_leaks=0)."""
    hipcc = _hipcc()
    build_dir = BUILD_DIR + ("_hostsan" if host_sanitizers else "")
    lib = LIB_HOSTSAN if host_sanitizers else LIB
    flags = HIPCC_FLAGS + (HOST_SAN_FLAGS if host_sanitizers else [])
    link_flags = ["-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize"] if host_sanitizers else []
    os.makedirs(build_dir, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(build_dir, os.path.basename(s)[:-4] + ".o") for s in srcs]

    def compile_one(pair):
        src, obj = pair
        cmd = [hipcc, *flags, "-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose:
            print(f"[build] {os.path.basename(src)} ok", flush=True)
        return obj

    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(srcs)))) as ex:
        list(ex.map(compile_one, zip(srcs, objs)))
    tmp = lib + ".tmp"
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *link_flags, *objs, "-o", tmp],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    os.replace(tmp, lib)
    if verbose:
        print(f"[build] linked {lib}", flush=True)
    return lib


if __name__ == "__main__":
    build_library(host_sanitizers="--host-sanitizers" in sys.argv[1:])
    sys.exit(0)
