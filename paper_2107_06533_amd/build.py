"""Build the HIP shared library in-tree for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkfac_hip.so")
SOURCES = ["kfac_api.hip", "tile_kernels.hip", "inverse_kernels.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


SANITIZE_HOST = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-omit-frame-pointer", "-g", "-O1"]


def build(verbose: bool = True, extra_flags=tuple(os.environ.get("KFAC_EXTRA_FLAGS", "").split()),
          sanitize_host_dir: str | None = None) -> str:
    """Compile every HIP source and link libkfac_hip.so next to this file.

    sanitize_host_dir: build a second library there instead, whose HOST code (argument validation,
    the planners' index arithmetic) is instrumented with the address and undefined-behaviour
    sanitizers; device code is unchanged.  Run the host-only tests on it with
        LD_PRELOAD=$(ls /opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so) \
        ASAN_OPTIONS=detect_leaks=0 KFAC_HIP_LIBRARY=<dir>/libkfac_hip.so python -m pytest tests/test_api_host.py
    (GPU sanitizers are not used)."""
    objdir = sanitize_host_dir or os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()
    lib = os.path.join(sanitize_host_dir, "libkfac_hip.so") if sanitize_host_dir else LIB
    if sanitize_host_dir:
        extra_flags = tuple(extra_flags) + tuple(SANITIZE_HOST)

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                        if "packed-fp32-ops" not in l)       # the host pass does not know this device feature
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{out}")
        if verbose and out.strip():
            print(out, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(4, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    link_extra = ["-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize"] if sanitize_host_dir else []
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *link_extra, *objs, "-o", lib]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    if verbose:
        print(f"built {lib}", file=sys.stderr)
    return lib


if __name__ == "__main__":
    if len(sys.argv) == 3 and sys.argv[1] == "--sanitize-host":
        build(sanitize_host_dir=sys.argv[2])
    else:
        build()
