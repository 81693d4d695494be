"""Builds libs2d2.so (the C-ABI HIP library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libs2d2.so")
SOURCES = ["api.hip", "plan.hip", "elementwise.hip", "gemm.hip", "gemm_stream.hip", "gemm_tile.hip", "moe.hip", "attention.hip", "attention_wide.hip", "vocab.hip"]
FLAGS = (["-DS2D2_KERNEL_TIMING"] if os.environ.get("S2D2_KERNEL_TIMING") else []) + ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
    os.makedirs(os.path.dirname(obj), exist_ok=True)
    cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_lib(jobs: int = 6) -> str:
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


def build_host_check() -> str:
    """Builds tests/host/host_check: the library's objects with api.hip (all host-side argument checks and size
    arithmetic) rebuilt under AddressSanitizer and UndefinedBehaviorSanitizer on the host side, linked with a driver
    that calls every entry point with extreme and invalid arguments.  Device code is not instrumented."""
    root = os.path.dirname(HERE)
    out = os.path.join(HERE, "_build", "host_check")
    objs = []
    for src in SOURCES:
        obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
        if src == "api.hip" or not os.path.exists(obj):
            obj = _compile(src) if src != "api.hip" else obj
        objs.append(obj)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xarch_host", "-fno-omit-frame-pointer"]
    api_san = os.path.join(HERE, "_build", "api_san.o")
    drv = os.path.join(HERE, "_build", "host_check.o")
    host_san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
    cmds = [[_hipcc(), *FLAGS, *san, "-c", os.path.join(CSRC, "api.hip"), "-o", api_san],
            ["/opt/rocm/lib/llvm/bin/clang++", "-O1", "-g", "-std=c++17", *host_san, "-c", os.path.join(root, "tests", "host", "host_check.cpp"), "-o", drv],
            [_hipcc(), "--offload-arch=gfx950", *host_san, "-fno-gpu-sanitize", drv, api_san,
             *[o for o in objs if not o.endswith(os.sep + "api.o")], "-o", out]]
    for cmd in cmds:
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("host check build failed:\n" + " ".join(cmd) + "\n" + r.stderr)
    return out


if __name__ == "__main__":
    print(build_lib())
