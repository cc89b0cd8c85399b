"""Builds libcnnmem.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB_PATH = os.path.join(HERE, "libcnnmem.so")
SOURCES = ["api.hip", "transform.hip", "permute.hip", "pool.hip", "softmax.hip", "storage16.hip", "backward.hip"]
# host-only hooks of the CPU test-suite (include/cnnmem_debug.h): a library of their own, so that the product
# exports nothing but the C ABI; it carries the two translation units whose host code the hooks call
HOOKS_LIB_PATH = os.path.join(HERE, "libcnnmem_testhooks.so")
HOOKS_SOURCES = ["testhooks.hip"]
HOOKS_NEEDS = ["permute.hip", "transform.hip"]
# memory-system probes of `bench.py --workload access_patterns` (measurement support, a library of their own)
PROBES_LIB_PATH = os.path.join(HERE, "libcnnmem_probes.so")
PROBES_SOURCES = ["probes.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fvisibility=hidden", "-fno-gpu-rdc",
    # packed fp32 VALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]
BUILD_DIR = os.path.join(HERE, "_build")


def stale() -> bool:
    """True when the library is missing or older than any file under csrc/ or include/."""
    if not os.path.exists(LIB_PATH) or not os.path.exists(HOOKS_LIB_PATH):
        return True
    built = min(os.path.getmtime(LIB_PATH), os.path.getmtime(HOOKS_LIB_PATH))
    for folder in (CSRC, INCLUDE):
        for name in os.listdir(folder):
            if os.path.getmtime(os.path.join(folder, name)) > built:
                return True
    return False


def build(verbose: bool = False, jobs: int = 8) -> str:
    """Compile every HIP source (in parallel) and link ``paper_1610_03618_amd/libcnnmem.so``."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    pending = []
    for name in SOURCES + HOOKS_SOURCES + PROBES_SOURCES:
        obj = os.path.join(BUILD_DIR, os.path.splitext(name)[0] + ".o")
        cmd = [HIPCC] + FLAGS + ["-I", INCLUDE, "-I", CSRC, "-c", os.path.join(CSRC, name), "-o", obj]
        pending.append((cmd, obj))
    objs, running = [], []
    for cmd, obj in pending:
        if verbose:
            print(" ".join(cmd), flush=True)
        running.append((subprocess.Popen(cmd), cmd))
        objs.append(obj)
        if len(running) >= jobs:
            proc, c = running.pop(0)
            if proc.wait() != 0:
                raise subprocess.CalledProcessError(proc.returncode, c)
    for proc, c in running:
        if proc.wait() != 0:
            raise subprocess.CalledProcessError(proc.returncode, c)
    def obj_of(name):
        return os.path.join(BUILD_DIR, os.path.splitext(name)[0] + ".o")

    for sources, path in ((SOURCES, LIB_PATH), (HOOKS_SOURCES + HOOKS_NEEDS, HOOKS_LIB_PATH),
                          (PROBES_SOURCES, PROBES_LIB_PATH)):
        link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-Wl,--no-undefined"] + \
            [obj_of(n) for n in sources] + ["-o", path]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True)
    print(LIB_PATH)
    sys.exit(0)
