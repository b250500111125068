"""Build libmaze_cdna4.so in-tree with hipcc for gfx950."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libmaze_cdna4.so")
SOURCES = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
HEADERS = sorted(glob.glob(os.path.join(HERE, "csrc", "*.h"))) + \
    [os.path.join(ROOT, "include", "maze_cdna4.h")]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    "-ffp-contract=off",
    # packed-FP32 instructions are kept out of the generated code on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"),
]
OBJ_DIR = os.path.join(HERE, "csrc", "_build")
# measurement code of bench.py --store-patterns / --wave-latency: a library of its own, not linked
# into the product
PROBE_SRC = sorted(glob.glob(os.path.join(HERE, "probe", "*.hip")))
PROBE_LIB = os.path.join(HERE, "libmaze_storeprobe.so")


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def _run(cmd, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    return res.returncode


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile every csrc/*.hip to an object (side by side) and link them."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, os.path.basename(s)[:-4] + f".{os.getpid()}.o") for s in SOURCES]
    jobs = min(len(SOURCES), max(1, min(16, os.cpu_count() or 1)))
    try:
        with ThreadPoolExecutor(jobs) as pool:
            codes = list(pool.map(lambda so: _run([hipcc] + HIPCC_FLAGS + ["-c", so[0], "-o", so[1]], verbose),
                                  zip(SOURCES, objs)))
        if any(codes):
            raise RuntimeError("hipcc failed compiling libmaze_cdna4.so")
        tmp = LIB + f".tmp{os.getpid()}"
        if _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp], verbose):
            raise RuntimeError("hipcc failed linking libmaze_cdna4.so")
        os.replace(tmp, LIB)
    finally:
        for o in objs:
            if os.path.exists(o):
                os.remove(o)
    build_probe(verbose)
    return LIB


def build_probe(verbose: bool = False) -> str:
    """Compile the probes (probe/*.hip: store patterns, single-wave latencies) into their own library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = PROBE_LIB + f".tmp{os.getpid()}"
    flags = [f for f in HIPCC_FLAGS if not f.startswith("-I")]
    if _run([hipcc] + flags + ["-shared"] + PROBE_SRC + ["-o", tmp], verbose):
        raise RuntimeError("hipcc failed compiling libmaze_storeprobe.so")
    os.replace(tmp, PROBE_LIB)
    return PROBE_LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
