"""Builds libep.so (HIP kernels + host proxy) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libep.so")
SOURCES = ["layout.hip", "dispatch.hip", "combine.hip", "ht_ring.hip", "service.hip", "proxy.cpp", "api.cpp"]
HEADERS = ["ep_internal.h", "ep_device.h", "ep_host.h", os.path.join("..", "..", "include", "ep.h"),
           os.path.join("..", "..", "include", "ep_diag.h")]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build_lib(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP/C++ source of the library for gfx950 into libep.so."""
    if not force and not stale():
        return LIB
    objs = []
    common = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function"]
    for src in SOURCES:
        obj = os.path.join(CSRC, src + ".o")
        cmd = [hipcc(), *common, "-c", os.path.join(CSRC, src), "-o", obj]
        if src.endswith(".hip"):
            # packed fp32 ALU forms are kept off for all device code
            cmd[1:1] = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
        objs.append(obj)
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs, "-lpthread"]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


PROBE_SRC = os.path.join(HERE, "probes", "mem_patterns.hip")
PROBE_BIN = os.path.join(HERE, "probes", "mem_patterns")


def build_probes(verbose: bool = False) -> str:
    """The stand-alone access-pattern probe (a measuring program for rocprofv3, not part of the library)."""
    cmd = [hipcc(), "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", PROBE_SRC, "-o", PROBE_BIN]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return PROBE_BIN


if __name__ == "__main__":
    print(build_lib(verbose=True))
    print(build_probes(verbose=True))
