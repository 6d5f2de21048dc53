"""What the compiler made of a few lines the kernels depend on (CPU: hipcc cross-compiles gfx950 to assembly)."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2512_19849_amd", "csrc")
HIPCC = "/opt/rocm/bin/hipcc"


def _assembly(src, tmp_path):
    out = tmp_path / (src + ".s")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                    "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", str(out), os.path.join(CSRC, src)],
                   check=True, stderr=subprocess.DEVNULL)
    return out.read_text()


def _kernel_body(asm, mangled):
    start = asm.index("\n" + mangled + ":")
    end = asm.index(".end_amdhsa_kernel", start)
    return asm[start:end]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_combine_keeps_cached_and_streaming_loads_apart(tmp_path):
    """The combine kernel reads just-dispatched rows with cached loads and all others with streaming (nt) loads,
    in two loops that differ in nothing else; an optimiser that folds them drops the hint (seen: all loads
    became cached ones, combine 98 -> 111 us).  Both kinds must be there, as many of one as of the other."""
    asm = _assembly("combine.hip", tmp_path)
    for mangled in ("_ZN2ep14combine_kernelILi1ELi8EEEvNS_11CombineArgsE",
                    "_ZN2ep14combine_kernelILi1ELi2EEEvNS_11CombineArgsE"):
        loads = re.findall(r"global_load_dwordx4[^\n]*", _kernel_body(asm, mangled))
        nt = [l for l in loads if re.search(r"\bnt\b", l)]
        assert len(nt) > 0 and len(nt) * 2 == len(loads), (mangled, len(nt), len(loads))
