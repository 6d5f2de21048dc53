"""The boundary is a C ABI: the public header must compile as strict C99 and a plain C program must be able
to drive the library through it (host-only handle: no GPU needed)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib_dir():
    import paper_2512_19849_amd as ep
    ep.load_library()
    return os.path.dirname(ep.lib_path())


def test_header_is_strict_c99(tmp_path):
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    src = tmp_path / "only_header.c"
    src.write_text('#include "ep.h"\n#include "ep_diag.h"\nint main(void) { return sizeof(ep_config) > 0 ? 0 : 1; }\n')
    subprocess.run(["gcc", "-std=c99", "-pedantic-errors", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)


def test_plain_c_program_drives_the_library(tmp_path, lib_dir):
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    exe = str(tmp_path / "c_consumer")
    subprocess.run(["gcc", "-std=c99", "-pedantic-errors", "-Wall", "-Wextra", "-Werror", "-O1",
                    os.path.join(ROOT, "tests", "native", "c_consumer.c"), "-o", exe,
                    "-L", lib_dir, "-l:libep.so", f"-Wl,-rpath,{lib_dir}", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    p = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert p.returncode == 0, p.stdout + p.stderr
    assert "cmds 2 writes 1 atomics_applied 1 rejected 0 count[5] 1" in p.stdout
