"""The boundary is a C ABI: a plain C client (tests/c_abi/demo.c) is compiled with gcc against include/she.h and the
built library.  Linking is checked without a GPU; running it needs one."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "c_abi", "demo.c")


def build_demo(tmp_path) -> str:
    import paper_1906_00148_amd as she
    she.load_library()                                   # builds the library only if none is there
    lib = she.lib_path()
    exe = str(tmp_path / "she_demo")
    cmd = ["gcc", "-std=c99", "-Wall", "-Werror", "-O1", "-I", os.path.join(ROOT, "include"), SRC, lib,
           "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib", "-lamdhip64", "-lstdc++", "-lm",
           "-o", exe]
    subprocess.check_call(cmd)
    return exe


def test_c_client_compiles_and_links(tmp_path):
    assert os.path.exists(build_demo(tmp_path))


@pytest.mark.gpu
def test_c_client_runs_on_the_gpu(tmp_path):
    exe = build_demo(tmp_path)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "wrong results: 0" in r.stdout
