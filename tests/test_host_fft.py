"""The ring-degree-2048 transforms of the HIP library, emulated on the host (CPU only): the header's own stage,
table and index code with the 64 lanes looped over, against the transform's definition, the inverse round trip, and
an external-product-sized sum of products against 128-bit schoolbook arithmetic (tests/host_checks/plan2048_check.cpp)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_plan2048_transforms_on_the_host(tmp_path):
    from paper_1906_00148_amd import build as B
    exe = str(tmp_path / "plan2048_check")
    subprocess.check_call([B.HIPCC, "--offload-arch=gfx950", "-O2", "-std=c++17", "-ffp-contract=off",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", B.CSRC,
                           os.path.join(ROOT, "tests", "host_checks", "plan2048_check.cpp"), "-o", exe],
                          stderr=subprocess.DEVNULL)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "failures 0" in r.stdout, r.stdout + r.stderr
