"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU call): the C oracle through a
small driver, and the library's host-only calls (netlist builders, folding, scheduling, argument checks) with the whole
library built with the sanitizers on the host side only.  GPU code is never instrumented."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-ffp-contract=off", os.path.join(ROOT, "oracle", "tfhe_oracle.c"),
                           os.path.join(HERE, "oracle_driver.c"), "-lm", "-o", exe])
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "wrong results 0" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_library_host_calls_under_sanitizers(tmp_path):
    from paper_1906_00148_amd import build as B
    exe = str(tmp_path / "plan_san")
    flags = [f for f in B.FLAGS if f not in ("-shared", "-O3")] + ["-O1", "-g"]
    # the sanitizers instrument the host side only: each -fsanitize= follows an -Xarch_host
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined"]
    cmd = [B.HIPCC] + flags + san + ["-I", os.path.join(ROOT, "include")] + [os.path.join(B.CSRC, s) for s in B.SOURCES] + \
          [os.path.join(HERE, "plan_driver.cpp"), "-o", exe]
    subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "failures 0" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
    # the instrumented build plans like the ordinary one
    import numpy as np

    import paper_1906_00148_amd as pkg
    sign = np.array([1, -1, 1, 1, -1, 1, -1, -1, 1, 1, 1, -1, 1, 1, -1, -1, 1, 1], np.int8).reshape(2, 9)
    exp = np.array([0, -1, -7, -2, 0, -3, 0, -6, -1, -4, 0, 0, -2, -5, -1, 0, -3, -2], np.int8).reshape(2, 9)
    seen = {(int(m), int(b)): (int(g), int(lv)) for m, b, g, lv in
            re.findall(r"shift_acc mode (\d+) bias (\d+): rc 0 gates (\d+) levels (\d+)", r.stdout)}
    assert len(seen) == 10
    for (mode, withb), got in seen.items():
        want = pkg.plan_shift_acc(2, 9, 8, sign, exp, 16, bool(mode & 1), bool(mode & 4), bool(mode & 8),
                                  bias=[1000, -77] if withb else None)
        assert got == want, (mode, withb)
    assert f"accumulator bits {pkg.plan_accumulator_bits(sign, exp, 8, [1000, -77])}" in r.stdout
