"""The layout builder (csrc/am_layout.cpp, pure C++) under AddressSanitizer and
UndefinedBehaviorSanitizer on the CPU: tests/layout_sanitize.cpp is compiled together with it by g++
with -fsanitize=address,undefined and run; it builds hundreds of layouts (random lists under random
tuning values, crafted lists, the 2^31 / 2^48 limits, flag combinations) and checks the work tables
with arithmetic of its own.  Any sanitizer report aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_layout_builder_under_address_and_ub_sanitizers(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "layout_sanitize")
    # the sanitizer runtimes are linked statically: the program then does not depend on being the first
    # library the loader sees, whatever else the environment loads into a process
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-Wall", "-Wextra", "-fsanitize=address,undefined",
           "-static-libasan", "-static-libubsan", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           os.path.join(ROOT, "tests", "layout_sanitize.cpp"),
           os.path.join(ROOT, "paper_2406_16793_amd", "csrc", "am_layout.cpp"), "-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert res.returncode == 0, res.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, env=env)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "layout checks passed" in run.stdout
