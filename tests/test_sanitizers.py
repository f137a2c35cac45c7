"""The planner (csrc/hikonv_plan.cpp) and the C oracle under AddressSanitizer and
UndefinedBehaviorSanitizer, on the CPU: tests/sanitize_driver.cpp walks the planner's request
space (all widths, signs, modes, multiplier widths, tight, both objectives, taps up to 64, M up
to 2^20, max_N, random hand-made plans through hikonv_plan_check) and the oracle's edge shapes;
any finding aborts the run (-fno-sanitize-recover)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="needs gcc and g++")
def test_planner_and_oracle_run_clean_under_asan_and_ubsan(tmp_path):
    oracle_o = str(tmp_path / "oracle.o")
    exe = str(tmp_path / "sanitize_driver")
    subprocess.run(["gcc", "-std=c11", *FLAGS, "-c", os.path.join(ROOT, "oracle", "hikonv_oracle.c"), "-o", oracle_o],
                   check=True)
    subprocess.run(["g++", "-std=c++17", *FLAGS, os.path.join(ROOT, "tests", "sanitize_driver.cpp"),
                    os.path.join(ROOT, "paper_2208_00763_amd", "csrc", "hikonv_plan.cpp"), oracle_o, "-o", exe],
                   check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)        # the sanitizer runtime must come first in the driver's own process
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-6000:]
    assert "sanitize_driver: ok" in res.stdout
