"""The integer plan shared by the kernels and the host (paper_2506_01969_amd/csrc/mla_plan.h), checked on
the CPU under AddressSanitizer and UndefinedBehaviorSanitizer by tests/c/plan_check_main.cpp: unit
coverage, the agreement of the split and combine partitions, slot uniqueness and workspace bounds,
and the bounds of every address the kernels form from the plan."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_plan_rules_exhaustively_under_sanitizers(tmp_path):
    exe = str(tmp_path / "plan_check")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-Wall", "-Wextra", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",
           "-I" + os.path.join(ROOT, "paper_2506_01969_amd", "csrc"),
           os.path.join(ROOT, "tests", "c", "plan_check_main.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    res = subprocess.run([exe], capture_output=True, text=True, env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"), timeout=300)
    assert res.returncode == 0 and res.stdout.startswith("ok "), res.stdout + res.stderr
