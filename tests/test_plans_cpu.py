"""Host-side work lists of the streaming products, swept on the CPU under AddressSanitizer and
UndefinedBehaviorSanitizer: tests/plan_sweep.cpp includes the very header the library builds its
plans with (csrc/bbmm_plan.h) and asserts, over many sizes, compute-unit counts and workgroup
counts, that every (strip, 16-row step) is covered exactly once and every slot index is in range."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_plan_builders_cover_every_unit_exactly_once_under_sanitizers(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host C++ compiler")
    exe = tmp_path / "plan_sweep"
    subprocess.run([gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-I", os.path.join(ROOT, "paper_1809_11165_amd", "csrc"),
                    os.path.join(ROOT, "tests", "plan_sweep.cpp"), "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1")
    env.pop("LD_PRELOAD", None)
    proc = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600, env=env)
    assert proc.returncode == 0, proc.stderr[-3000:]
    assert proc.stdout.startswith("OK ")
