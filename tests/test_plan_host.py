"""Host logic of the library under sanitizers: the planner (csrc/plan.h) is compiled into a small
harness (tests/host/plan_fuzz.hip) with AddressSanitizer and UndefinedBehaviorSanitizer on the host
side only, and swept over seeded shapes, forced tilings, contraction tiles, accumulator forms and
row-skipping budgets; the same harness walks the workgroup-id -> work-item mappings of the kernels
(csrc/wg_map.h) over every grid size and checks that each is one-to-one.  No GPU: without a device the
planner assumes 256 compute units."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_planner_fuzz_under_asan_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "plan_fuzz")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           os.path.join(ROOT, "tests", "host", "plan_fuzz.hip"), "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True, cwd=str(tmp_path))
    assert res.returncode == 0, res.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe, "2500"], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "iterations ok" in run.stdout
