"""The library's host side (argument checks, planner, workspace sizes, partition functions, plan table) under
AddressSanitizer and UndefinedBehaviorSanitizer.

prism_api.hip is compiled once more with the sanitizers on its host code and linked with a driver that stubs the
kernel launchers (tests/sanitize/planner_driver.hip), so the run needs no GPU: 60,000 random and extreme shapes
through prism_plan / prism_workspace_bytes / the entry points / the plan table, and the weighted partition's integer
functions over random geometries.  Any sanitizer report (signed overflow, out-of-range shift, bad index) fails."""
import os
import shutil
import subprocess

import pytest


def test_planner_runs_clean_under_asan_and_ubsan(repo_root, tmp_path):
    hipcc = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else shutil.which("hipcc")
    if hipcc is None:
        pytest.skip("hipcc not found: the sanitizer build needs the HIP compiler")
    csrc = os.path.join(repo_root, "paper_2604_15272_amd", "csrc")
    exe = str(tmp_path / "planner_driver")
    san = []
    for flag in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"):
        san += ["-Xarch_host", flag]
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops"] + san + ["-I", os.path.join(repo_root, "include"), "-I", csrc,
                                        os.path.join(csrc, "prism_api.hip"),
                                        os.path.join(repo_root, "tests", "sanitize", "planner_driver.hip"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    report = run.stdout[-3000:] + run.stderr[-6000:]
    assert run.returncode == 0, report
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, report
    assert "no check failed" in run.stdout, report
