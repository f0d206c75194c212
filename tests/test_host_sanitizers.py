"""The host side of the library under AddressSanitizer + UndefinedBehaviorSanitizer: host_checks.cpp calls
everything that runs on the CPU before a launch (validation, launch planning, workspace sizing, the
anchor-layer selection against exhaustive search).  Sanitizers instrument host code only; device code is
compiled as usual and never launched.  Runs without a GPU."""
import os
import subprocess

from paper_2512_16391_amd import build

HERE = os.path.dirname(os.path.abspath(__file__))


def test_host_code_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "host_checks")
    srcs = [os.path.join(build.CSRC, s) for s in build.SOURCES]
    cmd = [build.hipcc_path(), "--offload-arch=gfx950", "-O1", "-std=c++17", "-fno-omit-frame-pointer",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-parallel-jobs=4", os.path.join(HERE, "host_checks.cpp"), *srcs, "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "host checks passed" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
