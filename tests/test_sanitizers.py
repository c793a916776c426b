"""CPU test: the library's host code (validation, planner, scheduler, the entry points' bookkeeping) and the fp64
checker, built with AddressSanitizer and UndefinedBehaviorSanitizer (CPU build only; the GPU code is not part of
it) and driven by tests/sanitize/host_paths.cpp, whose stand-ins for the kernel launchers walk exactly the
metadata the kernels read.  Any report from either sanitizer fails the run."""
import os
import subprocess

from paper_2403_02310_amd import build


def test_host_paths_and_checker_are_clean_under_asan_and_ubsan(tmp_path):
    exe = build.build_sanitized_host(str(tmp_path))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-6000:]
    assert "host paths clean" in res.stdout
    assert "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr, res.stderr[-6000:]
