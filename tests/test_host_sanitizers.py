"""The library's host code (planner, descriptor builder, plan objects, plan cache, error paths) under
AddressSanitizer + UndefinedBehaviorSanitizer: csrc/host_selftest.cpp built and run by build.py --sanitize."""
import subprocess

from paper_2112_01075_amd.build import build_host_selftest


def test_host_code_is_clean_under_asan_and_ubsan():
    exe = build_host_selftest(sanitize=True)
    proc = subprocess.run([exe, "150"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert proc.returncode == 0, proc.stdout[-3000:]
    assert "host self-test ok" in proc.stdout and "runtime error" not in proc.stdout and "AddressSanitizer" not in proc.stdout
