"""CPU-only: the planner and the argument checks of the C ABI, built for the host with
AddressSanitizer and UndefinedBehaviorSanitizer and run without a GPU (no device code is
sanitized: the kernel launchers are replaced by stand-ins)."""
import os
import subprocess

from paper_2506_17974_amd import build as b


def test_host_code_under_asan_and_ubsan():
    exe = b.build_host_sanitize(verbose=False)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert p.returncode == 0, p.stdout[-4000:]
    assert "all checks passed" in p.stdout
    assert "ERROR: AddressSanitizer" not in p.stdout and "runtime error:" not in p.stdout, p.stdout[-4000:]
