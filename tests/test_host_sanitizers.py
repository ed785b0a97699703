"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU needed): the argument validation of every
C-ABI entry point, the batch former / depth calibration / alignment check on random traffic, and the seeded
generators, driven by tests/host_sanitize/driver.cpp.  The build compiles the library's sources with the sanitizers on
the host code only."""
import os
import subprocess
import tempfile


def test_host_code_is_clean_under_asan_and_ubsan():
    from paper_2505_17052_amd import build
    with tempfile.TemporaryDirectory(prefix="sev_hostsan_") as d:
        exe = build.build_host_sanitized(d)
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
        if "LeakSanitizer has encountered a fatal error" in r.stderr:      # no ptrace in this sandbox: leaks cannot be checked
            env["ASAN_OPTIONS"] = "detect_leaks=0"
            r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
        assert r.returncode == 0, r.stdout + r.stderr
        assert "all checks passed" in r.stdout
        for bad in ("AddressSanitizer", "runtime error", "LeakSanitizer"):
            assert bad not in r.stderr, r.stderr
