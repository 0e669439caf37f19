"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the library's CSR encoder,
planner and C ABI (built without kernels) and the CPU oracle, linked with tests/sanitize/driver.cpp,
run random layers, geometries and launch overrides; the driver byte-compares every CSR with the oracle's
and checks every plan, and any sanitizer report fails the run."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_address_and_ub_sanitizers():
    from paper_2011_06295_amd import build as libbuild
    exe = libbuild.build_sanitize()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "sanitize driver: ok" in res.stdout and "runtime error" not in res.stdout
