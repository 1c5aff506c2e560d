"""Host sanitizer run of the oracle and the input generator: both C sources are compiled together with a small
driver (oracle/sanitize_check.c) under -fsanitize=address,undefined and run on tiny, awkward shapes; an
out-of-bounds index, a leak or undefined arithmetic in the host code fails the test with the sanitizer's report."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_generator_under_asan_ubsan(tmp_path):
    import oracle
    exe = oracle.build_sanitize_check(str(tmp_path / "sanitize_check"))
    env = dict(os.environ)
    # the sanitizer runtime is linked statically; whatever else the environment preloads need not come after it
    env["ASAN_OPTIONS"] = "detect_leaks=1:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    sys.stdout.write(r.stdout)
    sys.stderr.write(r.stderr)
    assert r.returncode == 0, "sanitizer run failed:\n" + r.stderr[-4000:]
    assert "sanitize_check: ok" in r.stdout
