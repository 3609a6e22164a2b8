"""The host side of the library (allocator, block tables, reference counts, undo of half-done calls)
under AddressSanitizer and UndefinedBehaviorSanitizer: a native driver walks the C ABI at random on
metadata-only pools and checks a shadow model; any sanitizer report or mismatch fails the test."""
import os
import subprocess
import tempfile

from paper_2605_13784_amd import _build

HERE = os.path.dirname(os.path.abspath(__file__))


def test_random_walk_over_the_host_library_under_asan_and_ubsan():
    with tempfile.TemporaryDirectory() as tmp:
        exe = _build.build_host_check(os.path.join(HERE, "host_sanitize_driver.cpp"), os.path.join(tmp, "host_check"))
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        r = subprocess.run([exe, "12000"], capture_output=True, text=True, timeout=600, env=env)
        assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-6000:]
        assert "host walk ok" in r.stdout
        assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
