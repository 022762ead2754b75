"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer: a CPU build (hipcc, sanitizers on the
host side only) of the library with tests/host/host_checks.cpp, which drives the batch former, its virtual-clock run,
the launch planners and the validation paths over seeded inputs.  No GPU call is made.  A sanitizer report aborts the
program."""
import os
import subprocess

from paper_2512_12928_amd import build as PB

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_logic_is_clean_under_asan_and_ubsan(tmp_path):
    exe = PB.build_host_checks(str(tmp_path / "host_checks"), os.path.join(ROOT, "tests", "host", "host_checks.cpp"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert p.returncode == 0 and "host_checks ok" in p.stdout, p.stdout[-4000:]
