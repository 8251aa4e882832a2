"""The host side of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer: the library's sources are
compiled with the sanitizers on the host pass only (the device code as always) together with tests/host_checks.c,
a plain C program that walks the host-only paths (defaults, descriptor validation, size queries, the argument
checks that come before any launch, create / destroy), and the program is run here, without a GPU."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.timeout(900)
def test_host_paths_under_asan_and_ubsan():
    from paper_2202_05008_amd import build
    if not (shutil.which("hipcc") or os.path.exists(build.HIPCC)):
        pytest.skip("no hipcc here")
    tmp = tempfile.mkdtemp(prefix="evo_san_")
    try:
        exe = build.build_checked_executable(os.path.join(ROOT, "tests", "host_checks.c"), os.path.join(tmp, "host_checks"),
                                             os.path.join(tmp, "obj"))
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        r = subprocess.run([exe], capture_output=True, text=True, timeout=120, env=env)
        assert r.returncode == 0, "exit %d\n%s\n%s" % (r.returncode, r.stdout[-2000:], r.stderr[-6000:])
        assert "host checks passed" in r.stdout
        assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-6000:]
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
