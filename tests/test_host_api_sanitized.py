"""The host half of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer: the library's sources are
compiled for the CPU only (no device code), and the host-only checks of test_host_api.py run against that build in a
child process with the sanitizer runtime loaded first.  Any report (a read past an argument array, an invalid enum
load, signed overflow in the layout arithmetic, ...) ends the child with an error."""
import glob
import os
import subprocess
import sys

import pytest

from paper_2406_11209_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_api_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    try:
        lib, runtime = build.build_host_sanitized(str(tmp_path / "san"))
    except RuntimeError as e:
        if "hipcc not found" in str(e):
            pytest.skip("hipcc not found")
        raise
    if not os.path.exists(runtime):
        pytest.skip("no shared AddressSanitizer runtime next to the compiler")
    env = dict(os.environ)
    log = str(tmp_path / "report")
    # the sanitizer runtime has to come first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = " ".join([runtime] + env.get("LD_PRELOAD", "").split())
    env["ASAN_OPTIONS"] = "detect_leaks=0:log_path=" + log        # the interpreter's own allocations are not the subject
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:log_path=" + log
    env["PBZ_LIBRARY"] = lib
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_host_api.py"), "-q", "-x",
                          "-p", "no:cacheprovider"], env=env, cwd=ROOT, capture_output=True, text=True, timeout=600)
    reports = "".join(open(f).read() for f in glob.glob(log + "*"))
    assert res.returncode == 0 and not reports, res.stdout[-3000:] + res.stderr[-3000:] + reports[:6000]
    assert " passed" in res.stdout and "failed" not in res.stdout
