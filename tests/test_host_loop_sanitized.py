"""The decoding loop's host logic (ahead noise, prompt lookup, tree refill: plain C++ with
no GPU dependency) built on its own under AddressSanitizer and
UndefinedBehaviorSanitizer and checked against the oracle in a child process.  Runs on the
CPU; the GPU kernels cannot be sanitized on this pool."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    r = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True)
    p = r.stdout.strip()
    return p if os.path.isabs(p) and os.path.exists(p) else None


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_host_logic_under_address_and_ub_sanitizers(tmp_path):
    asan, ubsan = _runtime("libasan.so"), _runtime("libubsan.so")
    if not asan or not ubsan:
        pytest.skip("sanitizer runtimes not installed")
    from paper_2406_17404_amd import build
    lib = build.build_host_logic_sanitized(str(tmp_path / "libtrj_loop_host_san.so"))
    env = dict(os.environ)
    # the sanitizer runtime must come first in the loader's list; whatever is preloaded
    # already stays behind it
    env["LD_PRELOAD"] = ":".join([asan, ubsan] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else []))
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, os.path.join(ROOT, "tests", "host_loop_sanitized_driver.py"), lib],
                       capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "random cases equal the oracle" in r.stdout
