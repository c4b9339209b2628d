"""The header is plain C: a C99 program that includes it compiles with -pedantic -Werror,
links against the library and gets, from the entry points that need no GPU, the values the
oracle gives."""
import os
import shutil
import subprocess

import pytest

from oracle import tr_loop as LP

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2406_17404_amd")


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no C compiler")
def test_c99_program_links_and_runs(tmp_path):
    assert os.path.exists(os.path.join(PKG, "libtrjacobi.so")), "build the library first"
    exe = str(tmp_path / "c_abi_probe")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi_probe.c"), "-o", exe, "-L", PKG, "-ltrjacobi",
           "-Wl,-rpath," + PKG]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    lines = r.stdout.split("\n")
    assert [int(v) for v in lines[:3]] == [LP.splitmix64_output(1234567, k) for k in (1, 2, 3)]
    want = LP.prompt_lookup([5, 1, 9, 5, 1, 7, 5, 1], 2, 2)
    assert lines[3].split() == ["0", str(len(want))] + [str(t) for t in want]
    assert lines[4] == "-1"          # null descriptor
    assert lines[5] == "0 1"         # valid descriptor: a positive size
    assert "gfx950" in lines[6]
