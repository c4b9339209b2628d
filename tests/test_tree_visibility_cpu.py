"""The predicate with which the attention kernels decide which keys a tree node sees,
compiled for the host with -fsanitize=undefined (so a shift count outside 0..63 or any
other undefined operation aborts) and compared, for every prefix length modulo the
32-slot block, every node and every key slot around the tree's slots, with the tree's
definition (the oracle's ancestor mask): prefix slots visible, slot L + j visible iff j
is on the node's root path, nothing visible past the tree's last node."""
import ctypes as C
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import tr_oracle as O
from paper_2406_17404_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_visibility_predicate_exhaustively_under_ubsan(tmp_path):
    so = str(tmp_path / "libtree_vis_probe.so")
    r = subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-shared", "-fPIC", "-fsanitize=undefined",
                        "-fno-sanitize-recover=all", os.path.join(ROOT, "tests", "tree_vis_probe.cpp"), "-o", so],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    lib = C.CDLL(so)
    lib.trj_test_visible.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_void_p]
    rng = np.random.default_rng(7)
    trees = [I.tree_chain(128), I.tree_random(128, rng), I.tree_c1(66, rng), I.tree_c3(128, rng),
             I.tree_random(65, rng), I.tree_random(64, rng), I.tree_c0(), np.asarray([-1], np.int32)]
    checked = 0
    for parent in trees:
        n = len(parent)
        mask = O.ancestor_mask(parent)
        bits = np.ascontiguousarray(O.ancestor_bits(parent))
        for L in list(range(0, 70)) + [1024, 4095, 4096, 2**30]:
            key0 = max(0, L - 40)
            n_keys = L - key0 + 128 + 70         # some prefix slots, all tree slots, slots past node 127
            out = np.zeros((n, n_keys), np.uint8)
            lib.trj_test_visible(L, key0, n_keys, bits.ctypes.data, n, out.ctypes.data)
            want = np.zeros((n, n_keys), bool)
            want[:, :L - key0] = True
            want[:, L - key0:L - key0 + n] = mask
            assert np.array_equal(out.astype(bool), want), (n, L)
            checked += out.size
    assert checked > 10**6
