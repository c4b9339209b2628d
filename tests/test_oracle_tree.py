"""Pins for the oracle's tree bookkeeping (depth, ancestor-or-self mask) against closed
forms: the sparse mask of the appendix "Templates for Token Tree" is exactly "node j is
on the path from the root to node i"."""
import numpy as np
import pytest

from oracle import tr_oracle as O
from paper_2406_17404_amd import inputs as I


def walk(parent, i):
    s = set()
    while i != -1:
        s.add(i)
        i = int(parent[i])
    return s


def test_chain_is_lower_triangular():
    p = I.tree_chain(9)
    assert (O.ancestor_mask(p) == np.tril(np.ones((9, 9), bool))).all()
    assert (O.tree_depth(p) == np.arange(9)).all()


def test_star_is_root_plus_self():
    n = 7
    p = np.array([-1] + [0] * (n - 1), np.int32)
    m = O.ancestor_mask(p)
    want = np.eye(n, dtype=bool)
    want[:, 0] = True
    assert (m == want).all()
    assert (O.tree_depth(p) == np.array([0] + [1] * (n - 1))).all()


def test_c0_tree_shape():
    p = I.tree_c0()
    d = O.tree_depth(p)
    assert list(d) == [0, 1, 2, 3, 4, 1, 2, 3, 4, 5, 1, 2, 3, 4, 5]
    m = O.ancestor_mask(p)
    # node 9 = end of the first retrieval branch: sees root and 5..9 only
    assert set(np.nonzero(m[9])[0]) == {0, 5, 6, 7, 8, 9}
    assert set(np.nonzero(m[4])[0]) == {0, 1, 2, 3, 4}


@pytest.mark.parametrize("n,seed", [(2, 0), (16, 1), (64, 2), (65, 3), (128, 4)])
def test_random_tree_mask_by_walking(n, seed):
    p = I.tree_random(n, np.random.default_rng(seed))
    m = O.ancestor_mask(p)
    bits = O.ancestor_bits(p)
    d = O.tree_depth(p)
    for i in range(n):
        s = walk(p, i)
        assert set(np.nonzero(m[i])[0]) == s
        assert d[i] == len(s) - 1
        got = {j for j in range(128) if (int(bits[i, j // 64]) >> (j % 64)) & 1}
        assert got == s
        assert O.root_path(p, i) == sorted(s, key=lambda j: d[j])


def test_generators_respect_their_recipes():
    rng = np.random.default_rng(5)
    p = I.tree_c1(64, rng)
    assert list(p[:8]) == [-1, 0, 1, 2, 3, 4, 5, 6]
    assert O.validate_tree(p) and O.tree_depth(p).max() <= 8
    p3 = I.tree_c3(128, rng)
    assert O.validate_tree(p3) and list(p3[:16]) == list(range(-1, 15))
    d3 = O.tree_depth(p3)
    starts = [i for i in range(16, 128) if p3[i] == 0]
    assert starts[0] == 16
    lens = np.diff(starts + [128])
    assert (lens[:-1] >= 4).all() and (lens <= 12).all()
    assert d3[16:].max() <= 12


def test_validate_tree():
    assert O.validate_tree(np.array([-1]))
    assert O.validate_tree(np.array([-1, 0, 0, 2]))
    assert not O.validate_tree(np.array([0, 0]))          # root must be -1
    assert not O.validate_tree(np.array([-1, 1]))         # parent must precede
    assert not O.validate_tree(np.array([-1, 0, 3, 1]))
    assert not O.validate_tree(np.array([-1, -1]))
    assert not O.validate_tree(np.array([], np.int32))
