"""Host-side integer logic of the decoding loop (ahead noise, prompt lookup, tree
refill) in the C-ABI library against the oracle's, element by element.  These functions
never touch the GPU, so the comparison runs anywhere the library loads."""
import numpy as np
import pytest

from oracle import tr_loop as LP
from paper_2406_17404_amd import binding as b
from paper_2406_17404_amd import inputs as I
from test_oracle_loop import template


def test_splitmix64_matches():
    for seed in (0, 1234567, 2**64 - 1, 0xDEADBEEFCAFEF00D):
        for k in (1, 2, 3, 1000, 2**40 + 7):
            assert b.trj_splitmix64(seed, k) == LP.splitmix64_output(seed, k)


def test_ahead_noise_matches():
    rng = np.random.default_rng(0)
    for _ in range(200):
        ctx = list(rng.integers(0, 32000, size=rng.integers(1, 300)))
        seed, step, node = int(rng.integers(0, 2**63)), int(rng.integers(0, 5000)), int(rng.integers(0, 128))
        assert b.trj_ahead_noise(ctx, seed, step, node) == LP.ahead_noise(ctx, seed, step, node)


@pytest.mark.parametrize("alphabet", [2, 3, 8])
def test_prompt_lookup_matches(alphabet):
    rng = np.random.default_rng(alphabet)
    for _ in range(500):
        ctx = list(rng.integers(0, alphabet, size=rng.integers(1, 40)))
        ng, r = int(rng.integers(1, 6)), int(rng.integers(0, 8))
        assert b.trj_prompt_lookup(ctx, ng, r) == LP.prompt_lookup(ctx, ng, r)


@pytest.mark.parametrize("seed", range(10))
def test_fill_tree_matches(seed):
    rng = np.random.default_rng(seed)
    for _ in range(30):
        r = int(rng.integers(0, 6))
        parent = template(int(rng.integers(1, 128 - r)), r, rng)
        n = len(parent)
        ctx = list(rng.integers(0, 6, size=rng.integers(1, 50)))
        argmax = rng.integers(0, 32000, size=n).astype(np.int32)
        best = int(rng.integers(0, n))
        s, step, ng = int(rng.integers(0, 2**62)), int(rng.integers(0, 100)), int(rng.integers(1, 4))
        got0 = b.trj_fill_tree(parent, r, ctx, ng, s, step)
        assert got0 == list(LP.fill_tree(parent, r, ctx, ng, s, step))
        got = b.trj_fill_tree(parent, r, ctx, ng, s, step, argmax, best)
        assert got == list(LP.fill_tree(parent, r, ctx, ng, s, step, argmax, best))


def test_full_size_template():
    parent = template(123, 5, np.random.default_rng(3))
    assert len(parent) == 128
    argmax = np.arange(128, dtype=np.int32)
    got = b.trj_fill_tree(parent, 5, [1, 2, 3, 1, 2], 3, 5, 7, argmax, 127)
    assert got == list(LP.fill_tree(parent, 5, [1, 2, 3, 1, 2], 3, 5, 7, argmax, 127))


def test_bad_arguments_are_errors():
    with pytest.raises(b.TrjError):   # last two nodes are not a chain below the root
        b.trj_fill_tree([-1, 0, 0], 2, [1], 3, 0, 0)
    with pytest.raises(b.TrjError):   # parent after child
        b.trj_fill_tree([-1, 2, 0], 0, [1], 3, 0, 0)
    with pytest.raises(b.TrjError):
        b.trj_fill_tree([-1] + [0] * 128, 0, [1], 3, 0, 0)
    with pytest.raises(b.TrjError):
        b.trj_fill_tree([-1, 0], 0, [1], 3, 0, 0, [5, 6], 2)   # accepted node out of range
    with pytest.raises(b.TrjError):
        b.trj_prompt_lookup([1, 2], 0, 2)
