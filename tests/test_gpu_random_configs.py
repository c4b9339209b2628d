"""tr_verify_step on randomly drawn small configurations against the oracle: model shape
(heads, K/V heads, head size, widths that are not powers of two), dtype, number of packed
sequences, tree sizes on both sides of every row-tile boundary (32, 64, 96, 128), prefix
lengths on both sides of a K/V block boundary, and planted drafts so that accepted paths are
not all trivial.  Every case is seeded; the checks are those of test_gpu_step.py."""
import numpy as np
import pytest

from oracle import tr_oracle as O
from paper_2406_17404_amd import inputs as I
from test_gpu_step import TOL, prefix_normal, run_and_check

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(9000 + seed)
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    dh = int(rng.choice([64, 128])) if dtype == "bf16" else int(rng.choice([32, 64]))
    n_kv = int(rng.choice([1, 2, 4]))
    group = int(rng.choice([1, 1, 2, 4]))
    H = n_kv * group
    d = int(rng.choice([128, 192, 256, 320]))
    F = int(rng.choice([256, 352, 704]))
    V = int(rng.choice([96, 512, 1056]))
    shape = I.ModelShape(int(rng.integers(1, 3)), d, H, dh, F, V, dtype, 1e-5, 10000.0,
                         0 if group == 1 else n_kv)
    B = int(rng.choice([1, 1, 2, 3, 5]))
    sizes = [int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128])) for _ in range(B)]
    if sum(sizes) > 400:                       # keep the oracle's work small
        sizes = [min(n, 64) for n in sizes]
    lens = [int(rng.choice([0, 1, 31, 32, 33, 100, 255, 256, 300])) for _ in range(B)]
    return shape, rng, sizes, lens


@pytest.mark.parametrize("seed", range(24))
def test_random_configuration(seed):
    shape, rng, sizes, lens = draw_case(seed)
    w = I.gen_weights(shape, 77 + seed)
    trees = [I.tree_random(n, rng) if rng.random() < 0.7 else I.tree_chain(n) for n in sizes]
    toks = [I.gen_tokens(shape.vocab, n, 77 + seed, "tree", s) for s, n in enumerate(sizes)]
    pkv = [prefix_normal(shape, 77 + seed, s, L) for s, L in enumerate(lens)]
    # plant: give the children of the root (and theirs, one level down) the oracle's own
    # greedy prediction at their parent, so that some drafts are accepted
    for s, (tree, tok, L) in enumerate(zip(trees, toks, lens)):
        if len(tree) < 3:
            continue
        kv = [(np.concatenate([k, np.zeros((k.shape[0], len(tree), k.shape[2]))], 1),
               np.concatenate([v, np.zeros((v.shape[0], len(tree), v.shape[2]))], 1)) for k, v in pkv[s]]
        for _ in range(2):
            am = O.greedy_argmax(O.decoder_tree_forward(shape, w, [(k.copy(), v.copy()) for k, v in kv],
                                                        tok, tree, L))
            for i in range(1, len(tree)):
                if tree[i] == 0 or tree[tree[i]] == 0:
                    tok[i] = am[tree[i]]
    res, summary = run_and_check(shape, w, trees, toks, lens, pkv, TOL[shape.dtype])
    print("seed", seed, shape, "sizes", sizes, "prefixes", lens, "err/accept/flips", summary)
