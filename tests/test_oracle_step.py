"""Pins for the oracle's verify step: brute force with a separately written causal
model (tree verification must not change what plain greedy decoding produces, section
"Speculative Decoding"; each path is an ordinary Jacobi step, section "TR-Jacobi
Decoding"), planted acceptance cases, enumeration of all paths, and the compaction
invariant."""
import itertools

import numpy as np
import pytest

import brute_force_lm as B
from oracle import tr_oracle as O
from paper_2406_17404_amd import inputs as I

SMALL = I.ModelShape(2, 32, 2, 16, 64, 50, "f32")


def setup(shape, seed, L, std=0.3):
    """Weights with a larger spread than the workloads' 0.02 so that logits are well
    separated, a prefix of L random tokens and its K/V from the brute-force model."""
    w = I.gen_weights(shape, seed)
    rng = np.random.default_rng(seed)
    for k in ("embed", "w_lm"):
        w[k] = rng.standard_normal(w[k].shape) * std
    for lw in w["layers"]:
        for k in ("wqkv", "wo", "w_gate_up", "w_down"):
            lw[k] = rng.standard_normal(lw[k].shape) * std
        lw["g_attn"] = 1 + 0.1 * rng.standard_normal(shape.d_model)
        lw["g_ffn"] = 1 + 0.1 * rng.standard_normal(shape.d_model)
    w["g_final"] = 1 + 0.1 * rng.standard_normal(shape.d_model)
    prefix = rng.integers(0, shape.vocab, size=L)
    _, pkv = B.causal_forward(shape, w, prefix) if L else (None, None)
    return w, prefix, pkv


def make_cache(shape, pkv, L, n):
    kv = []
    for l in range(shape.n_layers):
        K = np.full((shape.n_heads, L + n + 3, shape.head_dim), np.nan)
        V = np.full_like(K, np.nan)
        if L:
            K[:, :L], V[:, :L] = pkv[l]
        kv.append((K, V))
    return kv


@pytest.mark.parametrize("seed,L,n", [(0, 7, 9), (1, 1, 12), (2, 0, 6), (3, 16, 15)])
def test_node_logits_equal_causal_forward_over_root_path(seed, L, n):
    w, prefix, pkv = setup(SMALL, seed, L)
    rng = np.random.default_rng(100 + seed)
    parent = I.tree_c0() if n == 15 else I.tree_random(n, rng)
    tok = rng.integers(0, SMALL.vocab, size=n)
    kv = make_cache(SMALL, pkv, L, n)
    logits = O.decoder_tree_forward(SMALL, w, kv, tok, parent, L)
    for i in range(n):
        path = O.root_path(parent, i)
        string = list(prefix) + [int(tok[j]) for j in path]
        want, wkv = B.causal_forward(SMALL, w, string)
        assert np.allclose(logits[i], want[-1], rtol=1e-9, atol=1e-11), i
        # the K/V written for node i are the causal model's K/V of its last token
        for l in range(SMALL.n_layers):
            assert np.allclose(kv[l][0][:, L + i], wkv[l][0][:, -1], rtol=1e-9, atol=1e-11)
            assert np.allclose(kv[l][1][:, L + i], wkv[l][1][:, -1], rtol=1e-9, atol=1e-11)


def test_root_only_tree_is_one_autoregressive_step():
    w, prefix, pkv = setup(SMALL, 5, 6)
    kv = make_cache(SMALL, pkv, 6, 1)
    r = O.tr_verify_step(SMALL, w, kv, np.array([11]), np.array([-1]), 6)
    assert r["accept_len"] == 0 and r["path"] == [0] and r["new_len"] == 7
    assert r["bonus"] == B.greedy_decode(SMALL, w, list(prefix) + [11], 1)[0]


@pytest.mark.parametrize("mismatch_at", [None, 1, 2, 4])
def test_planted_greedy_drafts_are_accepted(mismatch_at):
    """Chain drafts planted equal to the greedy continuation are all accepted; a
    mismatch planted at depth k leaves k-1 accepted drafts."""
    L, n = 5, 6
    w, prefix, pkv = setup(SMALL, 7, L)
    root = 3
    greedy = B.greedy_decode(SMALL, w, list(prefix) + [root], n)  # n tokens
    tok = np.array([root] + greedy[:n - 1])
    if mismatch_at is not None:
        tok[mismatch_at] = (tok[mismatch_at] + 1) % SMALL.vocab
    kv = make_cache(SMALL, pkv, L, n)
    r = O.tr_verify_step(SMALL, w, kv, tok, I.tree_chain(n), L)
    want = n - 1 if mismatch_at is None else mismatch_at - 1
    assert r["accept_len"] == want
    assert r["path"] == list(range(want + 1))
    emitted = [int(tok[j]) for j in r["path"][1:]] + [r["bonus"]]
    assert emitted == greedy[:want + 1]          # output identical to plain greedy
    assert r["new_len"] == L + want + 1


def test_compacted_cache_equals_causal_cache_over_accepted_string():
    """Tree with the greedy continuation planted on a side branch: after compaction
    the cache holds exactly what a causal forward over prefix ++ root ++ accepted
    tokens would have written."""
    L = 6
    w, prefix, pkv = setup(SMALL, 9, L)
    root = 8
    g = B.greedy_decode(SMALL, w, list(prefix) + [root], 4)
    # 0 root; 1-2 wrong chain; 3,4,5 = greedy branch hanging off the root; 6 wrong leaf
    parent = np.array([-1, 0, 1, 0, 3, 4, 4])
    tok = np.array([root, (g[0] + 1) % 50, 5, g[0], g[1], g[2], (g[2] + 1) % 50])
    kv = make_cache(SMALL, pkv, L, len(tok))
    r = O.tr_verify_step(SMALL, w, kv, tok, parent, L)
    assert r["accept_len"] == 3 and r["path"] == [0, 3, 4, 5] and r["bonus"] == g[3]
    string = list(prefix) + [root] + g[:3]
    _, wkv = B.causal_forward(SMALL, w, string)
    for l in range(SMALL.n_layers):
        assert np.allclose(kv[l][0][:, :r["new_len"]], wkv[l][0], rtol=1e-9, atol=1e-11)
        assert np.allclose(kv[l][1][:, :r["new_len"]], wkv[l][1], rtol=1e-9, atol=1e-11)


# ------------------------------------------------------------------ accept alone
def brute_accept(am, tok, parent):
    """Enumerate every root-to-node path; a path is accepted when each of its draft
    tokens equals the prediction at the node before it."""
    n = len(parent)
    best, best_len = 0, 0
    for i in range(n):
        path = O.root_path(parent, i)
        if all(tok[path[j]] == am[path[j - 1]] for j in range(1, len(path))):
            if len(path) - 1 > best_len:
                best, best_len = i, len(path) - 1
    return best_len, best


@pytest.mark.parametrize("seed", range(20))
def test_accept_against_enumeration(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 40))
    parent = I.tree_random(n, rng)
    vocab = 3  # tiny vocabulary so that matches are frequent
    am, tok = rng.integers(0, vocab, n), rng.integers(0, vocab, n)
    a, best, path, bonus = O.accept_path(am, tok, parent)
    assert (a, best) == brute_accept(am, tok, parent)
    assert path == O.root_path(parent, best) and len(path) == a + 1
    assert bonus == am[best]


def test_accept_ties_and_duplicates():
    # two children of the root carry the same (correct) token: lowest index wins
    parent = np.array([-1, 0, 0, 1, 2])
    am = np.array([7, 9, 9, 0, 0])
    tok = np.array([1, 7, 7, 9, 9])
    a, best, path, bonus = O.accept_path(am, tok, parent)
    assert (a, best, path, bonus) == (2, 3, [0, 1, 3], 0)
    # a deeper accepted node on a later branch beats an earlier shallow one
    tok = np.array([1, 7, 7, 8, 9])
    assert O.accept_path(am, tok, parent)[:3] == (2, 4, [0, 2, 4])
    # a match below a rejected node does not count
    tok = np.array([1, 6, 6, 9, 9])
    assert O.accept_path(am, tok, parent)[:3] == (0, 0, [0])


def test_uniform_random_drafts_are_rarely_accepted():
    rng = np.random.default_rng(0)
    hits = 0
    for _ in range(200):
        parent = I.tree_c0()
        am, tok = rng.integers(0, 2048, 15), rng.integers(0, 2048, 15)
        hits += O.accept_path(am, tok, parent)[0] > 0
    assert hits <= 3  # 3 root children, each matching with probability 1/2048


def test_argmax_rules():
    x = np.array([[1.0, 5.0, 5.0, 2.0], [np.nan, -1.0, np.nan, -3.0], [np.nan] * 4,
                  [-np.inf, -np.inf, -np.inf, -np.inf]])
    assert list(O.greedy_argmax(x)) == [1, 1, 0, 0]


def test_kv_compact_index_map():
    L, n, H, dh = 4, 7, 2, 3
    K = np.arange(H * (L + n) * dh, dtype=float).reshape(H, L + n, dh)
    V = -K.copy()
    K0, V0 = K.copy(), V.copy()
    path = [0, 2, 5, 6]
    new_len = O.kv_compact([(K, V)], path, 3, L)
    assert new_len == L + 4
    for j, pj in enumerate(path):
        assert np.array_equal(K[:, L + j], K0[:, L + pj])
        assert np.array_equal(V[:, L + j], V0[:, L + pj])
    assert np.array_equal(K[:, :L], K0[:, :L])


# ----------------------------------------------------------------------------- grouped-query
GQA_SMALL = I.ModelShape(2, 32, 4, 8, 64, 50, "f32", n_kv_heads=2)


def expand_to_mha(shape, w):
    """The multi-head model that a grouped-query model equals: every K/V head's rows of
    Wk and Wv repeated for each query head of its group."""
    from dataclasses import replace
    H, Hkv, dh = shape.n_heads, shape.kv_heads, shape.head_dim
    g = H // Hkv
    out = dict(w)
    out["layers"] = []
    for lw in w["layers"]:
        wq, wk, wv = np.split(lw["wqkv"], [H * dh, (H + Hkv) * dh])
        rep = lambda m: np.repeat(m.reshape(Hkv, dh, -1), g, axis=0).reshape(H * dh, -1)
        out["layers"].append(dict(lw, wqkv=np.concatenate([wq, rep(wk), rep(wv)])))
    return replace(shape, n_kv_heads=0), out


@pytest.mark.parametrize("seed,L,n", [(0, 5, 9), (1, 0, 7), (2, 12, 15)])
def test_grouped_query_node_logits_equal_causal_forward_over_root_path(seed, L, n):
    w, prefix, pkv = setup(GQA_SMALL, seed, L)
    rng = np.random.default_rng(300 + seed)
    parent = I.tree_c0() if n == 15 else I.tree_random(n, rng)
    tok = rng.integers(0, GQA_SMALL.vocab, size=n)
    kv = []
    for l in range(GQA_SMALL.n_layers):
        K = np.full((GQA_SMALL.kv_heads, L + n, GQA_SMALL.head_dim), np.nan)
        V = np.full_like(K, np.nan)
        if L:
            K[:, :L], V[:, :L] = pkv[l]
        kv.append((K, V))
    logits = O.decoder_tree_forward(GQA_SMALL, w, kv, tok, parent, L)
    for i in range(n):
        string = list(prefix) + [int(tok[j]) for j in O.root_path(parent, i)]
        want, _ = B.causal_forward(GQA_SMALL, w, string)
        assert np.allclose(logits[i], want[-1], rtol=1e-9, atol=1e-11), i


def test_grouped_query_equals_multi_head_with_repeated_kv_weights():
    """Closed relation: sharing a K/V head between g query heads is the multi-head model
    whose Wk, Wv rows are repeated g times (checked inside the oracle, both ways round)."""
    w, prefix, pkv = setup(GQA_SMALL, 4, 6)
    mha_shape, mha_w = expand_to_mha(GQA_SMALL, w)
    rng = np.random.default_rng(9)
    n, L = 11, 6
    parent = I.tree_random(n, rng)
    tok = rng.integers(0, GQA_SMALL.vocab, size=n)
    def cache(shape, heads_kv):
        out = []
        for l in range(shape.n_layers):
            K = np.zeros((heads_kv, L + n, shape.head_dim)); V = np.zeros_like(K)
            k, v = pkv[l]
            g = heads_kv // k.shape[0]
            K[:, :L], V[:, :L] = np.repeat(k, g, axis=0), np.repeat(v, g, axis=0)
            out.append((K, V))
        return out
    a = O.decoder_tree_forward(GQA_SMALL, w, cache(GQA_SMALL, 2), tok, parent, L)
    b = O.decoder_tree_forward(mha_shape, mha_w, cache(mha_shape, 4), tok, parent, L)
    assert np.allclose(a, b, rtol=1e-11, atol=1e-12)


def test_grouped_query_attention_reads_the_group_head():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((5, 6, 4)); k = rng.standard_normal((2, 9, 4)); v = rng.standard_normal((2, 9, 4))
    parent = I.tree_chain(5)
    got = O.tree_attention(q, k, v, parent, 4)
    want = O.tree_attention(q, np.repeat(k, 3, axis=0), np.repeat(v, 3, axis=0), parent, 4)
    assert np.allclose(got, want, rtol=0, atol=1e-14)
    assert not np.allclose(got[:, 0], O.tree_attention(q, k[::-1].repeat(3, axis=0), v[::-1].repeat(3, axis=0), parent, 4)[:, 0])


# ---- the storage hooks (a model of a 16-bit mode's storage; off by default)
def test_storage_hooks_default_off_and_identity_changes_nothing():
    w, prefix, pkv = setup(SMALL, 5, 9)
    rng = np.random.default_rng(5)
    tree = I.tree_random(11, rng)
    tok = rng.integers(0, SMALL.vocab, size=11)
    plain = O.decoder_tree_forward(SMALL, w, make_cache(SMALL, pkv, 9, 11), tok, tree, 9)
    ident = {k: (lambda a: a) for k in ("h", "q", "kv", "p", "attn", "act")}
    kv = make_cache(SMALL, pkv, 9, 11)
    same = O.decoder_tree_forward(SMALL, w, kv, tok, tree, 9, storage=ident)
    # the hooked attention divides after the product with V instead of before: rounding order only
    assert np.abs(same - plain).max() <= 1e-12 * np.abs(plain).max()
    assert O.decoder_tree_forward(SMALL, w, make_cache(SMALL, pkv, 9, 11), tok, tree, 9, storage={}) is not None
    assert np.array_equal(O.decoder_tree_forward(SMALL, w, make_cache(SMALL, pkv, 9, 11), tok, tree, 9,
                                                 storage=None), plain)


def test_storage_hooks_see_the_tensors_they_name():
    """Every hook is applied to the tensor its name says, once per layer and use: told apart
    by shape (h twice per layer, K and V once each, the attention weights one vector per
    node and head over prefix + root path)."""
    shape = I.ModelShape(2, 32, 2, 16, 64, 50, "f32")
    w, prefix, pkv = setup(shape, 6, 7)
    tree = I.tree_chain(5)
    tok = np.arange(5)
    seen = {}

    def rec(name):
        def f(a):
            seen.setdefault(name, []).append(np.asarray(a).shape)
            return a
        return f
    O.decoder_tree_forward(shape, w, make_cache(shape, pkv, 7, 5), tok, tree, 7,
                           storage={k: rec(k) for k in ("h", "q", "kv", "p", "attn", "act")})
    n, H, dh, d, F, L = 5, 2, 16, 32, 64, 7
    assert seen["h"] == [(n, d)] * 4
    assert seen["q"] == [(n, H, dh)] * 2 and seen["kv"] == [(n, H, dh)] * 4
    assert seen["attn"] == [(n, H, dh)] * 2 and seen["act"] == [(n, F)] * 2
    # chain tree: node i sees the prefix and nodes 0..i
    assert seen["p"] == [(L + i + 1,) for i in range(n) for _ in range(H)] * 2


def test_storage_rounding_moves_the_result_by_about_the_rounding_step():
    """Rounding the stored tensors to bf16 changes a shallow model's logits by a few units of
    the bf16 step (2^-8 relative), not more and not nothing."""
    w, prefix, pkv = setup(SMALL, 7, 9, std=0.15)
    rng = np.random.default_rng(7)
    tree = I.tree_random(12, rng)
    tok = rng.integers(0, SMALL.vocab, size=12)
    plain = O.decoder_tree_forward(SMALL, w, make_cache(SMALL, pkv, 9, 12), tok, tree, 9)
    rnd = lambda a: I.bf16_round(np.asarray(a, np.float32)).astype(np.float64)
    got = O.decoder_tree_forward(SMALL, w, make_cache(SMALL, pkv, 9, 12), tok, tree, 9,
                                 storage={k: rnd for k in ("h", "q", "kv", "p", "attn", "act")})
    dev = np.abs(got - plain).max() / np.abs(plain).max()
    assert 1e-4 < dev < 3e-2
