"""Pins for the oracle's decoding loop: the committed tokens equal plain greedy decoding
with a separately written autoregressive model (section "Speculative Decoding": the
output is unchanged), the noise generator reproduces SplitMix64's published outputs,
prompt lookup agrees with a string search, the refill agrees with the Jacobi update on a
chain (section "Jacobi Decoding") and with a walk over child ranks on a tree."""
import numpy as np
import pytest

import brute_force_lm as B
from oracle import tr_loop as LP
from oracle import tr_oracle as O
from paper_2406_17404_amd import inputs as I
from test_oracle_step import SMALL, setup


def template(n_jacobi, r, rng):
    """Random tree of n_jacobi nodes (root included) plus a retrieval chain of r."""
    parent = list(I.tree_random(n_jacobi, rng))
    for j in range(r):
        parent.append(0 if j == 0 else len(parent) - 1)
    return np.asarray(parent, np.int32)


# ----------------------------------------------------------------------------- noise
def test_splitmix64_published_outputs():
    # first outputs of the reference SplitMix64 for seed 1234567 (Vigna's splitmix64.c)
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423,
            4593380528125082431, 16408922859458223821]
    assert [LP.splitmix64_output(1234567, k) for k in range(1, 6)] == want


def test_ahead_noise_draws_only_from_context_and_is_roughly_uniform():
    ctx = [7, 7, 9, 11, 13]
    draws = [LP.ahead_noise(ctx, 5, s, v) for s in range(200) for v in range(1, 21)]
    assert set(draws) <= set(ctx)
    share7 = draws.count(7) / len(draws)
    assert abs(share7 - 0.4) < 0.05          # two of five positions hold token 7
    assert draws != [LP.ahead_noise(ctx, 6, s, v) for s in range(200) for v in range(1, 21)]


# ----------------------------------------------------------------------------- lookup
def test_prompt_lookup_worked_cases():
    assert LP.prompt_lookup([1, 2, 3, 4, 1, 2, 3], 3, 2) == [4, 1]
    assert LP.prompt_lookup([5, 1, 9, 5, 1, 7, 5, 1], 2, 2) == [7, 5]     # most recent wins
    assert LP.prompt_lookup([5, 1, 9, 5, 1, 7, 5, 1], 2, 5) == [7, 5, 1]  # runs into the end
    assert LP.prompt_lookup([1, 2, 3], 3, 4) == []                        # nothing repeats
    assert LP.prompt_lookup([4, 4, 4], 3, 2) == [4]                       # overlap allowed
    assert LP.prompt_lookup([9, 8, 3, 7, 3], 3, 3) == [7, 3]              # falls back to 1-gram
    assert LP.prompt_lookup([3], 3, 3) == []
    assert LP.prompt_lookup([1, 2, 1, 2], 2, 0) == []


def lookup_by_string_search(ctx, max_ngram, r):
    s = "".join(chr(65 + t) for t in ctx)
    for n in range(min(max_ngram, len(s) - 1), 0, -1):
        i = s.rfind(s[len(s) - n:], 0, len(s) - 1)   # last match that ends before the end
        if i >= 0:
            return [ord(c) - 65 for c in s[i + n:i + n + r]]
    return []


@pytest.mark.parametrize("seed", range(6))
def test_prompt_lookup_equals_string_search(seed):
    rng = np.random.default_rng(seed)
    for _ in range(300):
        ctx = list(rng.integers(0, 3, size=rng.integers(1, 24)))
        ng, r = int(rng.integers(1, 5)), int(rng.integers(1, 6))
        assert LP.prompt_lookup(ctx, ng, r) == lookup_by_string_search(ctx, ng, r)


# ----------------------------------------------------------------------------- refill
def test_first_tree_is_all_noise_plus_lookup():
    rng = np.random.default_rng(0)
    parent = template(9, 3, rng)
    ctx = [4, 5, 6, 4, 5]
    tok = LP.fill_tree(parent, 3, ctx, 3, 11, 0)
    assert tok[0] == 5
    assert list(tok[-3:]) == [6, 4, 5]
    assert list(tok[1:9]) == [LP.ahead_noise(ctx, 11, 0, v) for v in range(1, 9)]


@pytest.mark.parametrize("m,a", [(6, 0), (6, 2), (6, 5), (1, 0)])
def test_refill_on_a_chain_is_the_jacobi_update(m, a):
    """Chain root -> y1 .. ym with predictions p0 .. pm; y1..ya accepted.  The next
    draft is pa (new root), then p(a+1) .. pm, then noise (section "Jacobi Decoding":
    every position is replaced by the prediction made one position earlier)."""
    parent = np.arange(-1, m, dtype=np.int32)
    p = np.arange(100, 101 + m, dtype=np.int32)
    ctx = [1, 2, 3, int(p[a])]
    tok = LP.fill_tree(parent, 0, ctx, 3, 3, 4, argmax=p, best=a)
    want = [int(p[a])] + [int(x) for x in p[a + 1:]]
    want += [LP.ahead_noise(ctx, 3, 4, v) for v in range(len(want), m + 1)]
    assert list(tok) == want


@pytest.mark.parametrize("seed", range(8))
def test_refill_on_a_tree_follows_child_ranks(seed):
    rng = np.random.default_rng(seed)
    r = int(rng.integers(0, 4))
    parent = template(int(rng.integers(2, 20)), r, rng)
    n = len(parent)
    argmax = rng.integers(1000, 2000, size=n).astype(np.int32)
    best = int(rng.integers(0, n))
    ctx = [1000 + int(t) for t in rng.permutation(40)[:12]] + [int(argmax[best])]  # no repeats: lookup finds nothing
    tok = LP.fill_tree(parent, r, ctx, 3, 9, 2, argmax=argmax, best=best)
    kids = lambda u: [i for i in range(n) if parent[i] == u]
    for v in range(n):
        ranks = []                      # child ranks along root -> v
        x = v
        while x != 0:
            ranks.append(kids(parent[x]).index(x))
            x = parent[x]
        u = best                        # walk the same ranks down from the accepted node
        for k in reversed(ranks):
            u = kids(u)[k] if u >= 0 and k < len(kids(u)) else -1
        want = argmax[u] if u >= 0 else LP.ahead_noise(ctx, 9, 2, v)
        assert tok[v] == want, v


def test_lookup_overrides_the_retrieval_chain_only():
    parent = template(5, 2, np.random.default_rng(1))
    n = len(parent)
    argmax = np.arange(50, 50 + n, dtype=np.int32)
    ctx = [8, 9, 3, 8, 9]
    tok = LP.fill_tree(parent, 2, ctx, 2, 0, 1, argmax=argmax, best=0)
    assert list(tok[-2:]) == [3, 8]
    base = LP.fill_tree(parent, 0, ctx, 2, 0, 1, argmax=argmax, best=0)
    assert list(tok[:-2]) == list(base[:-2])


# ----------------------------------------------------------------------------- loop
@pytest.mark.parametrize("seed,n_jacobi,r,plen,max_new", [(0, 8, 3, 5, 14), (1, 1, 0, 1, 6), (2, 12, 0, 9, 12),
                                                            (3, 5, 4, 3, 16), (4, 15, 2, 12, 10)])
def test_generate_equals_autoregressive_greedy(seed, n_jacobi, r, plen, max_new):
    w, _, _ = setup(SMALL, seed, 0)
    rng = np.random.default_rng(50 + seed)
    prompt = rng.integers(0, SMALL.vocab, size=plen)
    parent = template(n_jacobi, r, rng)
    res = LP.generate(SMALL, w, prompt, parent, r, 3, max_new, -1, seed)
    assert res["tokens"] == B.greedy_decode(SMALL, w, prompt, max_new)
    assert len(res["accept_hist"]) == res["n_steps"] <= max_new
    assert sum(a + 1 for a in res["accept_hist"]) >= max_new
    assert sum(a + 1 for a in res["accept_hist"][:-1]) < max_new


def test_generate_stops_at_eos_and_keeps_it():
    w, _, _ = setup(SMALL, 0, 0)
    prompt = [3, 1, 4, 1, 5]
    parent = template(8, 3, np.random.default_rng(0))
    full = B.greedy_decode(SMALL, w, prompt, 12)
    eos = full[6]
    cut = full.index(eos) + 1
    res = LP.generate(SMALL, w, prompt, parent, 3, 3, 12, eos, 0)
    assert res["tokens"] == full[:cut]


def test_drafts_get_accepted_when_the_continuation_repeats():
    """A context whose greedy continuation loops lets both the lookup and the model's
    own drafts be accepted: fewer forwards than tokens."""
    w, _, _ = setup(SMALL, 0, 0)
    prompt = [3, 1, 4, 1, 5]
    parent = template(8, 4, np.random.default_rng(0))
    res = LP.generate(SMALL, w, prompt, parent, 4, 3, 40, -1, 0)
    assert res["tokens"] == B.greedy_decode(SMALL, w, prompt, 40)
    print("accept history", res["accept_hist"])
    assert res["n_steps"] < 40 and max(res["accept_hist"]) >= 2


def test_generate_rejects_bad_templates():
    w, _, _ = setup(SMALL, 0, 0)
    with pytest.raises(ValueError):
        LP.generate(SMALL, w, [1, 2], np.array([-1, 0, 0], np.int32), 2, 3, 4, -1, 0)  # last 2 nodes are no chain
    with pytest.raises(ValueError):
        LP.generate(SMALL, w, [1, 2], np.array([-1, 1, 0], np.int32), 0, 3, 4, -1, 0)


def test_generate_with_grouped_query_attention_equals_autoregressive_greedy():
    from test_oracle_step import GQA_SMALL
    w, _, _ = setup(GQA_SMALL, 5, 0)
    prompt = [7, 3, 9, 3, 1, 4]
    parent = template(10, 3, np.random.default_rng(5))
    res = LP.generate(GQA_SMALL, w, prompt, parent, 3, 3, 12, -1, 5)
    assert res["tokens"] == B.greedy_decode(GQA_SMALL, w, prompt, 12)
